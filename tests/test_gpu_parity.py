"""GPU parity: the HIP library through its C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
import vq_synth as s
from cases import SMALL, MULTI, small_layer, multi_layers

pytestmark = pytest.mark.gpu

TOL = 1e-2        # max |y - y_ref| <= TOL * RMS(y_ref): the stated bar for GEMV and GEMM


def _check_matmul(y_gpu, y_ref, what):
    y = y_gpu.float().cpu().numpy().astype(np.float64)
    rms = np.sqrt((y_ref ** 2).mean())
    err = np.abs(y - y_ref).max()
    assert np.isfinite(y).all(), what
    assert err <= TOL * rms, "%s: max abs err %.3e > %.0e * rms %.3e" % (what, err, TOL, rms)


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("pad", [8, 16, 24])
def test_dequant_leaves_the_padding_of_aligned_rows_alone(gpu_lib, name, pad):
    """Leading dimensions that keep every row 16-byte aligned (the layouts the kernels with 16-byte stores take): the
    logical columns bit-exact, the columns [in_features, ldw) still holding the caller's sentinel."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    ldw = (L.in_features + 7) // 8 * 8 + pad
    W = torch.full((L.out_features, ldw), -3.5, dtype=torch.float16, device="cuda")
    rc = gpu_lib.vq_dequant(dl.desc, W.data_ptr(), ldw, torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    got = W.cpu().numpy()
    want = oracle.dequant(L, L.in_features)
    assert np.array_equal(got[:, :L.in_features].view(np.uint16), want.view(np.uint16)), name
    assert (got[:, L.in_features:] == np.float16(-3.5)).all(), name


@pytest.mark.parametrize("name", list(SMALL))
def test_dequant_bit_exact_small(gpu_lib, name):
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    for ldw in (L.in_features, L.in_features + 11):
        W = gpu_lib.dequant(dl, ldw)
        torch.cuda.synchronize()
        want = oracle.dequant(L, ldw)
        assert np.array_equal(W.cpu().numpy().view(np.uint16), want.view(np.uint16)), name


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("batch", [1, 2, 3, 4, 8, 16])
@pytest.mark.parametrize("kernel", ["auto", "m", "d"])
def test_gemv_small(gpu_lib, monkeypatch, name, batch, kernel):
    """Every batch through the default dispatch, then with the matrix-core kernel and the dot-product kernels forced
    (layers they do not take fall through to the generic kernel)."""
    import torch
    if kernel != "auto":
        monkeypatch.setenv("VQ_SWITCHES", "gemv=" + kernel)
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(300, L, batch)
    y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    _check_matmul(y, oracle.gemv(L, x), "%s batch %d" % (name, batch))


# (the restore-then-multiply route exists for layers whose in_features is a multiple of 256: only those get its cases)
GEMM_CASES = [(name, ws) for name in SMALL for ws in (None, "fast", "fast, 256 x 256 tiles")
              if ws is None or SMALL[name]["in_features"] % 256 == 0]


@pytest.mark.parametrize("name,workspace", GEMM_CASES)
@pytest.mark.parametrize("tokens", [1, 37, 130, 300])
def test_gemm_small(gpu_lib, monkeypatch, name, tokens, workspace):
    """Without a workspace (weights restored on the fly) and with the one that lets vq_gemm restore W once (that
    route forced: by itself the library keeps small token counts on the on-the-fly kernel where it has one), the dense
    product by the kernel with producer waves and by the four-wave kernel with 256 x 256 tiles."""
    import torch
    if workspace is not None:
        monkeypatch.setenv("VQ_SWITCHES", "gemm=w,dense=" + ("1" if "256" in workspace else "0"))      # the dense product's two kernels
        workspace = "fast"
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    if workspace == "fast":
        assert gpu_lib.vq_gemm_fast_workspace_bytes(dl.desc, tokens) > 0
    x = s.make_activations(300, L, tokens)
    ldx = (L.in_features + 7) // 8 * 8
    X = torch.zeros((tokens, ldx), dtype=torch.float16, device="cuda")
    X[:, : L.in_features] = torch.from_numpy(x).cuda()
    if ldx > L.in_features:
        X[:, L.in_features:] = float("nan")           # padding of the caller's buffer must never be read into the sum
    Y = gpu_lib.gemm(dl, X, workspace=workspace)
    torch.cuda.synchronize()
    _check_matmul(Y, oracle.gemm(L, x), "%s tokens %d workspace %s" % (name, tokens, workspace))


V6_GEMM = ["v6_gemm_plain", "v6_gemm_res8", "v6_gemm_res12", "single_row", "v6_exact_fit", "v6_gemm_outlier32", "v6_gemm_outlier48",
           "v6_gemm_outlier16_res12"]


@pytest.mark.parametrize("name", V6_GEMM)
@pytest.mark.parametrize("tokens", [1, 37, 130, 300, 700])
def test_gemm_v6_on_the_fly(gpu_lib, monkeypatch, name, tokens):
    """The kernel that restores v = 6 layers from tables in LDS, forced for every token count (by itself vq_gemm takes it
    without a workspace from 65 tokens on), with NaN in the padding of X and a sentinel in the padding of Y."""
    import torch
    monkeypatch.setenv("VQ_SWITCHES", "gemm=6")
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(300, L, tokens)
    X = torch.full((tokens, L.in_features + 8), float("nan"), dtype=torch.float16, device="cuda")
    X[:, : L.in_features] = torch.from_numpy(x).cuda()
    Y = torch.full((tokens, L.out_features + 3), 7.0, dtype=torch.float16, device="cuda")
    gpu_lib.gemm(dl, X, out=Y)
    torch.cuda.synchronize()
    _check_matmul(Y[:, : L.out_features], oracle.gemm(L, x), "%s tokens %d on the fly" % (name, tokens))
    assert (Y[:, L.out_features:] == 7.0).all()


@pytest.mark.parametrize("kernel", ["auto", "m", "d"])
@pytest.mark.parametrize("batch", [1, 4, 5, 16])
@pytest.mark.parametrize("name,pad_x,pad_y", [("v6_res256_outlier", 10, 6), ("v6_k4096_res4096", 2, 1), ("v6_passes", 6, 3)])
def test_gemv_strided_buffers_and_untouched_padding(gpu_lib, monkeypatch, name, pad_x, pad_y, batch, kernel):
    """Row strides larger than the rows, NaN in the caller's padding (it must never reach a sum), sentinel values
    in the output padding (they must survive); odd output strides take the kernels' narrow store paths."""
    import torch
    if kernel != "auto":
        monkeypatch.setenv("VQ_SWITCHES", "gemv=" + kernel)
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(300, L, batch)
    xb = torch.full((batch, L.in_features + pad_x), float("nan"), dtype=torch.float16, device="cuda")
    xb[:, : L.in_features] = torch.from_numpy(x).cuda()
    yb = torch.full((batch, L.out_features + pad_y), 7.0, dtype=torch.float16, device="cuda")
    gpu_lib.gemv(dl, xb, out=yb)
    torch.cuda.synchronize()
    _check_matmul(yb[:, : L.out_features], oracle.gemv(L, x), "strided %s batch %d" % (name, batch))
    assert (yb[:, L.out_features:] == 7.0).all()


def test_unit_activation_reads_back_a_column(gpu_lib):
    import torch
    L = small_layer("v6_res256_outlier")
    dl = gpu_lib.DeviceLayer(L)
    W = oracle.dequant(L).astype(np.float64)
    cols = [0, 5, 23, 24, 29, 30, 1205, 1206]
    for c0 in range(0, len(cols), 4):
        x = np.zeros((4, L.in_features), dtype=np.float16)
        for t, c in enumerate(cols[c0:c0 + 4]):
            x[t, c] = 1.0
        y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda()).float().cpu().numpy()
        for t, c in enumerate(cols[c0:c0 + 4]):
            assert np.allclose(y[t], W[:, c], rtol=2e-3, atol=1e-7)


@pytest.mark.parametrize("batch", [1, 4, 16])
def test_runs_are_deterministic(gpu_lib, batch):
    import torch
    L = small_layer("v6_k4096_res4096")
    dl = gpu_lib.DeviceLayer(L)
    x = torch.from_numpy(s.make_activations(300, L, batch)).cuda()
    a = gpu_lib.gemv(dl, x).clone()
    for _ in range(3):
        assert torch.equal(gpu_lib.gemv(dl, x), a)


def test_non_default_stream(gpu_lib):
    import torch
    L = small_layer("v6_k4096")
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(300, L, 1)
    xs = torch.from_numpy(x).cuda()
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        y = gpu_lib.gemv(dl, xs)
    st.synchronize()
    _check_matmul(y, oracle.gemv(L, x), "side stream")


FUSED_SETS = ("qkv_v6", "gate_up_res12", "res8_outlier_pair", "many_rows", "eight_layers")
DOWN_FUSED_SETS = ("down_qkv", "down_gate_up_res12_outlier", "down_res8_many_streams")      # orientation 1: the same body for every batch


@pytest.mark.parametrize("name", list(MULTI))
@pytest.mark.parametrize("batch", [1, 3, 16])
def test_gemv_multi(gpu_lib, monkeypatch, name, batch):
    """Several layers on the same activations in one call: each output against the oracle's product for that layer,
    for more than one row bit-identical to the matrix-core kernel on the layer alone, and padding between output rows
    left alone."""
    import torch
    layers = multi_layers(name)
    dls = [gpu_lib.DeviceLayer(L) for L in layers]
    x_np = s.make_activations(400, layers[0], batch)
    x = torch.from_numpy(x_np).cuda()
    pad = 3
    outs = [torch.full((batch, L.out_features + pad), -7.0, dtype=torch.float16, device="cuda") for L in layers]
    ys = gpu_lib.gemv_multi(dls, x, outs=[o[:, :L.out_features] for o, L in zip(outs, layers)])
    torch.cuda.synchronize()
    monkeypatch.setenv("VQ_SWITCHES", "gemv=m")
    for L, dl, y, o in zip(layers, dls, ys, outs):
        _check_matmul(y, oracle.gemv(L, x_np), "%s / %s batch %d" % (name, L.name, batch))
        assert (o[:, L.out_features:] == -7.0).all()
        alone = gpu_lib.gemv(dl, x)
        torch.cuda.synchronize()
        if (name in FUSED_SETS and batch > 1) or name in DOWN_FUSED_SETS:       # one row runs the dot-product body, whose split (and so its summation
            assert torch.equal(alone, y), L.name   # order) depends on the rows per workgroup; the others go one by one


@pytest.mark.parametrize("name", FUSED_SETS)
def test_gemv_multi_single_row_with_the_matrix_core_body(gpu_lib, monkeypatch, name):
    import torch
    monkeypatch.setenv("VQ_SWITCHES", "gemv=m")
    layers = multi_layers(name)
    dls = [gpu_lib.DeviceLayer(L) for L in layers]
    x_np = s.make_activations(400, layers[0], 1)
    ys = gpu_lib.gemv_multi(dls, torch.from_numpy(x_np).cuda())
    torch.cuda.synchronize()
    for L, y in zip(layers, ys):
        _check_matmul(y, oracle.gemv(L, x_np), "%s / %s" % (name, L.name))


def test_gemv_multi_one_by_one_matches_fused(gpu_lib, monkeypatch):
    import torch
    layers = multi_layers("qkv_v6")
    dls = [gpu_lib.DeviceLayer(L) for L in layers]
    x = torch.from_numpy(s.make_activations(400, layers[0], 4)).cuda()
    fused = [y.clone() for y in gpu_lib.gemv_multi(dls, x)]
    monkeypatch.setenv("VQ_SWITCHES", "multi=0,gemv=m")
    apart = gpu_lib.gemv_multi(dls, x)
    torch.cuda.synchronize()
    for a, b in zip(fused, apart):
        assert torch.equal(a, b)


GROUPED_FAST = [n for n, kw in SMALL.items() if kw.get("group_vectors", 0) % 8 == 0 and kw.get("group_vectors", 0) > 0 and kw["v"] == 6]


@pytest.mark.parametrize("name", GROUPED_FAST)
@pytest.mark.parametrize("batch", [1, 4, 16])
def test_gemv_groups_with_workspace(gpu_lib, monkeypatch, name, batch):
    """Layers with codebook groups when the caller lends a workspace: one group per workgroup, then the sum over groups.
    Against the oracle, and against the route without a workspace (same per-group sums, added in the same order)."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    need = gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch)
    if L.in_features % 2:
        assert need == 0                # not a layer of the fast kernels: no workspace route
        return
    assert need >= L.n_groups * batch * L.out_features * 4
    x_np = s.make_activations(300, L, batch)
    x = torch.from_numpy(x_np).cuda()
    ws = torch.full((need + 256,), 0xFF, dtype=torch.uint8, device="cuda")       # NaN patterns: nothing may be read before it is written
    y = gpu_lib.gemv(dl, x, workspace=ws[:need])
    torch.cuda.synchronize()
    _check_matmul(y, oracle.gemv(L, x_np), "%s batch %d with workspace" % (name, batch))
    assert (ws[need:] == 0xFF).all()
    small = gpu_lib.gemv(dl, x, workspace=ws[:need - 256])                         # too small: the plain route
    plain = gpu_lib.gemv(dl, x)
    torch.cuda.synchronize()
    assert torch.equal(small, plain)
    _check_matmul(plain, oracle.gemv(L, x_np), "%s batch %d" % (name, batch))


LDS_SLOTS = ["lds_v12_groups_res_outlier", "lds_v12_groups_perm", "lds_v4_k256_groups", "down_lds_v12_groups_outlier", "down_lds_v12_odd_groups"]


@pytest.mark.parametrize("name", LDS_SLOTS)
@pytest.mark.parametrize("batch", [1, 3, 4, 7, 16])
def test_gemv_lds_table_slots_with_workspace(gpu_lib, name, batch):
    """The layers of the LDS-table pass kernel with two codebook groups or more when the caller lends a workspace: a group per
    workgroup (the first group's also take the outlier columns), then the sum over the groups.  Workspace filled with NaN
    patterns beforehand, guarded behind; too small a workspace is the plain route."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    need = gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch)
    assert need >= L.n_groups * batch * L.out_features * 4
    x_np = s.make_activations(300, L, batch)
    x = torch.from_numpy(x_np).cuda()
    ws = torch.full((need + 256,), 0xFF, dtype=torch.uint8, device="cuda")
    y = gpu_lib.gemv(dl, x, workspace=ws[:need])
    torch.cuda.synchronize()
    _check_matmul(y, oracle.gemv(L, x_np), "%s batch %d with workspace" % (name, batch))
    assert (ws[need:] == 0xFF).all()
    small = gpu_lib.gemv(dl, x, workspace=ws[:need - 256])
    plain = gpu_lib.gemv(dl, x)
    torch.cuda.synchronize()
    assert torch.equal(small, plain)


PERMUTED = [n for n in SMALL if n.startswith("perm_")]


@pytest.mark.parametrize("name", PERMUTED)
@pytest.mark.parametrize("batch", [1, 2, 5, 16])
def test_gemv_permuted_columns_with_workspace(gpu_lib, name, batch):
    """Sec. 3.2.3: stored column order a permutation of the layer's.  With a workspace the activations are gathered into it
    first and the layer's usual kernels run; one row of a short-row v = 6 layer is gathered inside the kernel instead and
    asks for no workspace.  Also through the library's own static workspace."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    need = gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch)
    in_kernel = batch == 1 and L.v == 6 and L.orientation == 0 and not L.group_vectors and L.in_features % 2 == 0 and L.in_features < 16384
    assert (need == 0) == in_kernel, (name, batch, need)
    x_np = s.make_activations(300, L, batch)
    x = torch.full((batch, L.in_features + 4), float("nan"), dtype=torch.float16, device="cuda")
    x[:, : L.in_features] = torch.from_numpy(x_np).cuda()
    ws = torch.full((need + 256,), 0xFF, dtype=torch.uint8, device="cuda")
    y = gpu_lib.gemv(dl, x, workspace=ws[:need] if need else ws[:256])
    torch.cuda.synchronize()
    ref = oracle.gemv(L, x_np)
    _check_matmul(y, ref, "%s batch %d with workspace" % (name, batch))
    assert (ws[need:] == 0xFF).all()
    y2 = torch.empty_like(y)
    rc = gpu_lib.vq_gemv_static_workspace(dl.desc, x.data_ptr(), x.stride(0), batch, y2.data_ptr(), y2.stride(0), torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    plain = gpu_lib.gemv(dl, x)                               # no workspace: gathered in the kernel, or the generic kernels
    torch.cuda.synchronize()
    _check_matmul(plain, ref, "%s batch %d" % (name, batch))


@pytest.mark.parametrize("name", PERMUTED)
def test_dequant_permuted_columns_by_the_scattering_kernels(gpu_lib, monkeypatch, name):
    """The generic kernels, which store every value at its column themselves (rows too long for LDS take them)."""
    import torch
    monkeypatch.setenv("VQ_SWITCHES", "dequant=g")
    L = small_layer(name)
    W = gpu_lib.dequant(gpu_lib.DeviceLayer(L), L.in_features + 5)
    torch.cuda.synchronize()
    assert np.array_equal(W.cpu().numpy().view(np.uint16), oracle.dequant(L, L.in_features + 5).view(np.uint16)), name


@pytest.mark.parametrize("name", ["lds_v12_two_tables", "lds_v12_groups_res_outlier", "down_lds_v12_two_tables", "down_lds_v12_odd_groups"])
def test_dequant_two_tables_beyond_lds_in_two_passes(gpu_lib, monkeypatch, name):
    """Two tables that do not fit LDS together: by default the residual entries come from memory; dequant=s is the scheme
    with two passes and a read-back of the main centroids.  Both bit for bit."""
    import torch
    L = small_layer(name)
    want = oracle.dequant(L, L.in_features + 6).view(np.uint16)
    for switch in (None, "dequant=s"):
        if switch:
            monkeypatch.setenv("VQ_SWITCHES", switch)
        W = gpu_lib.dequant(gpu_lib.DeviceLayer(L), L.in_features + 6)
        torch.cuda.synchronize()
        assert np.array_equal(W.cpu().numpy().view(np.uint16), want), (name, switch)


def test_permuted_unit_activation_reads_back_the_layers_column(gpu_lib):
    """x = e_t returns column t of the LAYER (not of the stored order), outlier columns included."""
    import torch
    L = small_layer("perm_v6_res8_outlier")
    dl = gpu_lib.DeviceLayer(L)
    W = oracle.dequant(L).astype(np.float64)
    cols = [int(L.col_perm[0]), int(L.col_perm[23]), int(L.col_perm[24]), int(L.col_perm[1207]), 0, 1207]
    for ws in (None, "fast"):
        for t in cols:
            x = np.zeros((2, L.in_features), dtype=np.float16)
            x[0, t] = 1.0
            x[1, t] = -2.0
            y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda(), workspace=ws).float().cpu().numpy()
            assert np.allclose(y[0], W[:, t], rtol=2e-3, atol=1e-7) and np.allclose(y[1], -2.0 * W[:, t], rtol=2e-3, atol=1e-7)


def test_permutation_entries_outside_the_row_are_ignored(gpu_lib):
    """The library does not check that col_perm is a permutation: an entry outside [0, in_features) must neither be
    read nor written through.  Such a stored column then contributes nothing, which is the same layer with a zero
    activation there."""
    import torch
    L = small_layer("perm_v6_res8_outlier")
    x_np = s.make_activations(300, L, 3)
    bad = [5, 30, 700]                                  # stored columns whose entries go out of range
    ref_x = x_np.copy()
    ref_x[:, L.col_perm[bad]] = 0
    ref = oracle.gemv(L, ref_x)
    want_W = oracle.dequant(L)
    M = small_layer("perm_v6_res8_outlier")
    M.col_perm = L.col_perm.copy()
    M.col_perm[bad] = [-1, L.in_features, 2 ** 31 - 1]
    dl = gpu_lib.DeviceLayer(M)
    x = torch.from_numpy(x_np).cuda()
    for ws in (None, "fast"):
        for batch in (1, 3):
            y = gpu_lib.gemv(dl, x[:batch], workspace=ws)
            torch.cuda.synchronize()
            _check_matmul(y, ref[:batch], "out-of-range entries, batch %d, workspace %s" % (batch, ws))
    W = torch.full((M.out_features, M.in_features + 8), -3.5, dtype=torch.float16, device="cuda")
    assert gpu_lib.vq_dequant(dl.desc, W.data_ptr(), W.stride(0), torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    got = W.cpu().numpy()
    keep = np.setdiff1d(np.arange(M.in_features), L.col_perm[bad])
    assert np.array_equal(got[:, keep].view(np.uint16), want_W[:, keep].view(np.uint16))
    assert (got[:, M.in_features:] == np.float16(-3.5)).all()


def test_gemv_multi_with_permuted_layers(gpu_lib):
    """Layers with a column permutation of their own run one after the other: same results as single calls."""
    import torch
    a, b = small_layer("perm_v6_k4096"), small_layer("v6_k4096")
    dls = [gpu_lib.DeviceLayer(a), gpu_lib.DeviceLayer(b)]
    for batch in (1, 4):
        x_np = s.make_activations(300, a, batch)
        ys = gpu_lib.gemv_multi(dls, torch.from_numpy(x_np).cuda())
        torch.cuda.synchronize()
        for L, y in zip((a, b), ys):
            _check_matmul(y, oracle.gemv(L, x_np), "multi with a permuted layer, batch %d" % batch)


def test_gemv_workspace_is_not_asked_for_without_groups(gpu_lib):
    for name in ("v6_k4096", "v8_k65536", "grp_v6_unaligned", "grp_odd"):
        dl = gpu_lib.DeviceLayer(small_layer(name))
        assert gpu_lib.vq_gemv_workspace_bytes(dl.desc, 4) == 0, name


NATIVE_PLAIN = [n for n, kw in SMALL.items() if n.startswith("down_fast") and not kw.get("group_vectors") and kw.get("n_outlier_cols", 0) % 2 == 0]


@pytest.mark.parametrize("name", NATIVE_PLAIN)
@pytest.mark.parametrize("batch", [2, 3, 6, 16])
def test_gemv_native_orientation_column_parts_with_workspace(gpu_lib, name, batch):
    """Vectors down the output dimension, one codebook group, two rows or more: with a workspace the matrix-core kernel
    cuts the columns into parts that run side by side and a second kernel adds them up."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    need = gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch)
    if L.in_features - L.n_outlier_cols < 2 * 8 * 32 or L.out_features > 16 * 6 * 128:
        assert need == 0, name          # a part needs a window of 32 columns per wave; more blocks of 16 streams than half the chip need no parts
        return
    assert need >= 2 * batch * L.out_features * 4, name
    x_np = s.make_activations(300, L, batch)
    x = torch.from_numpy(x_np).cuda()
    ws = torch.full((need + 256,), 0xFF, dtype=torch.uint8, device="cuda")
    y = gpu_lib.gemv(dl, x, workspace=ws[:need])
    torch.cuda.synchronize()
    _check_matmul(y, oracle.gemv(L, x_np), "%s batch %d with workspace" % (name, batch))
    assert (ws[need:] == 0xFF).all()
    need1 = gpu_lib.vq_gemv_workspace_bytes(dl.desc, 1)
    if name != "down_fast_long_rows_res12":
        assert need1 == 0                # a single row stays on the kernel that needs none
        return
    # ... unless the row is too long for that kernel's LDS beside the tables: then one row runs in column parts as well,
    # and without a workspace on the matrix-core kernel alone
    assert need1 >= 2 * L.out_features * 4
    for workspace in (ws[:need1], None):
        y1 = gpu_lib.gemv(dl, x[:1], workspace=workspace)
        torch.cuda.synchronize()
        _check_matmul(y1, oracle.gemv(L, x_np[:1]), "%s one row, workspace %s" % (name, workspace is not None))


@pytest.mark.parametrize("workspace", [None, "fast"])
@pytest.mark.parametrize("batch", [1, 3, 5, 16])
@pytest.mark.parametrize("name,pad_x,pad_y", [("down_fast_res12", 8, 1), ("down_fast_outlier", 24, 6), ("down_fast_parts", 16, 3),
                                               ("down_fast_groups_outlier_tall", 8, 5),
                                               ("down_v6", 1, 3)])       # 391 columns: the last row ends inside a dword
def test_native_orientation_strided_buffers_and_untouched_padding(gpu_lib, name, pad_x, pad_y, batch, workspace):
    """Vectors down the output dimension, fast kernels (row stride of x a multiple of 8): NaN in the caller's padding of x
    must never reach a sum, and sentinels in the padding of y must survive; with and without the workspace route."""
    import torch
    L = small_layer(name)
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(300, L, batch)
    xb = torch.full((batch, L.in_features + pad_x), float("nan"), dtype=torch.float16, device="cuda")
    xb[:, : L.in_features] = torch.from_numpy(x).cuda()
    yb = torch.full((batch, L.out_features + pad_y), 7.0, dtype=torch.float16, device="cuda")
    gpu_lib.gemv(dl, xb, out=yb, workspace=workspace)
    torch.cuda.synchronize()
    _check_matmul(yb[:, : L.out_features], oracle.gemv(L, x), "strided %s batch %d workspace %s" % (name, batch, workspace))
    assert (yb[:, L.out_features:] == 7.0).all()


@pytest.mark.parametrize("seed", range(12))
def test_eight_component_layers_random_shapes(gpu_lib, seed):
    """Layers of 8-component vectors in both orientations with random sizes, table sizes (8- and 16-bit indices), residual
    tables and codebook groups: vq_dequant bit for bit, vq_gemv on padded buffers (NaN in x's padding, sentinels in y's)."""
    import torch
    rng = np.random.default_rng(4321 + seed)
    orientation = seed % 2
    out, P = int(rng.integers(1, 1500)), int(rng.integers(1, 700))
    k = int(rng.choice([65536, 256, 40000, 200, 17]))
    kw = {}
    r = int(rng.integers(0, 3))
    if r == 1:
        kw["k_res"] = int(rng.choice([256, 100]))
    if r == 2:
        kw["k_res"] = int(rng.choice([65536, 5000]))
    if rng.integers(0, 3) == 0:
        kw["group_vectors"] = int(rng.integers(1, max(2, P)))
    in_features = P * 8 if orientation == 0 else int(rng.integers(1, 3000))
    L = s.make_layer(9200 + seed, "v8_random_%d" % seed, out, in_features, 8, k, orientation=orientation, **kw)
    dl = gpu_lib.DeviceLayer(L)
    W = gpu_lib.dequant(dl)
    torch.cuda.synchronize()
    assert np.array_equal(W.cpu().numpy().view(np.uint16), oracle.dequant(L).view(np.uint16)), (out, in_features, k, kw)
    for batch in (1, 2, int(rng.integers(3, 17))):
        x = s.make_activations(9200 + seed, L, batch)
        xb = torch.full((batch, (in_features + 7) // 8 * 8 + 8), float("nan"), dtype=torch.float16, device="cuda")
        xb[:, :in_features] = torch.from_numpy(x).cuda()
        yb = torch.full((batch, out + 3), 7.0, dtype=torch.float16, device="cuda")
        gpu_lib.gemv(dl, xb, out=yb)
        torch.cuda.synchronize()
        _check_matmul(yb[:, :out], oracle.gemv(L, x), "v = 8, orientation %d, %d x %d, k %d, %s, batch %d" % (orientation, out, in_features, k, kw, batch))
        assert (yb[:, out:] == 7.0).all()


@pytest.mark.parametrize("seed", range(48))
def test_lds_table_kernels_random_shapes(gpu_lib, seed):
    """The (v, index width) pairs of the LDS-table kernels, in both orientations, with random sizes, table sizes, residual
    tables of the same index width, codebook groups, outlier columns of v = 4 (up to 13 index bits) and permutations: vq_dequant bit for bit (W with a
    padded, sentinel-filled pitch), vq_gemv on padded buffers (NaN in x's padding, sentinels in y's), vq_gemm with the
    restore-then-multiply workspace where the layer has one."""
    import torch
    rng = np.random.default_rng(97531 + seed)
    v, bits = [(2, 4), (4, 8), (6, 8), (8, 8), (4, 12), (8, 12), (12, 12), (6, 12)][seed % 8]
    k = int(rng.integers(2 ** (bits - 1) + 1, 2 ** bits + 1))
    out = int(rng.integers(1, 6000)) if seed % 3 == 0 else int(rng.integers(1, 700))
    orientation = 1 if seed >= 24 else 0               # (the second half: vectors down the output dimension, any number of outlier columns)
    n_out = (4 if orientation == 0 else 1) * int(rng.integers(0, 12)) if rng.integers(0, 2) else 0
    in_features = n_out + int(rng.integers(1, 2600))
    kw = {}
    if rng.integers(0, 2):
        kw["k_res"] = int(rng.integers(2 ** (bits - 1) + 1, 2 ** bits + 1))
    if n_out:
        kw.update(n_outlier_cols=n_out, v_out=4, k_out=int(rng.choice([8192, 4096, 300, 5000])))
    P = -(-(in_features - n_out) // v) if orientation == 0 else in_features - n_out
    if rng.integers(0, 2):
        kw["group_vectors"] = int(rng.integers(max(1, P // 17), P + 1))
    if rng.integers(0, 3) == 0:
        kw["permute"] = True
    if orientation:
        kw["orientation"] = 1
    what = "v %d, %d-bit, %d x %d, k %d, %s" % (v, bits, out, in_features, k, kw)
    L = s.make_layer(9300 + seed, "lds_random_%d" % seed, out, in_features, v, k, **kw)
    dl = gpu_lib.DeviceLayer(L)
    ldw = in_features + int(rng.choice([0, 2, 5, 8]))
    W = torch.full((out, ldw), 3.0, dtype=torch.float16, device="cuda")
    assert gpu_lib.vq_dequant(dl.desc, W.data_ptr(), ldw, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert np.array_equal(W[:, :in_features].cpu().numpy().view(np.uint16), oracle.dequant(L).view(np.uint16)), what
    assert (W[:, in_features:] == 3.0).all(), what
    for batch in (1, 2, 4, int(rng.integers(3, 17))):
        x = s.make_activations(9300 + seed, L, batch)
        xb = torch.full((batch, (in_features + 7) // 8 * 8 + 8), float("nan"), dtype=torch.float16, device="cuda")
        xb[:, :in_features] = torch.from_numpy(x).cuda()
        yb = torch.full((batch, out + 3), 7.0, dtype=torch.float16, device="cuda")
        ref = oracle.gemv(L, x)
        for workspace in (None, "fast"):     # (with a workspace: a codebook group or the outlier columns per workgroup, then a sum)
            yb.fill_(7.0)
            gpu_lib.gemv(dl, xb, out=yb, workspace=workspace)
            torch.cuda.synchronize()
            _check_matmul(yb[:, :out], ref, what + ", batch %d, workspace %s" % (batch, workspace))
            assert (yb[:, out:] == 7.0).all()
    if in_features % 256 == 0:
        x = s.make_activations(9300 + seed, L, 70)
        Y = gpu_lib.gemm(dl, torch.from_numpy(x).cuda(), workspace="fast")
        torch.cuda.synchronize()
        _check_matmul(Y, oracle.gemm(L, x), what + ", 70 tokens")
