"""GPU parity at the five benchmark configurations, full size, through the C ABI."""
import numpy as np
import pytest

import oracle
import vq_synth as s

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def layers():
    cache = {}

    def get(cfg, name=None):
        key = (cfg, name)
        if key not in cache:
            cache.clear()                      # one big layer resident at a time
            cache[key] = next(s.config_layers(cfg, only=name))
        return cache[key]
    return get


def _dequant_exact(gpu_lib, L):
    import torch
    dl = gpu_lib.DeviceLayer(L)
    W = gpu_lib.dequant(dl)
    torch.cuda.synchronize()
    got = W.cpu().numpy().view(np.uint16)
    del W
    want = oracle.dequant(L).view(np.uint16)
    assert np.array_equal(got, want)
    return dl


def _matmul_ok(y, ref, what):
    y = y.float().cpu().numpy().astype(np.float64)
    rms = np.sqrt((ref ** 2).mean())
    err = np.abs(y - ref).max()
    assert np.isfinite(y).all() and err <= TOL * rms, "%s: err %.3e rms %.3e" % (what, err, rms)


@pytest.mark.parametrize("cfg,name", [(0, "tiny"), (1, "up"), (2, "q"), (2, "o"), (2, "gate"), (2, "down"), (3, "down70b"), (4, "prefill")])
def test_config_dequant_and_gemv(gpu_lib, layers, monkeypatch, cfg, name):
    import torch
    ordinal, L = layers(cfg, name)
    dl = _dequant_exact(gpu_lib, L)
    spec = s.CONFIGS[cfg]
    batches = spec["rows"] if cfg != 4 else [1, 16]
    for batch in batches:
        x = s.make_activations(cfg, L, batch, layer_ordinal=ordinal, outlier_gain=spec.get("outlier_gain", 1.0))
        ref = oracle.gemv(L, x)
        xd = torch.from_numpy(x).cuda()
        for kernel in ("auto", "m", "d"):              # default dispatch, matrix-core kernel, dot-product kernels
            if kernel != "auto":
                monkeypatch.setenv("VQ_SWITCHES", "gemv=" + kernel)
            y = gpu_lib.gemv(dl, xd)
            torch.cuda.synchronize()
            monkeypatch.delenv("VQ_SWITCHES", raising=False)
            _matmul_ok(y, ref, "cfg%d %s batch %d kernel %s" % (cfg, name, batch, kernel))


@pytest.mark.parametrize("tokens", [512, 1024, 2048])
@pytest.mark.parametrize("workspace", [None, "fast"])
def test_config4_prefill_gemm(gpu_lib, layers, tokens, workspace):
    import torch
    _, L = layers(4, "prefill")
    dl = gpu_lib.DeviceLayer(L)
    x = s.make_activations(4, L, tokens)
    Y = gpu_lib.gemm(dl, torch.from_numpy(x).cuda(), workspace=workspace)
    torch.cuda.synchronize()
    if tokens == 512:
        _matmul_ok(Y, oracle.gemm(L, x), "cfg4 T=512 full")
    else:
        # larger token counts: every 16th output row plus the edges, all tokens
        rows = np.unique(np.concatenate([np.arange(0, L.out_features, 16), [L.out_features - 1, 127, 128, 8191 - 128]])).astype(np.int32)
        ref = oracle.gemm(L, x, rows=rows)
        _matmul_ok(Y[:, torch.from_numpy(rows.astype(np.int64)).cuda()], ref, "cfg4 T=%d sampled rows" % tokens)


@pytest.mark.parametrize("workspace", [None, "fast"])
def test_config3_small_gemm_with_outliers(gpu_lib, layers, workspace):
    import torch
    _, L = layers(3, "down70b")
    sub = s.make_layer(3, "slice", 256, L.in_features, 6, 4096, 256, 288, 4, 4096)
    dl = gpu_lib.DeviceLayer(sub)
    x = s.make_activations(3, sub, 64, outlier_gain=10.0)
    Y = gpu_lib.gemm(dl, torch.from_numpy(x).cuda(), workspace=workspace)
    torch.cuda.synchronize()
    _matmul_ok(Y, oracle.gemm(sub, x), "cfg3 slice gemm")


@pytest.mark.parametrize("names", [("q", "k", "v"), ("gate", "up")])
def test_config2_projections_in_one_launch(gpu_lib, names):
    """vq_gemv_multi as the benchmark runs it: the 7B decoder layer's q, k, v (and gate, up) on one x, every output row."""
    import torch
    pairs = [next(s.config_layers(2, only=n)) for n in names]
    dls = [gpu_lib.DeviceLayer(L) for _, L in pairs]
    for batch in s.CONFIGS[2]["rows"]:
        x = s.make_activations(2, pairs[0][1], batch, layer_ordinal=pairs[0][0])
        ys = gpu_lib.gemv_multi(dls, torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        for (_, L), y in zip(pairs, ys):
            _matmul_ok(y, oracle.gemv(L, x), "cfg2 %s of %s batch %d" % (L.name, "+".join(names), batch))


@pytest.mark.parametrize("group_vectors", [176, 48])
def test_headline_shape_with_codebook_groups(gpu_lib, group_vectors):
    """The 11008 x 4096 layer split into 4 and 15 codebook groups, as bench.py's detail lines time it."""
    import torch
    L = s.make_layer(1, "up", 11008, 4096, 6, 4096, group_vectors=group_vectors)
    dl = _dequant_exact(gpu_lib, L)
    for batch in (1, 16):
        x = s.make_activations(1, L, batch)
        ref = oracle.gemv(L, x)
        for workspace in (None, "fast"):
            y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda(), workspace=workspace)
            torch.cuda.synchronize()
            _matmul_ok(y, ref, "grouped headline shape, %d vectors a group, batch %d, workspace %s" % (group_vectors, batch, workspace))


@pytest.mark.parametrize("extra", [dict(), dict(k_res=4096, n_outlier_cols=40, v_out=4, k_out=4096), dict(group_vectors=256, k_res=256)])
def test_headline_shape_in_the_papers_orientation(gpu_lib, extra):
    """The 11008 x 4096 layer with vectors down the output dimension, as bench.py's detail lines time it: the vector-ALU
    kernel (one row), the matrix-core kernel alone and with the column parts of the workspace route."""
    import torch
    L = s.make_layer(1, "up", 11008, 4096, 6, 4096, orientation=1, **extra)
    dl = _dequant_exact(gpu_lib, L)
    for batch in (1, 4, 7, 16):
        x = s.make_activations(1, L, batch)
        ref = oracle.gemv(L, x)
        for workspace in (None, "fast"):
            y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda(), workspace=workspace)
            torch.cuda.synchronize()
            _matmul_ok(y, ref, "headline shape, orientation 1, batch %d, %s, workspace %s" % (batch, extra, workspace))


def test_config3_with_scattered_outlier_columns(gpu_lib):
    """The 8192 x 28672 layer of the 70B setting with its columns stored in a permuted order, so that the 288 outlier
    columns lie scattered over the layer (Sec. 3.2.3): restored matrix bit-exact, products with and without a workspace."""
    import torch
    c = s.CONFIGS[3]
    L = s.make_layer(3, "down70b", 8192, 28672, c["v"], c["k"], c["k_res"], c["n_outlier_cols"], c["v_out"], c["k_out"], permute=True)
    assert sorted(L.col_perm[:288]) != list(range(288))
    dl = _dequant_exact(gpu_lib, L)
    for batch in (1, 8):
        x = s.make_activations(3, L, batch, outlier_gain=c["outlier_gain"])
        ref = oracle.gemv(L, x)
        for workspace in (None, "fast"):
            y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda(), workspace=workspace)
            torch.cuda.synchronize()
            _matmul_ok(y, ref, "cfg3 with permuted columns, batch %d, workspace %s" % (batch, workspace))


@pytest.mark.parametrize("cfg,name,tokens", [(1, "up", 512), (2, "q", 300), (2, "down", 130), (3, "down70b", 130)])
def test_prefill_without_workspace_on_the_v6_layers(gpu_lib, layers, cfg, name, tokens):
    """vq_gemm without a workspace on the 7B-shaped v = 6 layers (no residual; 12-bit residual) and on the 70B-shaped one (8-bit
    residual, 288 outlier columns): the kernel that restores W on the fly from tables in LDS, every 16th output row plus the
    edges against the oracle."""
    import torch
    ordinal, L = layers(cfg, name)
    dl = gpu_lib.DeviceLayer(L)
    assert gpu_lib.vq_gemm_workspace_bytes(dl.desc, tokens) == 0
    x = s.make_activations(cfg, L, tokens, layer_ordinal=ordinal)
    Y = gpu_lib.gemm(dl, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, L.out_features, 16), [L.out_features - 1, 127, 128, L.out_features - 128]])).astype(np.int32)
    _matmul_ok(Y[:, torch.from_numpy(rows.astype(np.int64)).cuda()], oracle.gemm(L, x, rows=rows), "cfg%d %s T=%d on the fly" % (cfg, name, tokens))


@pytest.mark.parametrize("orientation", [0, 1])
def test_the_2_26_bit_setting_at_full_size(gpu_lib, orientation):
    """The 11008 x 4096 layer in the 2.26-bit setting of Table "Quantization parameters" (v = 12, two 4096-entry tables, four
    codebook groups, 40 outlier columns of v = 4 with 8192 entries), both orientations: vq_dequant bit for bit, vq_gemv with one
    and with five rows, without and with a workspace, vq_gemm at 300 tokens through the restore-then-multiply route on every
    16th output row."""
    import torch
    P = -(-(4096 - 40) // 12) if orientation == 0 else 4096 - 40
    L = s.make_layer(1, "up", 11008, 4096, 12, 4096, 4096, n_outlier_cols=40, v_out=4, k_out=8192, group_vectors=-(-P // 4),
                     orientation=orientation)
    dl = _dequant_exact(gpu_lib, L)
    for batch in (1, 5):
        x = s.make_activations(1, L, batch)
        ref = oracle.gemv(L, x)
        for workspace in (None, "fast"):
            y = gpu_lib.gemv(dl, torch.from_numpy(x).cuda(), workspace=workspace)
            torch.cuda.synchronize()
            _matmul_ok(y, ref, "2.26-bit setting, orientation %d, batch %d, workspace %s" % (orientation, batch, workspace))
    x = s.make_activations(1, L, 300)
    Y = gpu_lib.gemm(dl, torch.from_numpy(x).cuda(), workspace="fast")
    torch.cuda.synchronize()
    rows = np.arange(0, L.out_features, 16).astype(np.int32)
    _matmul_ok(Y[:, torch.from_numpy(rows.astype(np.int64)).cuda()], oracle.gemm(L, x, rows=rows), "2.26-bit setting, 300 tokens")
