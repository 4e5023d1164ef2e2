"""GPU parity of vq_assign (nearest-centroid assignment, Eq. 2 / residual stage of Sec. 3.2.2) through the C ABI:
the packed index streams bit for bit against the oracle's indices packed by the input generator's packer."""
import numpy as np
import pytest

import oracle
import vq_synth as s

pytestmark = pytest.mark.gpu

# rows, cols, v, k: ragged last vectors, several lanes' segments per row, partly filled workgroups, a table walked in
# LDS chunks (k = 65536), k not a power of two, cols < v
CASES = {
    "v6_k4096_ragged": (70, 391, 6, 4096),
    "v6_k256_exact": (256, 384, 6, 256),
    "v8_k65536_chunks": (33, 520, 8, 65536),
    "v4_k4096": (50, 1200, 4, 4096),
    "v5_k37": (37, 203, 5, 37),
    "v1_k2": (9, 77, 1, 2),
    "v16_k300": (33, 530, 16, 300),
    "v12_k4096": (20, 600, 12, 4096),
    "v6_k3000_many_rows": (3000, 390, 6, 3000),
    "one_short_vector": (5, 4, 6, 64),
    "v7_long_rows": (3, 9000, 7, 512),
}


def _inputs(name, with_base):
    rows, cols, v, k = CASES[name]
    seed = 7000 + list(CASES).index(name)
    ld = cols + 5
    W = s.to_fp16(s.normal(seed, rows * ld, 0.02)).reshape(rows, ld)
    C = s.to_fp16(s.normal(seed + 100, k * v, 0.02)).reshape(k, v)
    B = s.to_fp16(s.normal(seed + 200, rows * ld, 0.015)).reshape(rows, ld) if with_base else None
    return W, C, B, cols


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("with_base", [False, True])
def test_assign_bit_exact(gpu_lib, name, with_base):
    import torch
    W, C, B, cols = _inputs(name, with_base)
    k, v = C.shape
    idx = gpu_lib.assign(torch.from_numpy(W).cuda(), torch.from_numpy(C).cuda(),
                         base=torch.from_numpy(B).cuda() if with_base else None, cols=cols)
    torch.cuda.synchronize()
    want = oracle.assign(W, C, base=B, cols=cols)
    bits = oracle.index_bits(k)
    packed = s.pack_indices(want, bits, idx.shape[1])
    got = idx.cpu().numpy()
    if not np.array_equal(got, packed):
        mine = np.stack([oracle.unpack_row(got[o], bits, want.shape[1]) for o in range(got.shape[0])])
        bad = np.argwhere(mine != want)
        raise AssertionError("%s: %d of %d indices differ, first at %s: %d vs %d" %
                             (name, len(bad), want.size, bad[0], mine[tuple(bad[0])], want[tuple(bad[0])]))


def test_assign_leaves_the_rest_of_the_stride_alone(gpu_lib):
    import torch
    W, C, _, cols = _inputs("v6_k4096_ragged", False)
    P = -(-cols // 6)
    used = -(-P * 12 // 32) * 4
    stride = (used + 15) // 16 * 16 + 32
    idx = torch.full((W.shape[0], stride), 0xAB, dtype=torch.uint8, device="cuda")
    Wd, Cd = torch.from_numpy(W).cuda(), torch.from_numpy(C).cuda()
    rc = gpu_lib.vq_assign(Wd.data_ptr(), None, W.shape[1], W.shape[0], cols, Cd.data_ptr(), 6, 4096, idx.data_ptr(), stride,
                           torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == 0
    got = idx.cpu().numpy()
    assert (got[:, used:] == 0xAB).all()
    assert np.array_equal(got[:, :used], s.pack_indices(oracle.assign(W, C, cols=cols), 12, used))


def test_encode_then_decode_on_the_gpu(gpu_lib):
    """Two stages (Sec. 3.2.2) on the device, then vq_dequant: the oracle restores the same matrix from the same streams,
    and the second stage lowers the error."""
    import torch
    L = s.make_layer(7100, "enc", 64, 600, 6, 4096, k_res=256, with_scale=False, with_bias=False)
    W = s.to_fp16(s.normal(7101, 64 * 600, 0.02)).reshape(64, 600)
    Wd, Cd, Crd = (torch.from_numpy(a).cuda() for a in (W, L.codebook, L.codebook_res))
    idx = gpu_lib.assign(Wd, Cd)
    L.idx = idx.cpu().numpy()
    plain = s.VQLayer("stage1", 64, 600, 6, 4096)
    plain.codebook, plain.idx = L.codebook, L.idx
    stage1 = gpu_lib.dequant(gpu_lib.DeviceLayer(plain))
    idx_res = gpu_lib.assign(Wd, Crd, base=stage1)
    L.idx_res = idx_res.cpu().numpy()
    both = gpu_lib.dequant(gpu_lib.DeviceLayer(L))
    torch.cuda.synchronize()
    assert np.array_equal(both.cpu().numpy().view(np.uint16), oracle.dequant(L).view(np.uint16))
    e1 = ((W.astype(np.float64) - stage1.cpu().numpy().astype(np.float64)) ** 2).sum()
    e2 = ((W.astype(np.float64) - both.cpu().numpy().astype(np.float64)) ** 2).sum()
    assert e2 < e1


def test_assign_at_the_headline_size_on_sampled_rows(gpu_lib):
    """The 11008 x 4096 layer against its own 4096 x 6 table: every row on the GPU, sampled rows through the oracle."""
    import torch
    _, L = next(s.config_layers(1))
    W = s.to_fp16(s.normal(7200, L.out_features * L.in_features, 0.02)).reshape(L.out_features, L.in_features)
    idx = gpu_lib.assign(torch.from_numpy(W).cuda(), torch.from_numpy(L.codebook).cuda())
    torch.cuda.synchronize()
    rows = [0, 1, 4095, 7777, 11006, 11007]
    want = oracle.assign(W[rows], L.codebook)
    assert np.array_equal(idx.cpu().numpy()[rows], s.pack_indices(want, 12, idx.shape[1]))


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("with_base", [False, True])
def test_assign_down_bit_exact(gpu_lib, name, with_base):
    """The paper's own vectors (v consecutive rows of a column): index streams per block of rows, bit for bit."""
    import torch
    W, C, B, cols = _inputs(name, with_base)
    k, v = C.shape
    idx = gpu_lib.assign(torch.from_numpy(W).cuda(), torch.from_numpy(C).cuda(),
                         base=torch.from_numpy(B).cuda() if with_base else None, cols=cols, orientation=1)
    torch.cuda.synchronize()
    want = oracle.assign(W, C, base=B, cols=cols, orientation=1)
    assert idx.shape[0] == want.shape[0] == -(-W.shape[0] // v)
    assert np.array_equal(idx.cpu().numpy(), s.pack_indices(want, oracle.index_bits(k), idx.shape[1])), name


def test_encode_then_decode_in_the_papers_orientation(gpu_lib):
    import torch
    L = s.make_layer(7300, "enc_down", 70, 600, 6, 4096, with_scale=False, with_bias=False, orientation=1)
    W = s.to_fp16(s.normal(7301, 70 * 600, 0.02)).reshape(70, 600)
    idx = gpu_lib.assign(torch.from_numpy(W).cuda(), torch.from_numpy(L.codebook).cuda(), orientation=1)
    L.idx = idx.cpu().numpy()
    What = gpu_lib.dequant(gpu_lib.DeviceLayer(L))
    torch.cuda.synchronize()
    assert np.array_equal(What.cpu().numpy().view(np.uint16), oracle.dequant(L).view(np.uint16))
    # every restored vector is the nearest centroid of its block of rows: re-encoding returns the same streams
    again = gpu_lib.assign(What, torch.from_numpy(L.codebook).cuda(), orientation=1)
    torch.cuda.synchronize()
    assert torch.equal(again, idx)
