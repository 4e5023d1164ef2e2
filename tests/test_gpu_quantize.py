"""GPU check of vq_quantize_columns (Algorithm 1, Sec. 3.1) against the CPU oracle.  The loop decides integers from
floating-point distances and several summation orders are legitimate, so the check is one of validity, complete in both
directions: (a) every chosen index is a nearest centroid, within EPS, of the column as the GPU itself propagated it (T),
checked in fp64; (b) T is what the algorithm's recurrence gives for the GPU's own choices, replayed by the oracle in fp64;
(c) the quantized weights are exactly what the indices restore; (d) the second-order loss is within a stated factor of
the loss of the oracle's own run."""
import numpy as np
import pytest

import oracle
import vq_synth as s

pytestmark = pytest.mark.gpu

EPS = 1e-4            # a chosen centroid may be this much (relative) farther than the nearest one: binary32 distances
TOL_T = 1e-4          # max |T_gpu - T_replayed| <= TOL_T * RMS(W): binary32 updates against the fp64 replay
LOSS_BAND = (0.9, 1.1)

CASES = {
    "v6_k4096_three_blocks": dict(M=384, N=300, v=6, k=4096, k_res=0, B=128),       # ragged last block of 44 columns
    "v6_res16_ragged_rows": dict(M=100, N=200, v=6, k=256, k_res=16, B=64),          # last vector of 4 rows
    "v8_k65536_tables_in_memory": dict(M=64, N=130, v=8, k=65536, k_res=0, B=128),   # 1 MB table: read through L2, not LDS
    "v4_res256_small_blocks": dict(M=33, N=70, v=4, k=256, k_res=256, B=32),
    "v12_k4096": dict(M=40, N=50, v=12, k=4096, k_res=0, B=128),
    "v1_scalar": dict(M=70, N=40, v=1, k=16, k_res=0, B=7),
    "v6_res4096_one_block": dict(M=60, N=100, v=6, k=4096, k_res=4096, B=128),
}


def _tables(seed, k, v, k_res):
    C = s.to_fp16(s.normal(s.tensor_seed(600 + seed, 0), k * v, 0.02)).reshape(k, v)
    R = s.to_fp16(s.normal(s.tensor_seed(600 + seed, 1), k_res * v, 0.006)).reshape(k_res, v) if k_res else None
    return C, R


def _unpack(stream_bytes, bits, count):
    return np.stack([oracle.unpack_row(np.ascontiguousarray(row), bits, count) for row in stream_bytes])


def _vector_rows(M, v):
    for p in range(-(-M // v)):
        yield p, slice(p * v, min(M, p * v + v))


@pytest.mark.parametrize("name", list(CASES))
def test_quantize_columns_is_valid_both_ways(gpu_lib, name):
    import torch
    case = CASES[name]
    M, N, v, k, k_res, B = (case[n] for n in ("M", "N", "v", "k", "k_res", "B"))
    seed = list(CASES).index(name)
    W0 = s.make_weights(600 + seed, M, N)
    H = s.make_hessian(600 + seed, N)
    U = np.ascontiguousarray(np.linalg.cholesky(np.linalg.inv(H)).T, dtype=np.float32)             # upper factor of H^-1, as the GPU gets it
    C, R = _tables(seed, k, v, k_res)
    Wd = torch.from_numpy(W0.astype(np.float32)).cuda()
    idx_b, idx_res_b, T = gpu_lib.quantize_columns(Wd, torch.from_numpy(U).cuda(), torch.from_numpy(C).cuda(),
                                                   torch.from_numpy(R).cuda() if k_res else None, block=B)
    torch.cuda.synchronize()
    S = -(-M // v)
    bits, bits_res = oracle.index_bits(k), oracle.index_bits(k_res) if k_res else 0
    idx_bytes = idx_b.cpu().numpy()
    idx = _unpack(idx_bytes, bits, N)
    idx_res = _unpack(idx_res_b.cpu().numpy(), bits_res, N) if k_res else None
    assert idx.shape == (S, N) and idx.max() < k
    # the stream's dwords are written whole (pad bits zero), the rest of the stride is left alone
    used = (N * bits + 31) // 32 * 4
    assert (idx_bytes[:, used:] == 0xEE).all()
    tail_bits = np.unpackbits(idx_bytes[:, :used], axis=1, bitorder="little")[:, N * bits:]
    assert not tail_bits.any()
    Tg = T.cpu().numpy().astype(np.float64)
    What = Wd.cpu().numpy().astype(np.float64)
    Cd = C.astype(np.float64)
    # (a) and (c)
    for p, rows in _vector_rows(M, v):
        ln = rows.stop - rows.start
        t = Tg[rows].T                                                          # [N][ln]
        d = ((t[:, None, :] - Cd[None, :, :ln]) ** 2).sum(2) if k * N * ln < 5e7 else None
        for n in range(N):
            dn = d[n] if d is not None else ((t[n][None, :] - Cd[:, :ln]) ** 2).sum(1)
            assert dn[idx[p, n]] <= dn.min() * (1 + EPS) + 1e-14, (name, p, n)
        q = Cd[idx[p], :ln]                                                     # [N][ln]
        if k_res:
            r = (t.astype(np.float32) - q.astype(np.float32)).astype(np.float64)   # the kernel's residual: one binary32 subtraction
            Rd = R.astype(np.float64)
            dr = ((r[:, None, :] - Rd[None, :, :ln]) ** 2).sum(2)
            chosen = dr[np.arange(N), idx_res[p]]
            assert (chosen <= dr.min(1) * (1 + EPS) + 1e-14).all(), (name, p)
            q = (C[idx[p], :ln].astype(np.float32) + R[idx_res[p], :ln].astype(np.float32)).astype(np.float16).astype(np.float64)
        assert np.array_equal(What[rows].T, q), (name, p)
    # (b) the recurrence, replayed in fp64 with the GPU's choices
    replay = oracle.quantize_columns(W0, U, C, R, block=B, given=(idx, idx_res))
    rms = np.sqrt((W0 ** 2).mean())
    assert np.abs(replay["T"] - Tg).max() <= TOL_T * rms, (name, np.abs(replay["T"] - Tg).max() / rms)
    assert np.array_equal(replay["What"], What)
    # (d) the loss the algorithm is after
    own = oracle.quantize_columns(W0, U, C, R, block=B)
    def loss(Wq):
        d = W0 - Wq
        return np.einsum("on,nm,om->", d, H, d)
    ratio = loss(What) / loss(own["What"])
    assert LOSS_BAND[0] <= ratio <= LOSS_BAND[1], (name, ratio)
    print("%s: indices equal to the oracle's own run: %.4f, max |T - replay| / rms %.2e, loss ratio %.4f"
          % (name, (idx == own["idx"]).mean(), np.abs(replay["T"] - Tg).max() / rms, ratio))


def test_quantize_columns_restores_through_the_layer_path(gpu_lib):
    """The streams it writes are a layer of orientation 1: vq_dequant restores exactly the quantized weights it returned."""
    import torch
    M, N, v, k, k_res = 90, 136, 6, 4096, 256
    W0 = s.make_weights(650, M, N)
    U = np.ascontiguousarray(np.linalg.cholesky(np.linalg.inv(s.make_hessian(650, N))).T, dtype=np.float32)
    C, R = _tables(50, k, v, k_res)
    Wd = torch.from_numpy(W0.astype(np.float32)).cuda()
    idx_b, idx_res_b, _ = gpu_lib.quantize_columns(Wd, torch.from_numpy(U).cuda(), torch.from_numpy(C).cuda(), torch.from_numpy(R).cuda(), block=128, want_T=False)
    again = torch.from_numpy(W0.astype(np.float32)).cuda()
    idx_b2, idx_res_b2, _ = gpu_lib.quantize_columns(again, torch.from_numpy(U).cuda(), torch.from_numpy(C).cuda(), torch.from_numpy(R).cuda(), block=128, want_T=False)
    torch.cuda.synchronize()
    assert torch.equal(idx_b, idx_b2) and torch.equal(idx_res_b, idx_res_b2) and torch.equal(Wd, again)      # deterministic
    L = s.VQLayer("quantized", M, N, v, k, k_res, orientation=1)
    L.codebook, L.codebook_res = C, R
    L.idx, L.idx_res = idx_b.cpu().numpy(), idx_res_b.cpu().numpy()
    restored = gpu_lib.dequant(gpu_lib.DeviceLayer(L))
    torch.cuda.synchronize()
    assert np.array_equal(restored.float().cpu().numpy(), Wd.cpu().numpy())
    assert np.array_equal(oracle.dequant(L).astype(np.float32), Wd.cpu().numpy())


def test_quantize_columns_rejects_bad_arguments(gpu_lib):
    import torch
    W = torch.zeros((12, 16), dtype=torch.float32, device="cuda")
    Hi = torch.eye(16, dtype=torch.float32, device="cuda")
    C = torch.zeros((16, 6), dtype=torch.float16, device="cuda")
    idx = torch.zeros((2, 16), dtype=torch.uint8, device="cuda")
    need = gpu_lib.vq_quantize_columns_workspace_bytes(12, 6, 16, 0)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    def call(**kw):
        a = dict(W=W.data_ptr(), ldw=16, rows=12, cols=16, Hinv=Hi.data_ptr(), ldh=16, cb=C.data_ptr(), v=6, k=16, cbr=None, k_res=0, block=8,
                 idx=idx.data_ptr(), stride=16, idxr=None, strider=0, T=None, ldt=0, ws=ws.data_ptr(), wsb=need)
        a.update(kw)
        return gpu_lib.vq_quantize_columns(a["W"], a["ldw"], a["rows"], a["cols"], a["Hinv"], a["ldh"], a["cb"], a["v"], a["k"], a["cbr"], a["k_res"],
                                           a["block"], a["idx"], a["stride"], a["idxr"], a["strider"], a["T"], a["ldt"], a["ws"], a["wsb"], None)
    assert call() == gpu_lib.VQ_OK
    assert call(W=None) == gpu_lib.VQ_ERR_NULL and call(idx=None) == gpu_lib.VQ_ERR_NULL
    assert call(block=0) == gpu_lib.VQ_ERR_SHAPE and call(block=129) == gpu_lib.VQ_ERR_SHAPE and call(ldw=15) == gpu_lib.VQ_ERR_SHAPE
    assert call(k_res=16) == gpu_lib.VQ_ERR_NULL
    assert call(stride=4) == gpu_lib.VQ_ERR_SHAPE and call(stride=24) == gpu_lib.VQ_ERR_ALIGNMENT
    assert call(wsb=need - 1) == gpu_lib.VQ_ERR_WORKSPACE and call(ws=None) == gpu_lib.VQ_ERR_WORKSPACE
    torch.cuda.synchronize()
