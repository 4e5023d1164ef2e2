"""Pins for the oracle's restatement of the quantizer's column loop (Algorithm 1, Sec. 3.1), CPU only: a test-local
restatement without blocks, special cases that reduce to pinned routines, and the second-order loss the algorithm is
derived from."""
import numpy as np
import pytest

import oracle
import vq_synth as s


def _tables(seed, k, v, k_res=0, sigma=0.02):
    rng = np.random.default_rng(seed)
    C = rng.normal(0, sigma, (k, v)).astype(np.float16)
    R = rng.normal(0, sigma / 4, (k_res, v)).astype(np.float16) if k_res else None
    return C, R


def _upper_factor(H):
    """U upper triangular with U^T U = H^-1: what callers in the GPTQ tradition pass as the algorithm's H^-1."""
    return np.linalg.cholesky(np.linalg.inv(H)).T


def _naive(W, Hinv, C, R):
    """The column loop without blocks, straight from the error-update equation of Sec. 3.1: quantize column q, then
    W[:, q:] -= (W[:, q] - What[:, q]) / Hinv[q, q] * Hinv[q, q:].  numpy only; shares nothing with the oracle."""
    W = W.astype(np.float64).copy()
    M, N = W.shape
    k, v = C.shape
    Cd = C.astype(np.float64)
    Rd = None if R is None else R.astype(np.float64)
    S = -(-M // v)
    idx = np.zeros((S, N), dtype=np.int64)
    idx_res = np.zeros((S, N), dtype=np.int64)
    What = np.zeros_like(W)
    T = np.zeros_like(W)
    for q in range(N):
        T[:, q] = W[:, q]
        for p in range(S):
            rows = slice(p * v, min(M, p * v + v))
            t = W[rows, q]
            i = int(np.argmin(((t[None, :] - Cd[:, : len(t)]) ** 2).sum(1)))
            idx[p, q] = i
            w = Cd[i, : len(t)]
            if Rd is not None:
                r = t - w
                j = int(np.argmin(((r[None, :] - Rd[:, : len(t)]) ** 2).sum(1)))
                idx_res[p, q] = j
                w = (C[i, : len(t)].astype(np.float32) + R[j, : len(t)].astype(np.float32)).astype(np.float16).astype(np.float64)
            What[rows, q] = w
        err = (W[:, q] - What[:, q]) / Hinv[q, q]
        W[:, q:] -= np.outer(err, Hinv[q, q:])
    return idx, idx_res, What, T


CASES = [
    dict(M=12, N=9, v=6, k=16, k_res=0, B=4),
    dict(M=13, N=17, v=6, k=64, k_res=0, B=5),          # ragged last vector, ragged last block
    dict(M=8, N=10, v=4, k=32, k_res=8, B=3),
    dict(M=7, N=6, v=8, k=300, k_res=0, B=128),         # one vector shorter than v, one block
    dict(M=10, N=12, v=1, k=4, k_res=0, B=1),           # scalar quantization, a block per column
]


@pytest.mark.parametrize("case", CASES)
def test_equals_the_loop_without_blocks(case):
    M, N, v, k, k_res, B = (case[n] for n in ("M", "N", "v", "k", "k_res", "B"))
    W = s.make_weights(500, M, N)
    U = _upper_factor(s.make_hessian(500, N))
    C, R = _tables(1, k, v, k_res)
    got = oracle.quantize_columns(W, U, C, R, block=B)
    idx, idx_res, What, T = _naive(W, U, C, R)
    assert np.array_equal(got["idx"], idx)
    if k_res:
        assert np.array_equal(got["idx_res"], idx_res)
    assert np.allclose(got["T"], T, rtol=1e-10, atol=1e-13) and np.allclose(got["What"], What, rtol=0, atol=0)


def test_identity_matrix_means_no_propagation():
    """With Hinv = I nothing is spread: every column is quantized as it came, which is nearest-centroid assignment."""
    W = s.make_weights(501, 20, 14)
    C, R = _tables(2, 64, 6, 16)
    got = oracle.quantize_columns(W, np.eye(14), C, R, block=4)
    assert np.array_equal(got["T"], W)
    first = oracle.assign(W.astype(np.float16), C, orientation=1)
    assert np.array_equal(got["idx"], first)
    restored = C[first].astype(np.float64)                        # [S][N][v] -> rows
    base = np.zeros_like(W)
    for p in range(first.shape[0]):
        rows = slice(p * 6, min(20, p * 6 + 6))
        base[rows] = restored[p].T[: rows.stop - rows.start]
    assert np.array_equal(got["idx_res"], oracle.assign(W.astype(np.float16), R, base=base.astype(np.float16), orientation=1))


def test_block_size_only_regroups_the_updates():
    W = s.make_weights(502, 18, 23)
    U = _upper_factor(s.make_hessian(502, 23))
    C, _ = _tables(3, 128, 6)
    ref = oracle.quantize_columns(W, U, C, block=1)
    for B in (2, 7, 23, 1000):
        got = oracle.quantize_columns(W, U, C, block=B)
        assert np.array_equal(got["idx"], ref["idx"]) and np.allclose(got["T"], ref["T"], rtol=1e-10, atol=1e-13), B


def test_sum_of_squared_errors_is_the_second_order_loss():
    """The optimisation problem of Sec. 3.1 measures a quantization by Delta W H Delta W^T.  With the upper Cholesky factor
    of H^-1 in the role of the algorithm's H^-1, the loop's scaled errors E carry exactly that loss: for every row,
    sum_n E[o, n]^2 = dW[o] H dW[o]^T with dW = W - What."""
    M, N = 12, 20
    W = s.make_weights(503, M, N)
    H = s.make_hessian(503, N)
    U = _upper_factor(H)
    C, R = _tables(4, 64, 6, 16)
    for tables in ((C, None), (C, R)):
        got = oracle.quantize_columns(W, U, *tables, block=6)
        E = (got["T"] - got["What"]) / np.diag(U)[None, :]
        dW = W - got["What"]
        loss = np.einsum("on,nm,om->o", dW, H, dW)
        assert np.allclose((E ** 2).sum(1), loss, rtol=1e-8)
    # ... and spreading the error pays: the loss is below that of rounding every column as it came
    plain = oracle.quantize_columns(W, np.eye(N), C, block=6)
    dP = W - plain["What"]
    got = oracle.quantize_columns(W, U, C, block=6)
    dG = W - got["What"]
    assert np.einsum("on,nm,om->", dG, H, dG) < np.einsum("on,nm,om->", dP, H, dP)


def test_representable_weights_come_back_unchanged():
    C, _ = _tables(5, 32, 6)
    pick = np.random.default_rng(6).integers(0, 32, (3, 11))
    W = np.zeros((18, 11))
    for p in range(3):
        W[p * 6:(p + 1) * 6] = C[pick[p]].astype(np.float64).T
    got = oracle.quantize_columns(W, _upper_factor(s.make_hessian(504, 11)), C, block=4)
    assert np.array_equal(got["What"], W) and np.array_equal(got["T"], W)
    assert np.array_equal(C[got["idx"]], C[pick])                # (equal centroids may carry different numbers)


def test_replaying_given_choices():
    W = s.make_weights(505, 12, 15)
    U = _upper_factor(s.make_hessian(505, 15))
    C, R = _tables(7, 64, 6, 16)
    own = oracle.quantize_columns(W, U, C, R, block=4)
    again = oracle.quantize_columns(W, U, C, R, block=4, given=(own["idx"], own["idx_res"]))
    assert np.array_equal(again["T"], own["T"]) and np.array_equal(again["What"], own["What"])
    # other choices: the propagation follows them (checked against the loop without blocks run with the same choices)
    other = (own["idx"] + 1) % 64
    got = oracle.quantize_columns(W, U, C, R, block=4, given=(other, own["idx_res"]))
    Wd = W.copy()
    for q in range(15):
        assert np.allclose(got["T"][:, q], Wd[:, q], rtol=1e-10, atol=1e-13)
        err = (Wd[:, q] - got["What"][:, q]) / U[q, q]
        Wd[:, q:] -= np.outer(err, U[q, q:])
    assert np.array_equal(got["idx"], other)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_columns(W, U, C, R, block=4, given=(other + 64, own["idx_res"]))
