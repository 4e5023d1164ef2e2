"""Pins for the oracle's nearest-centroid assignment (Eq. 2 of Sec. 2.2; residual stage of Sec. 3.2.2): exact rational
brute force, constructed ties, a library routine, the decoder's own format."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.cluster.vq import vq as scipy_vq

import oracle
import vq_synth as s


def _exact_distances(t, C):
    """Exact squared distances of one vector (its valid elements) to every centroid."""
    return [sum((Fraction(float(a)) - Fraction(float(c))) ** 2 for a, c in zip(t, row)) for row in C]


@pytest.mark.parametrize("v,k,cols", [(6, 64, 31), (4, 17, 16), (8, 300, 21), (1, 2, 5), (5, 37, 23)])
def test_assign_is_the_exact_argmin_up_to_binary32_rounding(v, k, cols):
    rng = np.random.default_rng(v * 1000 + k)
    C = rng.normal(0, 0.02, (k, v)).astype(np.float16)
    W = rng.normal(0, 0.02, (5, cols + 3)).astype(np.float16)          # ld > cols: the padding must not be read as data
    W[:, cols:] = np.float16(9.0)
    idx = oracle.assign(W, C, cols=cols)
    P = -(-cols // v)
    assert idx.shape == (5, P)
    same = 0
    for o in range(5):
        for p in range(P):
            t = W[o, p * v:min(p * v + v, cols)]
            d = _exact_distances(t, C)
            best = min(d)
            # the chosen centroid is a nearest one within the rounding of a sum of v binary32 terms
            assert d[idx[o, p]] <= best * (1 + Fraction(v + 2, 2 ** 23)), (o, p)
            same += d[idx[o, p]] == best and idx[o, p] == d.index(best)
    assert same >= 5 * P - 1                                            # near-ties at that scale are rare


def test_ties_go_to_the_lowest_index():
    C = np.array([[1, 0], [0.5, 0.5], [-1, 0], [1, 0], [0, 1]], dtype=np.float16)
    W = np.array([[0, 0,   1, 0,   0.75, 0.25,   0, 2]], dtype=np.float16)
    # (0,0): centroids 0, 2, 3, 4 at distance 1, centroid 1 at 0.5 -> 1;  (1,0): 0 and 3 coincide -> 0;
    # (0.75,0.25): 0, 1 and 3 at 0.125 -> 0;  (0,2): 4 alone at 1 -> 4
    assert oracle.assign(W, C).tolist() == [[1, 0, 0, 4]]
    # the same with the tied pair swapped in the table: still the lower index
    assert oracle.assign(W, C[[3, 1, 2, 0, 4]]).tolist() == [[1, 0, 0, 4]]


def test_codebook_rows_map_to_themselves():
    rng = np.random.default_rng(5)
    C = np.unique(rng.normal(0, 0.02, (500, 6)).astype(np.float16), axis=0)
    rng.shuffle(C)
    order = rng.permutation(len(C))
    W = C[order].reshape(10, -1)
    assert np.array_equal(oracle.assign(W, C).reshape(-1), order)


def test_agrees_with_scipy_where_the_margin_is_clear():
    rng = np.random.default_rng(11)
    C = rng.normal(0, 0.02, (256, 6)).astype(np.float16)
    W = rng.normal(0, 0.02, (40, 60)).astype(np.float16)
    idx = oracle.assign(W, C).reshape(-1)
    obs = W.astype(np.float64).reshape(-1, 6)
    code, _ = scipy_vq(obs, C.astype(np.float64))
    d = ((obs[:, None, :] - C.astype(np.float64)[None]) ** 2).sum(-1)
    two = np.sort(d, axis=1)[:, :2]
    clear = two[:, 1] - two[:, 0] > 1e-9
    assert clear.mean() > 0.99 and np.array_equal(idx[clear], code[clear])


def test_ragged_last_vector_uses_only_its_own_elements():
    # last vector holds one element, 0.3: nearest first element wins, whatever the centroids' other elements are
    C = np.array([[0.3, 5, 5], [0.1, 0, 0], [0.29, -7, 2]], dtype=np.float16)
    W = np.array([[0.1, 0, 0, 0.3]], dtype=np.float16)
    assert oracle.assign(W, C).tolist() == [[1, 0]]
    # zero padding instead would pick centroid 1 for the last vector
    Wp = np.array([[0.1, 0, 0, 0.3, 0, 0]], dtype=np.float16)
    assert oracle.assign(Wp, C).tolist() == [[1, 1]]


def test_residual_stage_assigns_the_difference():
    rng = np.random.default_rng(13)
    # values on a coarse grid: W - B is exact in binary16, so the residual stage must equal a plain stage on the difference
    W = (rng.integers(-40, 40, (6, 24)) / 64).astype(np.float16)
    B = (rng.integers(-40, 40, (6, 24)) / 64).astype(np.float16)
    C = (rng.integers(-20, 20, (50, 4)) / 64).astype(np.float16)
    D = (W.astype(np.float32) - B.astype(np.float32)).astype(np.float16)
    assert np.array_equal(D.astype(np.float32), W.astype(np.float32) - B.astype(np.float32))
    assert np.array_equal(oracle.assign(W, C, base=B), oracle.assign(D, C))
    assert np.array_equal(oracle.assign(W, C, base=np.zeros_like(W)), oracle.assign(W, C))
    assert not np.array_equal(oracle.assign(W, C, base=B), oracle.assign(W, C))


def test_two_stage_encode_then_decode_lowers_the_error():
    """Sec. 3.2.2: the second stage quantizes what the first left over; decode adds the two centroids."""
    rng = np.random.default_rng(17)
    L = s.make_layer(210, "enc", 12, 60, 6, 256, k_res=64, with_scale=False, with_bias=False)
    L.codebook_res[0] = 0                                               # "no correction" is on offer
    W = rng.normal(0, 0.02, (12, 60)).astype(np.float16)
    L.raw_idx = oracle.assign(W, L.codebook)
    L.idx = s.pack_indices(L.raw_idx, L.bits)
    stage1 = L.codebook[L.raw_idx].reshape(12, 60)
    L.raw_idx_res = oracle.assign(W, L.codebook_res, base=stage1)
    L.idx_res = s.pack_indices(L.raw_idx_res, L.bits_res)
    What = oracle.dequant(L).astype(np.float64)
    e1 = ((W.astype(np.float64) - stage1.astype(np.float64)) ** 2).reshape(12, 10, 6).sum(-1)
    e2 = ((W.astype(np.float64) - What) ** 2).reshape(12, 10, 6).sum(-1)
    assert (e2 <= e1 + 1e-9).all() and e2.sum() < 0.8 * e1.sum()


def test_encoding_a_decoded_layer_returns_its_indices():
    L = s.make_layer(211, "rt", 9, 100, 6, 256, with_scale=False, with_bias=False)
    assert len(np.unique(L.codebook, axis=0)) == 256
    W = oracle.dequant(L)
    idx = oracle.assign(W, L.codebook)
    assert np.array_equal(idx, L.raw_idx)
    assert np.array_equal(s.pack_indices(idx, L.bits, L.idx.shape[1]), L.idx)


@pytest.mark.parametrize("rows,cols,v", [(24, 11, 6), (23, 9, 6), (5, 4, 8), (7, 13, 1)])
def test_vectors_down_the_columns_are_the_transposed_problem(rows, cols, v):
    """Sec. 3.1 / Algorithm 1: the paper's vectors are v consecutive rows of a column -- the row-wise vectors of the
    transposed matrix, cut-off last block included."""
    rng = np.random.default_rng(rows * 100 + cols)
    W = rng.normal(0, 0.02, (rows, cols + 2)).astype(np.float16)
    B = rng.normal(0, 0.01, (rows, cols + 2)).astype(np.float16)
    C = rng.normal(0, 0.02, (50, v)).astype(np.float16)
    down = oracle.assign(W, C, cols=cols, orientation=1)
    assert down.shape == (-(-rows // v), cols)
    assert np.array_equal(down, oracle.assign(np.ascontiguousarray(W[:, :cols].T), C).T)
    down_b = oracle.assign(W, C, base=B, cols=cols, orientation=1)
    assert np.array_equal(down_b, oracle.assign(np.ascontiguousarray(W[:, :cols].T), C, base=np.ascontiguousarray(B[:, :cols].T)).T)
    assert not np.array_equal(down, down_b)


def test_encoding_a_decoded_layer_of_the_papers_orientation_returns_its_indices():
    L = s.make_layer(212, "rt_down", 20, 33, 6, 256, with_scale=False, with_bias=False, orientation=1)
    assert len(np.unique(L.codebook, axis=0)) == 256
    idx = oracle.assign(oracle.dequant(L), L.codebook, orientation=1)
    assert np.array_equal(idx, L.raw_idx)
