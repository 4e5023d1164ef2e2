"""Pins for the CPU oracle (CPU only): checks against what the paper and the mathematics fix,
never against the oracle itself.  A naive definition-level implementation lives in this file and
shares nothing with the oracle: it works on the unpacked integer indices with exact rationals."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import accounting
import vq_synth as s

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- unpacker
@pytest.mark.parametrize("bits", range(1, 17))
def test_unpack_roundtrip_all_widths(bits):
    rng = np.random.default_rng(bits)
    for P in (1, 7, 8, 63, 64, 683, 1835):
        for pattern in ("zero", "ones", "alt", "random"):
            if pattern == "zero":
                idx = np.zeros(P, dtype=np.int64)
            elif pattern == "ones":
                idx = np.full(P, (1 << bits) - 1)
            elif pattern == "alt":
                idx = np.where(np.arange(P) % 2 == 0, (1 << bits) - 1, 0)
            else:
                idx = rng.integers(0, 1 << bits, P)
            packed = s.pack_indices(idx[None, :], bits)
            got = oracle.unpack_row(packed[0], bits, P)
            assert np.array_equal(got, idx)
            assert np.array_equal(s.pack_indices(got[None, :], bits), packed)


def test_unpack_handwritten_bytes():
    for line in open(os.path.join(GOLDEN, "packing_bytes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        bits, idx, data = [f.strip() for f in line.split("|")]
        want = [int(t, 0) for t in idx.split()]
        row = np.frombuffer(bytes(int(t, 16) for t in data.split()) + bytes(16), dtype=np.uint8)
        assert list(oracle.unpack_row(row, int(bits), len(want))) == want


def test_unpack_plain_widths_are_reinterpretations():
    rng = np.random.default_rng(5)
    raw = rng.integers(0, 256, 64, dtype=np.uint8)
    assert np.array_equal(oracle.unpack_row(raw, 8, 64), raw)
    assert np.array_equal(oracle.unpack_row(raw, 16, 32), raw.view("<u2"))
    # 12 bit: bytes B0 B1 B2 hold i0 = B0 + ((B1 & 15) << 8), i1 = (B1 >> 4) + (B2 << 4)
    b = raw[:63].reshape(21, 3).astype(np.int64)
    want = np.stack([b[:, 0] + ((b[:, 1] & 15) << 8), (b[:, 1] >> 4) + (b[:, 2] << 4)], 1).ravel()
    assert np.array_equal(oracle.unpack_row(raw, 12, 42), want)


def test_index_bits():
    assert [oracle.index_bits(k) for k in (1, 2, 3, 4, 16, 255, 256, 257, 4096, 65536)] == [1, 1, 2, 2, 4, 8, 8, 9, 12, 16]


# ---------------------------------------------------------------- lookup / structure
def _tiny(**kw):
    args = dict(out_features=5, in_features=31, v=6, k=256)
    args.update(kw)
    name = kw.pop("name", "t")
    return s.make_layer(200, "t", args.pop("out_features"), args.pop("in_features"), args.pop("v"), args.pop("k"), **args)


def _repack(L):
    L.idx = s.pack_indices(L.raw_idx, L.bits)
    if L.k_res:
        L.idx_res = s.pack_indices(L.raw_idx_res, L.bits_res)
    if L.n_outlier_cols:
        L.idx_out = s.pack_indices(L.raw_idx_out, L.bits_out)


def test_one_hot_index_reproduces_codebook_row():
    L = _tiny(out_features=3, in_features=36, with_scale=False, with_bias=False)
    for r in range(L.k):
        L.raw_idx[:] = r
        _repack(L)
        W = oracle.dequant(L)
        want = np.tile(L.codebook[r], L.vectors_per_row)[: L.in_features]
        assert np.array_equal(W.view(np.uint16), np.tile(want.view(np.uint16), (3, 1)))


def test_residual_is_additive_and_zero_table_is_identity():
    L = _tiny(k_res=16)
    base = oracle.dequant(L)
    zeroed = _tiny(k_res=16)
    zeroed.codebook_res[:] = 0
    plain = _tiny()
    assert np.array_equal(oracle.dequant(zeroed).view(np.uint16), oracle.dequant(plain).view(np.uint16))
    only_res = _tiny(k_res=16, with_scale=False, with_bias=False)
    only_res.codebook[:] = 0
    W = oracle.dequant(only_res)
    P = only_res.vectors_per_row
    want = only_res.codebook_res[only_res.raw_idx_res].reshape(5, P * 6)[:, :31]
    assert np.array_equal(W.view(np.uint16), want.view(np.uint16))
    assert not np.array_equal(base, oracle.dequant(plain))


def test_outlier_columns_use_only_their_own_stream():
    kw = dict(out_features=4, in_features=50, k_res=16, n_outlier_cols=8, v_out=4, k_out=32)
    ref = oracle.dequant(_tiny(**kw)).view(np.uint16)
    for stream in ("raw_idx", "raw_idx_res", "raw_idx_out"):
        L = _tiny(**kw)
        a = getattr(L, stream)
        kk = {"raw_idx": L.k, "raw_idx_res": L.k_res, "raw_idx_out": L.k_out}[stream]
        a[:] = (a + 1) % kk
        _repack(L)
        W = oracle.dequant(L).view(np.uint16)
        changed_out = (W[:, :8] != ref[:, :8]).any()
        changed_main = (W[:, 8:] != ref[:, 8:]).any()
        assert (changed_out, changed_main) == ((True, False) if stream == "raw_idx_out" else (False, True))
    # outlier columns hold outlier-table rows: with identity scale/bias they are exact copies
    L = _tiny(with_scale=False, with_bias=False, **kw)
    W = oracle.dequant(L)
    assert np.array_equal(W[:, :8].view(np.uint16), L.codebook_out[L.raw_idx_out].reshape(4, 8).view(np.uint16))


def test_groups_are_the_concatenation_of_single_table_layers():
    """Sec. 3.1 (groups): every range of columns is a layer of its own with its own tables."""
    kw = dict(out_features=4, in_features=8 + 6 * 19 - 2, k=64, k_res=16, n_outlier_cols=8, v_out=4, k_out=32)
    Pg = 8
    L = _tiny(group_vectors=Pg, **kw)
    assert L.n_groups == 3 and L.codebook.shape == (3 * 64, 6) and L.codebook_res.shape == (3 * 16, 6)
    W = oracle.dequant(L).view(np.uint16)
    for g in range(L.n_groups):
        lo, hi = g * Pg, min((g + 1) * Pg, L.vectors_per_row)
        c0, c1 = 8 + lo * 6, min(8 + hi * 6, L.in_features)
        sub = s.VQLayer("sub", 4, c1 - c0, 6, 64, 16)
        sub.codebook, sub.codebook_res = L.codebook[g * 64:(g + 1) * 64], L.codebook_res[g * 16:(g + 1) * 16]
        sub.raw_idx, sub.raw_idx_res = L.raw_idx[:, lo:hi], L.raw_idx_res[:, lo:hi]
        sub.scale, sub.bias = L.scale, L.bias
        _repack(sub)
        assert np.array_equal(oracle.dequant(sub).view(np.uint16), W[:, c0:c1]), g
    # the outlier columns do not depend on the grouping
    assert np.array_equal(W[:, :8], oracle.dequant(_tiny(**kw)).view(np.uint16)[:, :8])


def test_group_tables_reach_only_their_own_columns():
    kw = dict(out_features=3, in_features=6 * 21, k=32, k_res=8)
    ref = oracle.dequant(_tiny(group_vectors=8, **kw)).view(np.uint16)
    for which in ("codebook", "codebook_res"):
        rows = 32 if which == "codebook" else 8
        for g in range(3):
            L = _tiny(group_vectors=8, **kw)
            getattr(L, which)[g * rows:(g + 1) * rows] += np.float16(0.25)
            W = oracle.dequant(L).view(np.uint16)
            differs = (W != ref).any(axis=0).reshape(21, 6).any(axis=1)
            assert np.array_equal(differs, np.arange(21) // 8 == g), (which, g)


def test_one_group_and_equal_tables_reduce_to_the_plain_layer():
    kw = dict(out_features=3, in_features=100, k=64, k_res=16)
    plain = _tiny(**kw)
    want = oracle.dequant(plain).view(np.uint16)
    for Pg in (plain.vectors_per_row, plain.vectors_per_row + 5):          # one group that holds every vector
        L = _tiny(group_vectors=Pg, **kw)
        assert L.n_groups == 1
        assert np.array_equal(oracle.dequant(L).view(np.uint16), want)
    L = _tiny(group_vectors=5, **kw)
    L.codebook = np.tile(plain.codebook, (L.n_groups, 1))
    L.codebook_res = np.tile(plain.codebook_res, (L.n_groups, 1))
    assert np.array_equal(oracle.dequant(L).view(np.uint16), want)
    x = s.make_activations(200, L, 2)
    assert np.array_equal(oracle.matmul(L, x), oracle.matmul(plain, x))


def test_vectors_down_the_output_dimension_are_the_transposed_layer():
    """Sec. 3.1 / Algorithm 1: a column of the quantized matrix is a stack of centroids.  With the same tables and the
    transposed index matrix this is the transpose of a layer whose vectors run along the rows."""
    M, N = 24, 11
    down = _tiny(out_features=M, in_features=N, v=6, k=64, k_res=16, orientation=1, with_scale=False, with_bias=False)
    assert down.raw_idx.shape == (M // 6, N)
    along = s.VQLayer("t", N, M, 6, 64, 16)
    along.codebook, along.codebook_res = down.codebook, down.codebook_res
    along.raw_idx, along.raw_idx_res = down.raw_idx.T.copy(), down.raw_idx_res.T.copy()
    _repack(along)
    assert np.array_equal(oracle.dequant(down).view(np.uint16), oracle.dequant(along).view(np.uint16).T)
    x = s.make_activations(200, down, 2)
    # y = W x for the layer; for its transpose the same numbers come out of the matrix restored above
    assert np.allclose(oracle.matmul(down, x), x.astype(np.float64) @ oracle.dequant(along).astype(np.float64), rtol=1e-12)


def test_vectors_down_the_output_dimension_streams_and_rows():
    kw = dict(out_features=14, in_features=21, v=4, k=32, k_res=8, n_outlier_cols=5, v_out=3, k_out=16, orientation=1)
    ref = oracle.dequant(_tiny(**kw)).view(np.uint16)
    # one index of main stream 2 (rows 8..11), position 7 (column 5 + 7): exactly those four weights change
    L = _tiny(**kw)
    L.raw_idx[2, 7] = (L.raw_idx[2, 7] + 1) % L.k
    _repack(L)
    diff = oracle.dequant(L).view(np.uint16) != ref
    assert diff[8:12, 12].any() and diff.sum() == diff[8:12, 12].sum()
    # one index of outlier stream 4 (rows 12, 13: the last block is cut at 14 rows), column 2
    L = _tiny(**kw)
    L.raw_idx_out[4, 2] = (L.raw_idx_out[4, 2] + 1) % L.k_out
    _repack(L)
    diff = oracle.dequant(L).view(np.uint16) != ref
    assert diff[12:14, 2].any() and diff.sum() == diff[12:14, 2].sum()
    # scale and bias stay per output row
    L = _tiny(**kw)
    L.scale[5] = np.float16(2.0) * L.scale[5]
    diff = oracle.dequant(L).view(np.uint16) != ref
    assert diff[5].any() and not np.delete(diff, 5, axis=0).any()


def test_scale_and_bias_semantics():
    L = _tiny(k_res=16)
    L.codebook[:] = 0
    L.codebook_res[:] = 0
    W = oracle.dequant(L)
    assert np.array_equal(W, np.repeat(L.bias[:, None], 31, 1))           # bias only
    L2 = _tiny(with_bias=False)
    L2.scale[:] = np.float16(4.0)
    L1 = _tiny(with_scale=False, with_bias=False)
    assert np.array_equal(oracle.dequant(L2), oracle.dequant(L1) * np.float16(4.0))   # power of two: exponent shift
    L3 = _tiny()
    L3.scale[:] = 1
    L3.bias[:] = 0
    assert np.array_equal(oracle.dequant(L3).view(np.uint16), oracle.dequant(L1).view(np.uint16))  # NULL == (1, 0)


def test_padding_columns_are_dropped_and_ldw_respected():
    L = _tiny()                       # 31 columns, 6 vectors of 6 -> 5 padded elements never appear
    W = oracle.dequant(L, ldw=40)
    assert W.shape == (5, 40) and not W[:, 31:].any()
    assert np.array_equal(W[:, :31], oracle.dequant(L))


def test_index_out_of_range_is_reported():
    L = _tiny(k=200)                  # 8-bit stream, only 200 entries
    L.raw_idx[2, 3] = 201
    L.idx = s.pack_indices(L.raw_idx, 8)
    with pytest.raises(oracle.OracleError):
        oracle.dequant(L)


def test_column_permutation_places_stored_columns():
    """Sec. 3.2.3: the outlier columns are wherever the Hessian's diagonal puts them; the stored order is a permutation."""
    kw = dict(out_features=4, in_features=50, k_res=16, n_outlier_cols=8, v_out=4, k_out=32)
    L = _tiny(permute=True, **kw)
    perm = L.col_perm
    assert sorted(perm) == list(range(50)) and list(perm) != list(range(50))
    stored = oracle.dequant(_tiny(**kw)).view(np.uint16)               # the same streams and tables without the permutation
    W = oracle.dequant(L).view(np.uint16)
    for c in range(50):
        assert np.array_equal(W[:, perm[c]], stored[:, c]), c
    # x = e_t picks column t of the layer: the token that is one at perm[c] returns stored column c
    y = oracle.matmul(L, np.eye(50, dtype=np.float16))
    assert np.array_equal(y[perm], oracle.dequant(_tiny(**kw)).astype(np.float64).T)
    # the product with x equals the product of the stored-order layer with the gathered activations, term for term
    x = s.make_activations(200, L, 3)
    got, want = oracle.matmul(L, x), oracle.matmul(_tiny(**kw), np.ascontiguousarray(x[:, perm]))
    assert np.allclose(got, want, rtol=1e-12, atol=1e-300)              # same terms, other order of summation
    # the outlier stream reaches exactly the columns perm[0 .. 8)
    M = _tiny(permute=True, **kw)
    M.raw_idx_out[:] = (M.raw_idx_out + 1) % M.k_out
    _repack(M)
    changed = (oracle.dequant(M).view(np.uint16) != W).any(axis=0)
    assert set(np.flatnonzero(changed)) <= set(perm[:8].tolist()) and changed[perm[:8]].any()
    # the identity is no permutation at all
    I = _tiny(**kw)
    I.col_perm = np.arange(50, dtype=np.int32)
    assert np.array_equal(oracle.dequant(I).view(np.uint16), stored)


def test_column_permutation_must_be_a_permutation():
    L = _tiny(permute=True)
    for bad in ("dup", "range", "neg"):
        M = _tiny(permute=True)
        M.col_perm = L.col_perm.copy()
        if bad == "dup":
            M.col_perm[3] = M.col_perm[4]
        elif bad == "range":
            M.col_perm[0] = 31
        else:
            M.col_perm[5] = -1
        with pytest.raises(oracle.OracleError):
            oracle.dequant(M)
        with pytest.raises(oracle.OracleError):
            oracle.matmul(M, s.make_activations(200, M, 1))


# ---------------------------------------------------------------- naive definition (test-local)
def _round_fraction(q: Fraction, precision: int, emin: int) -> Fraction:
    """Round an exact rational to a binary float with `precision` significand bits, min exponent emin, ties-to-even."""
    if q == 0:
        return q
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, emin)
    ulp = Fraction(2) ** (e - precision + 1)
    n = a / ulp
    f = n.numerator // n.denominator
    r = n - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return sign * f * ulp


def _naive_dequant(L):
    """Definition from unpacked indices, exact rationals, explicit roundings: fp32 add, fp32 fma, fp16."""
    W = np.zeros((L.out_features, L.in_features))
    for o in range(L.out_features):
        sc = Fraction(float(L.scale[o])) if L.scale is not None else Fraction(1)
        bi = Fraction(float(L.bias[o])) if L.bias is not None else Fraction(0)
        for c in range(L.in_features):
            down = L.orientation == 1          # vectors down the output dimension: stream o // v, element o % v, one index a column
            if c < L.n_outlier_cols:
                i = L.raw_idx_out[o // L.v_out, c] if down else L.raw_idx_out[o, c // L.v_out]
                d = Fraction(float(L.codebook_out[i, o % L.v_out if down else c % L.v_out]))
            else:
                cc = c - L.n_outlier_cols
                p = cc if down else cc // L.v
                stream, j = (o // L.v, o % L.v) if down else (o, cc % L.v)
                g = p // L.group_vectors if L.group_vectors else 0
                d = Fraction(float(L.codebook.reshape(-1, L.k, L.v)[g, L.raw_idx[stream, p], j]))
                if L.k_res:
                    r = L.codebook_res.reshape(-1, L.k_res, L.v)[g, L.raw_idx_res[stream, p], j]
                    d = _round_fraction(d + Fraction(float(r)), 24, -126)
            w32 = _round_fraction(sc * d + bi, 24, -126)
            W[o, c] = float(_round_fraction(w32, 11, -14))
    if L.col_perm is not None:                 # what was computed is the stored order: stored column c is column col_perm[c]
        placed = np.full_like(W, np.nan)
        for c in range(L.in_features):
            placed[:, int(L.col_perm[c])] = W[:, c]
        W = placed
    return W


CASES = [
    dict(out_features=5, in_features=31, v=6, k=256),
    dict(out_features=4, in_features=50, v=6, k=4096, k_res=4096),
    dict(out_features=3, in_features=47, v=6, k=4096, k_res=256, n_outlier_cols=8, v_out=4, k_out=4096),
    dict(out_features=3, in_features=40, v=8, k=65536),
    dict(out_features=2, in_features=23, v=5, k=37, k_res=11, n_outlier_cols=6, v_out=3, k_out=5),
    dict(out_features=2, in_features=9, v=1, k=2),
    dict(out_features=2, in_features=33, v=16, k=300, with_scale=False),
    dict(out_features=2, in_features=12, v=2, k=16, with_bias=False),
    dict(out_features=3, in_features=61, v=6, k=256, group_vectors=4),                        # 11 vectors: groups of 4, 4, 3
    dict(out_features=3, in_features=75, v=6, k=64, k_res=16, n_outlier_cols=8, v_out=4, k_out=32, group_vectors=8),
    dict(out_features=2, in_features=23, v=5, k=37, k_res=11, group_vectors=1),                # a table per vector
    # vectors down the output dimension: rows not a multiple of v, outlier columns not a multiple of v_out, groups of columns
    dict(out_features=20, in_features=37, v=6, k=64, k_res=16, n_outlier_cols=5, v_out=4, k_out=32, orientation=1),
    dict(out_features=13, in_features=9, v=8, k=300, orientation=1, with_scale=False),
    dict(out_features=7, in_features=30, v=3, k=16, k_res=4, orientation=1, group_vectors=8, with_bias=False),
    # stored column order is a permutation of the layer's (outlier columns scattered over the layer)
    dict(out_features=3, in_features=47, v=6, k=4096, k_res=256, n_outlier_cols=8, v_out=4, k_out=4096, permute=True),
    dict(out_features=4, in_features=29, v=6, k=64, permute=True),
    dict(out_features=3, in_features=75, v=6, k=64, k_res=16, n_outlier_cols=8, v_out=4, k_out=32, group_vectors=8, permute=True),
    dict(out_features=20, in_features=37, v=6, k=64, k_res=16, n_outlier_cols=5, v_out=4, k_out=32, orientation=1, permute=True),
]


@pytest.mark.parametrize("case", CASES)
def test_dequant_equals_naive_definition_bit_exact(case):
    L = _tiny(**case)
    assert np.array_equal(oracle.dequant(L).astype(np.float64), _naive_dequant(L))


def test_dequant_with_subnormal_and_rounding_stress():
    # residual + scale/bias chosen so that fp32 add rounds, fma differs from mul-then-add, and fp16 subnormals appear
    L = _tiny(out_features=6, in_features=36, k=64, k_res=64)
    rng = np.random.default_rng(3)
    L.codebook[:] = (rng.normal(0, 1, L.codebook.shape) * 2.0 ** rng.integers(-16, 2, L.codebook.shape)).astype(np.float16)
    L.codebook_res[:] = (rng.normal(0, 1, L.codebook_res.shape) * 2.0 ** rng.integers(-24, -6, L.codebook_res.shape)).astype(np.float16)
    L.scale[:] = rng.uniform(0.3, 3.0, 6).astype(np.float16)
    L.bias[:] = (rng.normal(0, 1, 6) * 2.0 ** rng.integers(-20, -4, 6)).astype(np.float16)
    W = oracle.dequant(L).astype(np.float64)
    assert np.array_equal(W, _naive_dequant(L))
    assert ((np.abs(W) < 2.0 ** -14) & (W != 0)).any()


@pytest.mark.parametrize("case", CASES)
def test_matmul_equals_bruteforce(case):
    L = _tiny(**case)
    W = _naive_dequant(L)
    x = s.make_activations(200, L, 3)
    want = np.zeros((3, L.out_features))
    for t in range(3):
        for o in range(L.out_features):
            acc = 0.0
            for c in range(L.in_features):
                acc += W[o, c] * float(x[t, c])
            want[t, o] = acc
    got = oracle.matmul(L, x)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-300)
    # the library routine gives the same product up to summation order
    assert np.allclose(got, x.astype(np.float64) @ W.T, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- matmul invariants
def test_unit_vector_extracts_column_exactly():
    L = _tiny(out_features=7, in_features=47, k=4096, k_res=256, n_outlier_cols=8, v_out=4, k_out=4096)
    W = oracle.dequant(L).astype(np.float64)
    x = np.eye(47, dtype=np.float16)
    y = oracle.matmul(L, x)              # token j is e_j
    assert np.array_equal(y, W.T)


def test_linearity_with_exact_inputs():
    L = _tiny(out_features=6, in_features=40, k=64, k_res=16)
    L.codebook[:] = np.round(L.codebook.astype(np.float64) * 2 ** 12) / 2 ** 12     # coarse grid: all sums exact in fp64
    L.codebook_res[:] = np.round(L.codebook_res.astype(np.float64) * 2 ** 12) / 2 ** 12
    L.scale[:] = 1
    L.bias[:] = np.float16(0.25)
    rng = np.random.default_rng(2)
    x1 = rng.integers(-8, 9, (1, 40)).astype(np.float16)
    x2 = rng.integers(-8, 9, (1, 40)).astype(np.float16)
    y = oracle.matmul(L, np.concatenate([x1, x2, 3 * x1 - 2 * x2]))
    assert np.array_equal(y[2], 3 * y[0] - 2 * y[1])


def test_tokens_are_independent_and_row_subset_matches():
    L = _tiny(out_features=9, in_features=50, k_res=16)
    x = s.make_activations(200, L, 4)
    y = oracle.matmul(L, x)
    for t in range(4):
        assert np.array_equal(oracle.matmul(L, x[t:t + 1])[0], y[t])
    rows = [8, 0, 3, 3]
    assert np.array_equal(oracle.matmul(L, x, rows=rows), y[:, rows])
    assert np.array_equal(oracle.matmul(L, x, n_threads=1), oracle.matmul(L, x, n_threads=5))
    assert oracle.matmul(L, x[:0]).shape == (0, 9)


def test_output_rms_matches_closed_form_on_7b_layer():
    # y = sum_c (s*d + b) x_c with independent d ~ N(0, 0.02), s ~ U(0.5, 1.5), b ~ N(0, 0.01), x ~ N(0, 1):
    # E[y^2] = in * (E[s^2] * 0.02^2 + 0.01^2), E[s^2] = 1 + 1/12.
    _, L = next(s.config_layers(1))
    x = s.make_activations(1, L, 1)
    rows = np.arange(0, L.out_features, 4)
    y = oracle.matmul(L, x, rows=rows)
    closed = np.sqrt(4096 * ((1 + 1 / 12) * 0.02 ** 2 + 0.01 ** 2))
    assert abs(np.sqrt((y ** 2).mean()) / closed - 1) < 0.05


# ---------------------------------------------------------------- bit accounting (paper's printed values)
def _golden_accounting():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_accounting.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, value, tol, _ = [f.strip() for f in line.split("|")]
        out[name] = (float(value), float(tol))
    return out


def test_accounting_reproduces_paper_values():
    g = _golden_accounting()

    def close(name, got):
        want, tol = g[name]
        assert abs(got - want) <= tol + 1e-12, (name, got, want)
    n = 4096 * 4096
    close("compression_ratio_4096x4096_v8_k256", accounting.compression_ratio(n, 8, 256))
    close("equivalent_bitwidth_4096x4096_v8_k256", accounting.equivalent_bitwidth(n, 8, 256))
    close("index_bits_v6_k4096", accounting.index_bits_per_weight(4096, 6))
    close("index_bits_v8_k65536", accounting.index_bits_per_weight(65536, 8))
    close("index_bits_v4_k4096", accounting.index_bits_per_weight(4096, 4))
    block_13b = 4 * 5120 * 5120 + 3 * 5120 * 13824        # LLaMA-2-13B: 4 attention + 3 FFN linears per block
    extra = accounting.equivalent_bitwidth(block_13b, 8, 65536, n_codebooks=7) - accounting.index_bits_per_weight(65536, 8)
    close("codebook_overhead_bits_13b_v8_k65536", extra)


def test_algorithmic_bytes_agree_with_layer_sizes():
    for cfg, batch in [(0, 1), (1, 1), (4, 512)]:
        c = s.CONFIGS[cfg]
        name, out_f, in_f = c["layers"][0]
        _, L = next(s.config_layers(cfg))
        assert accounting.layer_algorithmic_bytes(out_f, in_f, c["v"], c["k"], batch=batch) == L.algorithmic_bytes(batch)
    assert accounting.layer_algorithmic_bytes(8192, 28672, 6, 4096, 256, 288, 4, 4096, batch=1) == 97967104
    assert accounting.layer_algorithmic_bytes(11008, 4096, 6, 4096) == 11401088
