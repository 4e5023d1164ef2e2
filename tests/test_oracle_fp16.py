"""Pins for the oracle's own binary16 conversions (CPU only)."""
import numpy as np

import oracle


def test_half_to_float_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_float_to_half_roundtrip_identity():
    bits = np.arange(65536, dtype=np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    for b, x in zip(bits, f):
        if np.isnan(x):
            continue
        assert oracle.float_to_half(float(x)) == int(b)


def test_float_to_half_ties_go_to_even():
    # the midpoint of two adjacent non-negative halfs is exact in binary32; it must round to the even pattern
    for b in range(0, 0x7BFF):
        lo = np.array([b], dtype=np.uint16).view(np.float16).astype(np.float64)[0]
        hi = np.array([b + 1], dtype=np.uint16).view(np.float16).astype(np.float64)[0]
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2
        want = b if b % 2 == 0 else b + 1
        assert oracle.float_to_half(float(mid)) == want
        assert oracle.float_to_half(-float(mid)) == want | 0x8000
        # a hair above / below the tie goes to the nearer neighbour
        assert oracle.float_to_half(float(np.nextafter(mid, np.float32(np.inf)))) == b + 1
        assert oracle.float_to_half(float(np.nextafter(mid, np.float32(-np.inf)))) == b


def test_float_to_half_overflow_and_specials():
    assert oracle.float_to_half(65504.0) == 0x7BFF
    assert oracle.float_to_half(65519.996) == 0x7BFF
    assert oracle.float_to_half(65520.0) == 0x7C00
    assert oracle.float_to_half(-1e30) == 0xFC00
    assert oracle.float_to_half(float("inf")) == 0x7C00
    assert oracle.float_to_half(0.0) == 0 and oracle.float_to_half(-0.0) == 0x8000
    assert oracle.float_to_half(2.0 ** -25) == 0          # tie between 0 and the smallest subnormal -> even (0)
    assert oracle.float_to_half(2.0 ** -24) == 1
    assert (oracle.float_to_half(float("nan")) & 0x7C00) == 0x7C00 and (oracle.float_to_half(float("nan")) & 0x3FF)


def test_float_to_half_random_matches_numpy():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-5, 20000), rng.normal(0, 3e4, 5000)]).astype(np.float32)
    want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
