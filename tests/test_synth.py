"""The seeded input generators and the encode-side packer (CPU only)."""
import os
import numpy as np
import pytest

import vq_synth as s

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vector():
    # Reference outputs of SplitMix64 for seed 1234567 (the generator's widely reproduced test vector).
    z = s.splitmix64(1234567, 5)
    assert [int(v) for v in z] == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                                   4593380528125082431, 16408922859458223821]


def test_splitmix64_is_counter_based():
    a = s.splitmix64(99, 100)
    b = s.splitmix64(99, 40, start=60)
    assert np.array_equal(a[60:], b)


def test_uniform_and_normal_moments():
    u = s.uniform01(7, 200000)
    assert 0.0 <= u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5e-3 and abs(u.var() - 1 / 12) < 2e-3
    n = s.normal(8, 200000, 0.02)
    assert abs(n.mean()) < 2e-4 and abs(n.std() - 0.02) < 2e-4


def test_seeds_distinct():
    seeds = {s.tensor_seed(c, t, l, b) for c in range(5) for t in range(9) for l in range(7) for b in (0, 1, 4)}
    assert len(seeds) == 5 * 9 * 7 * 3


def _golden_packing():
    for line in open(os.path.join(GOLDEN, "packing_bytes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        bits, idx, data = [f.strip() for f in line.split("|")]
        yield int(bits), [int(t, 0) for t in idx.split()], bytes(int(t, 16) for t in data.split())


@pytest.mark.parametrize("bits,idx,data", list(_golden_packing()))
def test_packer_matches_handwritten_bytes(bits, idx, data):
    p = s.pack_indices(np.array([idx]), bits)
    assert p.shape[1] % 16 == 0
    assert bytes(p[0, : len(data)]) == data
    assert not p[0, len(data):].any()          # pad bits are zero


def test_packer_plain_widths():
    rng = np.random.default_rng(0)
    i8 = rng.integers(0, 256, (3, 37))
    assert np.array_equal(s.pack_indices(i8, 8)[:, :37], i8.astype(np.uint8))
    i16 = rng.integers(0, 65536, (3, 21))
    assert np.array_equal(s.pack_indices(i16, 16)[:, :42].copy().view("<u2"), i16.astype(np.uint16))


def test_packer_rejects_wide_index():
    with pytest.raises(ValueError):
        s.pack_indices(np.array([[16]]), 4)


def test_row_stride_values():
    # strides of the benchmark layers: 683 x 12 bit, 1835 x 12 bit, 4731 x 12 / 8 bit, 72 x 12 bit, 1024 x 16 bit
    assert [s.row_stride_bytes(p, b) for p, b in [(683, 12), (1835, 12), (4731, 12), (4731, 8), (72, 12), (1024, 16)]] \
        == [1040, 2768, 7104, 4736, 112, 2048]


def test_layer_shapes_and_bytes():
    _, L = next(s.config_layers(0))
    assert L.vectors_per_row == 64 and L.idx.shape == (256, 64) and L.algorithmic_bytes(1) == 21760
    L3 = s.make_layer(3, "slice", 4, 28672, 6, 4096, 256, 288, 4, 4096)
    assert L3.vectors_per_row == 4731 and L3.outlier_vectors_per_row == 72
    assert L3.idx.shape[1] == 7104 and L3.idx_res.shape[1] == 4736 and L3.idx_out.shape[1] == 112
