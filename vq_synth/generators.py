"""Counter-based random streams (SplitMix64) for the synthetic layers.

Element i of the stream with seed s is mix(s + (i+1)*GAMMA): every element is
a pure function of (seed, i), so any slice can be produced independently and
any language reproduces the same numbers.
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_BASE_SEED = 0x5650545100

# tensor ids inside one layer
T_CODEBOOK, T_CODEBOOK_RES, T_CODEBOOK_OUT = 0, 1, 2
T_IDX, T_IDX_RES, T_IDX_OUT = 3, 4, 5
T_SCALE, T_BIAS, T_ACT, T_PERM, T_HESSIAN, T_WEIGHT = 6, 7, 8, 9, 10, 11


def tensor_seed(config: int, tensor_id: int, layer_ordinal: int = 0, batch_or_tokens: int = 0) -> int:
    """Seed of one tensor: base + 16*config + tensor id (+256*layer, +4096*batch for activations)."""
    return (_BASE_SEED + 16 * config + tensor_id + 256 * layer_ordinal + 4096 * batch_or_tokens) & 0xFFFFFFFFFFFFFFFF


def splitmix64(seed: int, count: int, start: int = 0) -> np.ndarray:
    """Elements [start, start+count) of the SplitMix64 stream of `seed`, as uint64."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, count: int, start: int = 0) -> np.ndarray:
    """Uniform doubles in [0, 1): top 53 bits of each stream element."""
    return (splitmix64(seed, count, start) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53


def normal(seed: int, count: int, sigma: float) -> np.ndarray:
    """Box-Muller (cosine branch) in fp64: element i uses stream elements 2i and 2i+1."""
    z = splitmix64(seed, 2 * count)
    u1 = ((z[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53   # (0, 1]
    u2 = (z[1::2] >> np.uint64(11)).astype(np.float64) * 2.0 ** -53            # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2) * sigma


def to_fp16(a: np.ndarray) -> np.ndarray:
    """Round to IEEE binary16 (numpy rounds to nearest even)."""
    return np.asarray(a, dtype=np.float64).astype(np.float16)


def random_indices(seed: int, rows: int, per_row: int, k: int) -> np.ndarray:
    """Uniform indices in [0, k): stream element (row*per_row + p) mod k, as int32 [rows][per_row]."""
    out = np.empty((rows, per_row), dtype=np.int32)
    chunk = max(1, (1 << 22) // max(per_row, 1))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        z = splitmix64(seed, (r1 - r0) * per_row, start=r0 * per_row)
        out[r0:r1] = (z % np.uint64(k)).astype(np.int32).reshape(r1 - r0, per_row)
    return out


def permutation(seed: int, n: int) -> np.ndarray:
    """A permutation of 0 .. n-1 as int32: the order that sorts the first n stream elements (ties by position)."""
    return np.argsort(splitmix64(seed, n), kind="stable").astype(np.int32)
