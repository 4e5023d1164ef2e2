"""The synthetic layers: five benchmark configurations plus free-form test layers.

Shapes follow LLaMA-2 7B / 70B linear layers and the (v, k) settings the
method is evaluated with (v=6/k=4096, residual k=4096 or 256, outlier columns
with v=4/k=4096, v=8/k=65536).  Real checkpoints are not available, so table
entries are Gaussian and indices are uniform (the worst case for lookup
locality).  sigma means standard deviation throughout.
"""
from dataclasses import dataclass, field
import numpy as np

from . import generators as g
from .pack import pack_indices, row_stride_bytes, index_bits

SIGMA_MAIN, SIGMA_RES, SIGMA_OUT, SIGMA_BIAS = 0.02, 0.005, 0.1, 0.01


@dataclass
class VQLayer:
    """One stored layer: tables, packed index streams, scale/bias, and the unpacked indices (tests only)."""
    name: str
    out_features: int
    in_features: int
    v: int
    k: int
    k_res: int = 0
    n_outlier_cols: int = 0
    v_out: int = 0
    k_out: int = 0
    group_vectors: int = 0               # > 0: every range of this many vectors of a row has tables of its own
    orientation: int = 0                 # 0: vectors along the input dimension of a row; 1: down the output dimension
    codebook: np.ndarray = None          # fp16 [n_groups * k][v]: the groups' tables one after the other
    codebook_res: np.ndarray = None      # fp16 [n_groups * k_res][v] or None
    codebook_out: np.ndarray = None      # fp16 [k_out][v_out] or None
    idx: np.ndarray = None               # uint8 [out][stride]
    idx_res: np.ndarray = None
    idx_out: np.ndarray = None
    scale: np.ndarray = None             # fp16 [out] or None
    bias: np.ndarray = None              # fp16 [out] or None
    raw_idx: np.ndarray = None           # int32 [out][P]   (what was packed)
    raw_idx_res: np.ndarray = None
    raw_idx_out: np.ndarray = None
    col_perm: np.ndarray = None          # int32 [in_features] or None: stored column c is column col_perm[c] of the layer

    # An index stream holds `vectors_per_row` indices.  Orientation 0: one stream per output row, a vector covers v
    # consecutive input columns.  Orientation 1 (the paper's: Sec. 3.1, a column is a stack of centroids): one stream per v
    # consecutive output rows, one index per input column.
    @property
    def vectors_per_row(self) -> int:
        main = self.in_features - self.n_outlier_cols
        return main if self.orientation else -(-main // self.v)

    @property
    def outlier_vectors_per_row(self) -> int:
        if not self.n_outlier_cols:
            return 0
        return self.n_outlier_cols if self.orientation else self.n_outlier_cols // self.v_out

    @property
    def streams(self) -> int:
        return -(-self.out_features // self.v) if self.orientation else self.out_features

    @property
    def outlier_streams(self) -> int:
        if not self.n_outlier_cols:
            return 0
        return -(-self.out_features // self.v_out) if self.orientation else self.out_features

    @property
    def n_groups(self) -> int:
        return -(-self.vectors_per_row // self.group_vectors) if self.group_vectors > 0 else 1

    @property
    def bits(self) -> int:
        return index_bits(self.k)

    @property
    def bits_res(self) -> int:
        return index_bits(self.k_res) if self.k_res else 0

    @property
    def bits_out(self) -> int:
        return index_bits(self.k_out) if self.n_outlier_cols else 0

    def algorithmic_bytes(self, batch: int) -> int:
        """Bytes one call must move: unpadded index bits, tables, scale/bias, activations in, outputs out."""
        P, Q, M = self.vectors_per_row, self.outlier_vectors_per_row, self.out_features
        idx_bits = self.streams * P * (self.bits + self.bits_res) + self.outlier_streams * Q * self.bits_out
        tables = 2 * (self.n_groups * (self.k * self.v + self.k_res * self.v) + self.k_out * self.v_out)
        sb = 2 * M * ((self.scale is not None) + (self.bias is not None))
        return idx_bits // 8 + tables + sb + 2 * batch * self.in_features + 2 * batch * M


def make_layer(config: int, name: str, out_features: int, in_features: int, v: int, k: int,
               k_res: int = 0, n_outlier_cols: int = 0, v_out: int = 0, k_out: int = 0,
               layer_ordinal: int = 0, with_scale: bool = True, with_bias: bool = True,
               extra_stride: int = 0, group_vectors: int = 0, orientation: int = 0, permute: bool = False) -> VQLayer:
    """Build one layer from the seeded streams.  `extra_stride` adds 16-byte units of row padding; with
    `group_vectors` every range of that many vectors gets main (and residual) tables of its own, all drawn from
    one stream, group after group; `permute` stores the columns in a seeded random order (the outlier columns
    are then scattered over the layer, as columns picked by a Hessian's diagonal are)."""
    def seed(t):
        return g.tensor_seed(config, t, layer_ordinal)

    L = VQLayer(name, out_features, in_features, v, k, k_res, n_outlier_cols, v_out, k_out, group_vectors, orientation)
    P, Q = L.vectors_per_row, L.outlier_vectors_per_row
    n_groups = L.n_groups
    L.codebook = g.to_fp16(g.normal(seed(g.T_CODEBOOK), n_groups * k * v, SIGMA_MAIN)).reshape(n_groups * k, v)
    L.raw_idx = g.random_indices(seed(g.T_IDX), L.streams, P, k)
    L.idx = pack_indices(L.raw_idx, L.bits, row_stride_bytes(P, L.bits) + 16 * extra_stride)
    if k_res:
        L.codebook_res = g.to_fp16(g.normal(seed(g.T_CODEBOOK_RES), n_groups * k_res * v, SIGMA_RES)).reshape(n_groups * k_res, v)
        L.raw_idx_res = g.random_indices(seed(g.T_IDX_RES), L.streams, P, k_res)
        L.idx_res = pack_indices(L.raw_idx_res, L.bits_res, row_stride_bytes(P, L.bits_res) + 16 * extra_stride)
    if n_outlier_cols:
        assert orientation or n_outlier_cols % v_out == 0
        L.codebook_out = g.to_fp16(g.normal(seed(g.T_CODEBOOK_OUT), k_out * v_out, SIGMA_OUT)).reshape(k_out, v_out)
        L.raw_idx_out = g.random_indices(seed(g.T_IDX_OUT), L.outlier_streams, Q, k_out)
        L.idx_out = pack_indices(L.raw_idx_out, L.bits_out, row_stride_bytes(Q, L.bits_out) + 16 * extra_stride)
    if permute:
        L.col_perm = g.permutation(seed(g.T_PERM), in_features)
    if with_scale:
        L.scale = g.to_fp16(0.5 + g.uniform01(seed(g.T_SCALE), out_features))
    if with_bias:
        L.bias = g.to_fp16(g.normal(seed(g.T_BIAS), out_features, SIGMA_BIAS))
    return L


def make_activations(config: int, layer: VQLayer, rows: int, layer_ordinal: int = 0,
                     outlier_gain: float = 1.0) -> np.ndarray:
    """fp16 [rows][in_features] ~ N(0,1); the outlier columns are multiplied by `outlier_gain`."""
    s = g.tensor_seed(config, g.T_ACT, layer_ordinal, rows)
    x = g.normal(s, rows * layer.in_features, 1.0).reshape(rows, layer.in_features)
    if layer.n_outlier_cols and outlier_gain != 1.0:
        cols = np.arange(layer.n_outlier_cols) if layer.col_perm is None else layer.col_perm[: layer.n_outlier_cols]
        x[:, cols] *= outlier_gain
    return g.to_fp16(x)


# name, out, in, per-config extras
_L7B = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
        ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]

CONFIGS = {
    0: dict(layers=[("tiny", 256, 384)], v=6, k=256, rows=[1]),
    1: dict(layers=[("up", 11008, 4096)], v=6, k=4096, rows=[1]),
    2: dict(layers=_L7B, v=6, k=4096, k_res=4096, rows=[1, 4, 16]),
    3: dict(layers=[("down70b", 8192, 28672)], v=6, k=4096, k_res=256,
            n_outlier_cols=288, v_out=4, k_out=4096, rows=[1, 8], outlier_gain=10.0),
    4: dict(layers=[("prefill", 8192, 8192)], v=8, k=65536, rows=[512, 1024, 2048]),
}


def config_layers(config: int, only: str | None = None):
    """Yield (layer_ordinal, VQLayer) for a benchmark configuration (optionally one named layer)."""
    c = CONFIGS[config]
    for ordinal, (name, out_f, in_f) in enumerate(c["layers"]):
        if only is not None and name != only:
            continue
        yield ordinal, make_layer(config, name, out_f, in_f, c["v"], c["k"], c.get("k_res", 0),
                                  c.get("n_outlier_cols", 0), c.get("v_out", 0), c.get("k_out", 0),
                                  layer_ordinal=ordinal)


def make_hessian(config: int, n: int, samples: int = 0, damp: float = 0.01, mix: float = 0.6) -> np.ndarray:
    """A synthetic layer Hessian, fp64 [n][n], symmetric positive definite: X^T X / samples of `samples` seeded Gaussian
    activation rows (default 2 n) whose neighbouring channels are correlated (channel c = mix * channel c-1 + noise, with a
    per-channel gain that makes a few channels much larger than the rest, as calibration activations are), plus `damp`
    times the mean diagonal on the diagonal (the usual damping)."""
    samples = samples or 2 * n
    z = g.normal(g.tensor_seed(config, g.T_HESSIAN), samples * n, 1.0).reshape(samples, n)
    for c in range(1, n):
        z[:, c] += mix * z[:, c - 1]
    gain = 1.0 + 9.0 * (g.uniform01(g.tensor_seed(config, g.T_HESSIAN, 1), n) > 0.97)
    z *= gain
    H = z.T @ z / samples
    H += damp * np.mean(np.diag(H)) * np.eye(n)
    return H


def make_weights(config: int, rows: int, cols: int, sigma: float = SIGMA_MAIN) -> np.ndarray:
    """Seeded Gaussian weights, fp64 [rows][cols] (values of fp16 numbers)."""
    return g.to_fp16(g.normal(g.tensor_seed(config, g.T_WEIGHT), rows * cols, sigma)).astype(np.float64).reshape(rows, cols)
