"""Bit accounting of a vector-quantized layer -- TEST INFRASTRUCTURE ONLY.

Restates the paper's compression-ratio formulas (Sec. 2.2 worked example;
App. "Compression Ratio Calculation"): index bits per weight are log2(k)/v per
codebook stage, codebook bits are 16 per stored table element, and

    compression ratio   = original bits / (codebook bits + index bits)
    equivalent bitwidth = original bit width / compression ratio.

The appendix prints log2(k0/v0) for the outlier term; it is read as
log2(k0)/v0, which is what the worked examples (8/8 = 1 bit, 12/6 = 2 bits,
12/4 = 3 bits) require.
"""
import math


def index_bits_per_weight(k: int, v: int) -> float:
    return math.log2(k) / v


def codebook_bits(v1: int, k1: int, k2: int = 0, v0: int = 0, k0: int = 0) -> int:
    return (v0 * k0 + v1 * (k1 + k2)) * 16


def index_bits_total(n_weights: int, v1: int, k1: int, k2: int = 0,
                     outlier_fraction: float = 0.0, v0: int = 0, k0: int = 0) -> float:
    main = index_bits_per_weight(k1, v1) + (index_bits_per_weight(k2, v1) if k2 else 0.0)
    out = index_bits_per_weight(k0, v0) if outlier_fraction else 0.0
    return n_weights * outlier_fraction * out + n_weights * (1.0 - outlier_fraction) * main


def compression_ratio(n_weights: int, v1: int, k1: int, k2: int = 0, outlier_fraction: float = 0.0,
                      v0: int = 0, k0: int = 0, original_bits: int = 16, n_codebooks: int = 1) -> float:
    stored = n_codebooks * codebook_bits(v1, k1, k2, v0 if outlier_fraction else 0, k0 if outlier_fraction else 0) \
        + index_bits_total(n_weights, v1, k1, k2, outlier_fraction, v0, k0)
    return original_bits * n_weights / stored


def equivalent_bitwidth(*args, original_bits: int = 16, **kw) -> float:
    return original_bits / compression_ratio(*args, original_bits=original_bits, **kw)


def layer_algorithmic_bytes(out_features: int, in_features: int, v: int, k: int, k_res: int = 0,
                            n_outlier_cols: int = 0, v_out: int = 0, k_out: int = 0,
                            batch: int = 1, scale: bool = True, bias: bool = True) -> int:
    """Bytes one multiply must move: unpadded index streams + tables + scale/bias + activations + outputs."""
    def b(kk):
        return max(1, (kk - 1).bit_length())
    P = -(-(in_features - n_outlier_cols) // v)
    Q = n_outlier_cols // v_out if n_outlier_cols else 0
    bits = out_features * (P * (b(k) + (b(k_res) if k_res else 0)) + (Q * b(k_out) if Q else 0))
    tables = 2 * (k * v + k_res * v + (k_out * v_out if Q else 0))
    return bits // 8 + tables + 2 * out_features * (int(scale) + int(bias)) + 2 * batch * (in_features + out_features)
