"""Python binding of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the GPU library never does.  All arrays are host numpy arrays.
"""
import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvq_oracle.so")
_SRC = os.path.join(_HERE, "vq_oracle.cpp")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (a second of CPU work)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "vq_oracle.h")))
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < newest:
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
                               "-Wall", "-Wextra", _SRC, "-o", _LIB_PATH, "-lpthread"])
    return _LIB_PATH


class _Layer(ctypes.Structure):
    _fields_ = [
        ("out_features", ctypes.c_int32), ("in_features", ctypes.c_int32),
        ("v", ctypes.c_int32), ("k", ctypes.c_int32), ("k_res", ctypes.c_int32),
        ("n_outlier_cols", ctypes.c_int32), ("v_out", ctypes.c_int32), ("k_out", ctypes.c_int32),
        ("codebook", ctypes.c_void_p), ("codebook_res", ctypes.c_void_p), ("codebook_out", ctypes.c_void_p),
        ("idx", ctypes.c_void_p), ("idx_row_stride", ctypes.c_int64),
        ("idx_res", ctypes.c_void_p), ("idx_res_row_stride", ctypes.c_int64),
        ("idx_out", ctypes.c_void_p), ("idx_out_row_stride", ctypes.c_int64),
        ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p),
        ("group_vectors", ctypes.c_int32), ("orientation", ctypes.c_int32),
        ("col_perm", ctypes.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.vq_oracle_half_to_float.restype = ctypes.c_float
        L.vq_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        L.vq_oracle_float_to_half.restype = ctypes.c_uint16
        L.vq_oracle_float_to_half.argtypes = [ctypes.c_float]
        L.vq_oracle_index_bits.argtypes = [ctypes.c_int32]
        L.vq_oracle_unpack_row.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_void_p]
        L.vq_oracle_dequant.argtypes = [ctypes.POINTER(_Layer), ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
        L.vq_oracle_assign.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int]
        L.vq_oracle_assign_down.argtypes = L.vq_oracle_assign.argtypes
        L.vq_oracle_matmul.argtypes = [ctypes.POINTER(_Layer), ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                       ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int]
        L.vq_oracle_quantize_columns.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                                 ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = L
    return _lib


def default_threads() -> int:
    return max(1, len(os.sched_getaffinity(0)))


def _ptr(a):
    return a.ctypes.data if a is not None else None


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def _describe(layer):
    """ctypes layer record + the arrays it points into (kept alive by the caller)."""
    keep = dict(
        codebook=_c(layer.codebook, np.float16), codebook_res=_c(layer.codebook_res, np.float16),
        codebook_out=_c(layer.codebook_out, np.float16), idx=_c(layer.idx, np.uint8),
        idx_res=_c(layer.idx_res, np.uint8), idx_out=_c(layer.idx_out, np.uint8),
        scale=_c(layer.scale, np.float16), bias=_c(layer.bias, np.float16),
        col_perm=_c(getattr(layer, "col_perm", None), np.int32))

    def stride(a):
        return a.shape[1] if a is not None else 0
    d = _Layer(layer.out_features, layer.in_features, layer.v, layer.k, layer.k_res,
               layer.n_outlier_cols, layer.v_out, layer.k_out,
               _ptr(keep["codebook"]), _ptr(keep["codebook_res"]), _ptr(keep["codebook_out"]),
               _ptr(keep["idx"]), stride(keep["idx"]), _ptr(keep["idx_res"]), stride(keep["idx_res"]),
               _ptr(keep["idx_out"]), stride(keep["idx_out"]), _ptr(keep["scale"]), _ptr(keep["bias"]),
               int(getattr(layer, "group_vectors", 0)), int(getattr(layer, "orientation", 0)), _ptr(keep["col_perm"]))
    return d, keep


class OracleError(RuntimeError):
    pass


def half_to_float(bits: int) -> float:
    return lib().vq_oracle_half_to_float(int(bits))


def float_to_half(value) -> int:
    return lib().vq_oracle_float_to_half(ctypes.c_float(value))


def index_bits(k: int) -> int:
    return lib().vq_oracle_index_bits(int(k))


def unpack_row(row: np.ndarray, bits: int, count: int) -> np.ndarray:
    row = _c(row, np.uint8)
    out = np.empty(count, dtype=np.int32)
    rc = lib().vq_oracle_unpack_row(_ptr(row), bits, count, _ptr(out))
    if rc:
        raise OracleError("unpack_row failed: %d" % rc)
    return out


def dequant(layer, ldw: int | None = None, n_threads: int | None = None) -> np.ndarray:
    """Restored weights, fp16 [out][ldw]; columns >= in_features are left zero."""
    d, keep = _describe(layer)
    ldw = layer.in_features if ldw is None else ldw
    W = np.zeros((layer.out_features, ldw), dtype=np.float16)
    rc = lib().vq_oracle_dequant(ctypes.byref(d), _ptr(W), ldw, n_threads or default_threads())
    if rc:
        raise OracleError("dequant failed: %d" % rc)
    return W


def matmul(layer, x: np.ndarray, rows=None, n_threads: int | None = None) -> np.ndarray:
    """fp64 [tokens][out] (or [tokens][len(rows)]): restored weights times fp16 activations x [tokens][in]."""
    d, keep = _describe(layer)
    x = _c(x, np.float16)
    assert x.ndim == 2 and x.shape[1] >= layer.in_features
    tokens = x.shape[0]
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    n_rows = layer.out_features if rows_a is None else len(rows_a)
    y = np.zeros((tokens, n_rows), dtype=np.float64)
    rc = lib().vq_oracle_matmul(ctypes.byref(d), _ptr(x), x.shape[1], tokens, _ptr(rows_a), n_rows,
                                _ptr(y), n_rows, n_threads or default_threads())
    if rc:
        raise OracleError("matmul failed: %d" % rc)
    return y


def assign(W: np.ndarray, codebook: np.ndarray, base: np.ndarray | None = None, cols: int | None = None,
           n_threads: int | None = None, orientation: int = 0) -> np.ndarray:
    """Index of the nearest centroid (fp16 [k][v]) of every length-v vector of fp16 W [rows][>= cols]; with `base` (same
    shape), of W - base.  orientation 0: vectors along the rows, int32 [rows][ceil(cols / v)]; orientation 1: vectors
    down the columns, int32 [ceil(rows / v)][cols]."""
    W = _c(W, np.float16)
    codebook = _c(codebook, np.float16)
    base = _c(base, np.float16)
    assert W.ndim == 2 and codebook.ndim == 2 and (base is None or base.shape == W.shape)
    cols = W.shape[1] if cols is None else cols
    k, v = codebook.shape
    if orientation:
        out = np.empty((-(-W.shape[0] // v), cols), dtype=np.int32)
        fn = lib().vq_oracle_assign_down
    else:
        out = np.empty((W.shape[0], -(-cols // v)), dtype=np.int32)
        fn = lib().vq_oracle_assign
    rc = fn(_ptr(W), _ptr(base), W.shape[1], W.shape[0], cols, _ptr(codebook), v, k, _ptr(out), n_threads or default_threads())
    if rc:
        raise OracleError("assign failed: %d" % rc)
    return out


def quantize_columns(W, Hinv, codebook, codebook_res=None, block=128, given=None):
    """Algorithm 1's column loop.  W: [M][N], Hinv: [N][N] (any float dtype, widened to fp64); codebooks fp16 [k][v].
    given: (idx, idx_res or None) to replay somebody else's choices instead of taking the nearest centroids.
    Returns dict(idx, idx_res, What, T): int32 [ceil(M/v)][N] indices, fp64 [M][N] quantized weights and the columns as
    they stood when they were quantized."""
    W = np.ascontiguousarray(W, dtype=np.float64)
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    M, N = W.shape
    assert Hinv.shape == (N, N)
    codebook = _c(codebook, np.float16)
    codebook_res = _c(codebook_res, np.float16)
    k, v = codebook.shape
    k_res = 0 if codebook_res is None else codebook_res.shape[0]
    S = -(-M // v)
    g_idx = g_res = None
    if given is not None:
        g_idx = np.ascontiguousarray(given[0], dtype=np.int32)
        g_res = None if given[1] is None else np.ascontiguousarray(given[1], dtype=np.int32)
        assert g_idx.shape == (S, N) and (g_res is None) == (k_res == 0)
    idx = np.zeros((S, N), dtype=np.int32)
    idx_res = np.zeros((S, N), dtype=np.int32) if k_res else None
    What = np.zeros((M, N), dtype=np.float64)
    T = np.zeros((M, N), dtype=np.float64)
    rc = lib().vq_oracle_quantize_columns(_ptr(W), _ptr(Hinv), M, N, _ptr(codebook), v, k, _ptr(codebook_res), k_res, int(block),
                                          _ptr(g_idx), _ptr(g_res), _ptr(idx), _ptr(idx_res), _ptr(What), _ptr(T))
    if rc:
        raise OracleError("quantize_columns failed: %d" % rc)
    return dict(idx=idx, idx_res=idx_res, What=What, T=T)


# decode GEMV and prefill GEMM are the same definition at different token counts
gemv = matmul
gemm = matmul
