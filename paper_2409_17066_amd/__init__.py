"""Thin Python binding of libvq.so, the gfx950 vector-quantized linear layer (argument marshalling only).

Every step of the path (index unpack, codebook lookup, residual sum, outlier columns, scale/bias,
GEMV / GEMM) runs in the HIP kernels behind the C ABI of include/vq.h.  PyTorch is used for device
memory and streams only.  There is no CPU fallback: a missing library raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvq.so")

VQ_OK, VQ_ERR_NULL, VQ_ERR_SHAPE, VQ_ERR_ALIGNMENT, VQ_ERR_UNSUPPORTED, VQ_ERR_HIP, VQ_ERR_WORKSPACE = 0, -1, -2, -3, -4, -5, -6


class vq_layer_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
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


class VQError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, vq_status_string(status), status))


_lib = None


def load():
    """Load libvq.so (build it first with build.py or __graft_entry__.build()).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libvq.so is not built: run `python -m paper_2409_17066_amd.build` (needs hipcc)")
    try:
        import torch  # noqa: F401  -- loads the HIP runtime this process will share with the library
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(vq_layer_desc)
    L.vq_validate.argtypes = [P]
    L.vq_dequant.argtypes = [P, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    L.vq_gemv.argtypes = [P, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    L.vq_gemv_workspace_bytes.argtypes = [P, ctypes.c_int32]
    L.vq_gemv_workspace_bytes.restype = ctypes.c_size_t
    L.vq_gemv_with_workspace.argtypes = [P, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.vq_gemv_static_workspace.argtypes = L.vq_gemv.argtypes
    L.vq_gemv_multi.argtypes = [ctypes.POINTER(P), ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p]
    L.vq_assign.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                            ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    L.vq_assign_down.argtypes = L.vq_assign.argtypes
    L.vq_gemm.argtypes = [P, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                          ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.vq_gemm_workspace_bytes.argtypes = [P, ctypes.c_int32]
    L.vq_gemm_workspace_bytes.restype = ctypes.c_size_t
    L.vq_gemm_fast_workspace_bytes.argtypes = [P, ctypes.c_int32]
    L.vq_gemm_fast_workspace_bytes.restype = ctypes.c_size_t
    L.vq_quantize_columns_workspace_bytes.argtypes = [ctypes.c_int32] * 4
    L.vq_quantize_columns_workspace_bytes.restype = ctypes.c_size_t
    L.vq_quantize_columns.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                      ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.vq_quantize_columns.restype = ctypes.c_int
    L.vq_status_string.argtypes = [ctypes.c_int]
    L.vq_status_string.restype = ctypes.c_char_p
    L.vq_version.restype = ctypes.c_int
    for f in (L.vq_validate, L.vq_dequant, L.vq_gemv, L.vq_gemv_with_workspace, L.vq_gemv_static_workspace, L.vq_gemv_multi, L.vq_gemm, L.vq_assign, L.vq_assign_down):
        f.restype = ctypes.c_int
    _lib = L
    return L


EXPORTED = ["vq_validate", "vq_dequant", "vq_gemv", "vq_gemv_workspace_bytes", "vq_gemv_with_workspace", "vq_gemv_static_workspace", "vq_gemv_multi", "vq_gemm", "vq_gemm_workspace_bytes", "vq_gemm_fast_workspace_bytes",
            "vq_assign", "vq_assign_down", "vq_quantize_columns", "vq_quantize_columns_workspace_bytes", "vq_status_string", "vq_version"]


# ---- the C entry points, same names, raw pointers (ints) and sizes ---------------------------------------
def vq_validate(desc):
    return load().vq_validate(ctypes.byref(desc) if desc is not None else None)


def vq_dequant(desc, W_ptr, ldw, stream=None):
    return load().vq_dequant(ctypes.byref(desc) if desc is not None else None, W_ptr, ldw, stream)


def vq_gemv(desc, x_ptr, ldx, batch, y_ptr, ldy, stream=None):
    return load().vq_gemv(ctypes.byref(desc) if desc is not None else None, x_ptr, ldx, batch, y_ptr, ldy, stream)


def vq_gemv_workspace_bytes(desc, batch):
    return load().vq_gemv_workspace_bytes(ctypes.byref(desc), batch)


def vq_gemv_with_workspace(desc, x_ptr, ldx, batch, y_ptr, ldy, workspace_ptr=None, workspace_bytes=0, stream=None):
    return load().vq_gemv_with_workspace(ctypes.byref(desc) if desc is not None else None, x_ptr, ldx, batch, y_ptr, ldy,
                                         workspace_ptr, workspace_bytes, stream)


def vq_gemv_static_workspace(desc, x_ptr, ldx, batch, y_ptr, ldy, stream=None):
    return load().vq_gemv_static_workspace(ctypes.byref(desc) if desc is not None else None, x_ptr, ldx, batch, y_ptr, ldy, stream)


VQ_GEMV_STATIC_WORKSPACE_BYTES = 16 << 20


def vq_gemv_multi(descs, x_ptr, ldx, batch, y_ptrs, ldys, stream=None):
    """descs: sequence of vq_layer_desc; y_ptrs, ldys: sequences of device pointers (ints) and leading dimensions."""
    n = len(descs)
    P = ctypes.POINTER(vq_layer_desc)
    d = (P * n)(*[ctypes.pointer(x) for x in descs]) if descs is not None else None
    ys = (ctypes.c_void_p * n)(*y_ptrs) if y_ptrs is not None else None
    ld = (ctypes.c_int64 * n)(*ldys) if ldys is not None else None
    return load().vq_gemv_multi(d, n, x_ptr, ldx, batch, ys, ld, stream)


def vq_gemm(desc, X_ptr, ldx, tokens, Y_ptr, ldy, workspace_ptr=None, workspace_bytes=0, stream=None):
    return load().vq_gemm(ctypes.byref(desc) if desc is not None else None, X_ptr, ldx, tokens, Y_ptr, ldy,
                          workspace_ptr, workspace_bytes, stream)


def vq_assign(W_ptr, B_ptr, ld, rows, cols, codebook_ptr, v, k, idx_ptr, idx_row_stride, stream=None):
    return load().vq_assign(W_ptr, B_ptr, ld, rows, cols, codebook_ptr, v, k, idx_ptr, idx_row_stride, stream)


def vq_assign_down(W_ptr, B_ptr, ld, rows, cols, codebook_ptr, v, k, idx_ptr, idx_row_stride, stream=None):
    return load().vq_assign_down(W_ptr, B_ptr, ld, rows, cols, codebook_ptr, v, k, idx_ptr, idx_row_stride, stream)


def vq_quantize_columns_workspace_bytes(rows, v, k, k_res):
    return load().vq_quantize_columns_workspace_bytes(rows, v, k, k_res)


def vq_quantize_columns(W_ptr, ldw, rows, cols, Hinv_ptr, ldh, codebook_ptr, v, k, codebook_res_ptr, k_res, block, idx_ptr, idx_row_stride,
                        idx_res_ptr, idx_res_row_stride, T_ptr, ldt, workspace_ptr, workspace_bytes, stream=None):
    return load().vq_quantize_columns(W_ptr, ldw, rows, cols, Hinv_ptr, ldh, codebook_ptr, v, k, codebook_res_ptr, k_res, block, idx_ptr,
                                      idx_row_stride, idx_res_ptr, idx_res_row_stride, T_ptr, ldt, workspace_ptr, workspace_bytes, stream)


def vq_gemm_workspace_bytes(desc, tokens):
    return load().vq_gemm_workspace_bytes(ctypes.byref(desc), tokens)


def vq_gemm_fast_workspace_bytes(desc, tokens):
    return load().vq_gemm_fast_workspace_bytes(ctypes.byref(desc), tokens)


def vq_status_string(status):
    return load().vq_status_string(status).decode()


def vq_version():
    return load().vq_version()


# ---- conveniences over torch tensors (allocation and pointer extraction only) ----------------------------
class DeviceLayer:
    """Device copies of one layer's arrays plus the descriptor that points at them."""

    def __init__(self, layer, device="cuda"):
        import torch
        self.layer = layer
        self.tensors = {}

        def up(name, arr):
            if arr is None:
                return None
            t = torch.from_numpy(arr).to(device).contiguous()
            self.tensors[name] = t
            return t.data_ptr()

        def stride(a):
            return a.shape[1] if a is not None else 0
        self.desc = vq_layer_desc(
            ctypes.sizeof(vq_layer_desc), layer.out_features, layer.in_features, layer.v, layer.k, layer.k_res,
            layer.n_outlier_cols, layer.v_out, layer.k_out,
            up("codebook", layer.codebook), up("codebook_res", layer.codebook_res), up("codebook_out", layer.codebook_out),
            up("idx", layer.idx), stride(layer.idx), up("idx_res", layer.idx_res), stride(layer.idx_res),
            up("idx_out", layer.idx_out), stride(layer.idx_out), up("scale", layer.scale), up("bias", layer.bias),
            int(getattr(layer, "group_vectors", 0)), int(getattr(layer, "orientation", 0)),
            up("col_perm", getattr(layer, "col_perm", None)))


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def dequant(dl: DeviceLayer, ldw=None):
    """fp16 [out][ldw] restored weights on the device (columns >= in_features are zero-initialised, never written)."""
    import torch
    L = dl.layer
    ldw = L.in_features if ldw is None else ldw
    W = torch.zeros((L.out_features, ldw), dtype=torch.float16, device="cuda")
    rc = vq_dequant(dl.desc, W.data_ptr(), ldw, _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_dequant")
    return W


def gemv(dl: DeviceLayer, x, out=None, workspace=None):
    """x: fp16 [batch][>=in] device tensor -> fp16 [batch][out].  workspace: a uint8 device tensor, or "fast" to allocate
    the one vq_gemv_workspace_bytes asks for (layers with codebook groups), or None."""
    import torch
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    y = out if out is not None else torch.empty((x.shape[0], dl.layer.out_features), dtype=torch.float16, device="cuda")
    if workspace is None:
        rc = vq_gemv(dl.desc, x.data_ptr(), x.stride(0), x.shape[0], y.data_ptr(), y.stride(0), _stream())
    else:
        if isinstance(workspace, str):
            assert workspace == "fast"
            workspace = torch.empty(max(vq_gemv_workspace_bytes(dl.desc, x.shape[0]), 256), dtype=torch.uint8, device="cuda")
        rc = vq_gemv_with_workspace(dl.desc, x.data_ptr(), x.stride(0), x.shape[0], y.data_ptr(), y.stride(0),
                                    workspace.data_ptr(), workspace.numel(), _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_gemv")
    return y


def gemv_multi(dls, x, outs=None):
    """Several layers on the same x (fp16 [batch][>=in] device tensor) in one call -> list of fp16 [batch][out_i]."""
    import torch
    assert x.is_cuda and x.dtype == torch.float16 and x.dim() == 2 and x.stride(1) == 1
    ys = outs if outs is not None else [torch.empty((x.shape[0], dl.layer.out_features), dtype=torch.float16, device="cuda")
                                        for dl in dls]
    rc = vq_gemv_multi([dl.desc for dl in dls], x.data_ptr(), x.stride(0), x.shape[0], [y.data_ptr() for y in ys],
                       [y.stride(0) for y in ys], _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_gemv_multi")
    return ys


def assign(W, codebook, base=None, cols=None, orientation=0):
    """W (and base): fp16 [rows][>= cols] device tensors, codebook: fp16 [k][v] device tensor -> uint8 [streams][stride]
    packed indices of the nearest centroids (stride: a stream's bits rounded up to 16 bytes, padding zero).  orientation 0:
    vectors along the rows, a stream per row; 1: vectors down the columns, a stream per block of v rows."""
    import torch
    assert W.is_cuda and W.dtype == torch.float16 and W.dim() == 2 and W.stride(1) == 1
    assert base is None or (base.dtype == torch.float16 and base.shape == W.shape and base.stride() == W.stride())
    codebook = codebook.contiguous()
    k, v = codebook.shape
    cols = W.shape[1] if cols is None else cols
    bits = max(1, (k - 1).bit_length())
    per_stream = cols if orientation else -(-cols // v)
    streams = -(-W.shape[0] // v) if orientation else W.shape[0]
    stride = (per_stream * bits + 127) // 128 * 16
    idx = torch.zeros((streams, stride), dtype=torch.uint8, device="cuda")
    fn = vq_assign_down if orientation else vq_assign
    rc = fn(W.data_ptr(), base.data_ptr() if base is not None else None, W.stride(0), W.shape[0], cols, codebook.data_ptr(),
            v, k, idx.data_ptr(), stride, _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_assign_down" if orientation else "vq_assign")
    return idx


def quantize_columns(W, Hinv, codebook, codebook_res=None, block=128, want_T=True):
    """Algorithm 1's column loop.  W: fp32 [rows][cols] device tensor (overwritten with the quantized weights), Hinv: fp32
    [cols][cols], codebooks fp16 [k][v] device tensors -> (idx, idx_res or None, T or None): packed uint8 streams
    [ceil(rows / v)][stride] of orientation 1 and the fp32 columns as they stood when they were quantized."""
    import torch
    assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.stride(1) == 1
    assert Hinv.dtype == torch.float32 and Hinv.shape == (W.shape[1], W.shape[1]) and Hinv.stride(1) == 1
    codebook = codebook.contiguous()
    k, v = codebook.shape
    k_res = 0
    if codebook_res is not None:
        codebook_res = codebook_res.contiguous()
        k_res = codebook_res.shape[0]
    rows, cols = W.shape
    streams = -(-rows // v)

    def stream_buffer(kk):
        bits = max(1, (kk - 1).bit_length())
        stride = (cols * bits + 127) // 128 * 16
        return torch.full((streams, stride), 0xEE, dtype=torch.uint8, device="cuda"), stride
    idx, stride = stream_buffer(k)
    idx_res, stride_res = stream_buffer(k_res) if k_res else (None, 0)
    T = torch.empty_like(W) if want_T else None
    need = vq_quantize_columns_workspace_bytes(rows, v, k, k_res)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    rc = vq_quantize_columns(W.data_ptr(), W.stride(0), rows, cols, Hinv.data_ptr(), Hinv.stride(0), codebook.data_ptr(), v, k,
                             codebook_res.data_ptr() if k_res else None, k_res, block, idx.data_ptr(), stride,
                             idx_res.data_ptr() if k_res else None, stride_res, T.data_ptr() if want_T else None,
                             T.stride(0) if want_T else 0, ws.data_ptr(), need, _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_quantize_columns")
    return idx, idx_res, T


def gemm(dl: DeviceLayer, X, out=None, workspace=None):
    """X: fp16 [tokens][>=in] device tensor -> fp16 [tokens][out].  workspace: a uint8 device tensor, or "fast" to
    allocate the one vq_gemm_fast_workspace_bytes asks for (the restore-then-multiply route), or None."""
    import torch
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    Y = out if out is not None else torch.empty((X.shape[0], dl.layer.out_features), dtype=torch.float16, device="cuda")
    if isinstance(workspace, str):
        assert workspace == "fast"
        fast = vq_gemm_fast_workspace_bytes(dl.desc, X.shape[0])
        workspace = torch.empty(fast, dtype=torch.uint8, device="cuda") if fast else None
    need = vq_gemm_workspace_bytes(dl.desc, X.shape[0])
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
    rc = vq_gemm(dl.desc, X.data_ptr(), X.stride(0), X.shape[0], Y.data_ptr(), Y.stride(0),
                 workspace.data_ptr() if workspace is not None else None,
                 workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream())
    if rc != VQ_OK:
        raise VQError(rc, "vq_gemm")
    return Y
