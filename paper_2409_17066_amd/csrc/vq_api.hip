// C-ABI entry points: descriptor validation and dispatch.  All device work is in the kernel files.
#include "vq_common.hpp"
#include <cstdlib>
#include <cstring>
#include <mutex>

namespace vq {

int cu_count() {
  static const int n = [] {
    int dev = 0, c = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || c < 1) c = 256;
    return c;
  }();
  return n;
}

namespace {
thread_local Switches g_switches;
}
const Switches &switches() { return g_switches; }

// VQ_SWITCHES = "name=value,name=value": unknown names are ignored.
void read_switches() {
  Switches sw;
  const char *e = getenv("VQ_SWITCHES");
  while (e && *e) {
    const char *eq = strchr(e, '='), *end = strchr(e, ',');
    if (!end) end = e + strlen(e);
    if (eq && eq < end) {
      const size_t n = (size_t)(eq - e);
      const char v = eq[1] == ',' ? '\0' : eq[1];
      if (n == 4 && !strncmp(e, "gemv", 4)) sw.gemv = v;
      else if (n == 4 && !strncmp(e, "gemm", 4)) sw.gemm = v;
      else if (n == 7 && !strncmp(e, "dequant", 7)) sw.dequant = v;
      else if (n == 6 && !strncmp(e, "groups", 6)) sw.groups_loop = v == 'l';
      else if (n == 5 && !strncmp(e, "multi", 5)) sw.multi_off = v == '0';
      else if (n == 5 && !strncmp(e, "dense", 5)) sw.dense = v == '0' ? 0 : v == '1' ? 1 : -1;
    }
    e = *end ? end + 1 : end;
  }
  g_switches = sw;
}

static bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static int check_stream(const void *idx, long long stride, int per_row, int bits) {
  if (!idx) return VQ_ERR_NULL;
  if (stride < ((long long)per_row * bits + 7) / 8) return VQ_ERR_SHAPE;
  if (stride % 16 != 0 || !aligned(idx, 16)) return VQ_ERR_ALIGNMENT;
  return VQ_OK;
}

int make_params(const vq_layer_desc *d, Params *p) {
  if (!d) return VQ_ERR_NULL;
  if (d->struct_size != sizeof(vq_layer_desc) && d->struct_size != VQ_LAYER_DESC_SIZE_V1 && d->struct_size != VQ_LAYER_DESC_SIZE_V2)
    return VQ_ERR_SHAPE;
  const bool v2 = d->struct_size != VQ_LAYER_DESC_SIZE_V1;
  const int group_vectors = v2 ? d->group_vectors : 0;
  const int orientation = v2 ? d->orientation : 0;
  const int32_t *col_perm = d->struct_size == sizeof(vq_layer_desc) ? d->col_perm : nullptr;
  if (col_perm && !aligned(col_perm, 4)) return VQ_ERR_ALIGNMENT;
  if (group_vectors < 0 || (orientation != 0 && orientation != 1)) return VQ_ERR_SHAPE;
  const int lim = 1 << 24;
  if (d->out_features < 1 || d->out_features > lim || d->in_features < 1 || d->in_features > lim) return VQ_ERR_SHAPE;
  if (d->v < 1 || d->v > 16 || d->k < 2 || d->k > 65536) return VQ_ERR_SHAPE;
  if (d->k_res != 0 && (d->k_res < 2 || d->k_res > 65536)) return VQ_ERR_SHAPE;
  if (d->n_outlier_cols < 0) return VQ_ERR_SHAPE;
  if (d->n_outlier_cols > 0) {
    if (d->v_out < 1 || d->v_out > 16 || d->k_out < 2 || d->k_out > 65536) return VQ_ERR_SHAPE;
    if ((orientation == 0 && d->n_outlier_cols % d->v_out != 0) || d->n_outlier_cols >= d->in_features) return VQ_ERR_SHAPE;
  }
  Params q{};
  q.out_features = d->out_features; q.in_features = d->in_features;
  q.v = d->v; q.k = d->k; q.bits = index_bits(d->k);
  q.k_res = d->k_res; q.bits_res = d->k_res ? index_bits(d->k_res) : 0;
  q.n_out = d->n_outlier_cols;
  q.v_out = q.n_out ? d->v_out : 1; q.k_out = q.n_out ? d->k_out : 0; q.bits_out = q.n_out ? index_bits(d->k_out) : 0;
  q.orientation = orientation;
  if (orientation == 0) {
    q.P = (d->in_features - q.n_out + d->v - 1) / d->v;
    q.Q = q.n_out ? q.n_out / d->v_out : 0;
    q.S = d->out_features; q.S_out = q.n_out ? d->out_features : 0;
  } else {
    q.P = d->in_features - q.n_out;
    q.Q = q.n_out;
    q.S = (d->out_features + d->v - 1) / d->v; q.S_out = q.n_out ? (d->out_features + d->v_out - 1) / d->v_out : 0;
  }
  q.Pg = group_vectors > 0 && group_vectors < q.P ? group_vectors : q.P;
  q.n_groups = (q.P + q.Pg - 1) / q.Pg;
  if (!d->codebook) return VQ_ERR_NULL;
  if (!aligned(d->codebook, 16)) return VQ_ERR_ALIGNMENT;
  int rc = check_stream(d->idx, d->idx_row_stride, q.P, q.bits);
  if (rc != VQ_OK) return rc;
  if (q.k_res) {
    if (!d->codebook_res) return VQ_ERR_NULL;
    if (!aligned(d->codebook_res, 16)) return VQ_ERR_ALIGNMENT;
    rc = check_stream(d->idx_res, d->idx_res_row_stride, q.P, q.bits_res);
    if (rc != VQ_OK) return rc;
  }
  if (q.n_out) {
    if (!d->codebook_out) return VQ_ERR_NULL;
    if (!aligned(d->codebook_out, 16)) return VQ_ERR_ALIGNMENT;
    rc = check_stream(d->idx_out, d->idx_out_row_stride, q.Q, q.bits_out);
    if (rc != VQ_OK) return rc;
  }
  if ((d->scale && !aligned(d->scale, 2)) || (d->bias && !aligned(d->bias, 2))) return VQ_ERR_ALIGNMENT;
  q.cb = static_cast<const __half *>(d->codebook);
  q.cb_res = q.k_res ? static_cast<const __half *>(d->codebook_res) : nullptr;
  q.cb_out = q.n_out ? static_cast<const __half *>(d->codebook_out) : nullptr;
  q.idx = static_cast<const uint8_t *>(d->idx); q.stride = d->idx_row_stride;
  q.idx_res = q.k_res ? static_cast<const uint8_t *>(d->idx_res) : nullptr; q.stride_res = q.k_res ? d->idx_res_row_stride : 0;
  q.idx_out = q.n_out ? static_cast<const uint8_t *>(d->idx_out) : nullptr; q.stride_out = q.n_out ? d->idx_out_row_stride : 0;
  q.scale = static_cast<const __half *>(d->scale);
  q.bias = static_cast<const __half *>(d->bias);
  q.perm = col_perm;
  if (p) *p = q;
  return VQ_OK;
}

}  // namespace vq

using vq::aligned;

extern "C" int vq_validate(const vq_layer_desc *desc) { return vq::make_params(desc, nullptr); }

extern "C" int vq_dequant(const vq_layer_desc *desc, void *W, int64_t ldw, void *hip_stream) {
  vq::read_switches();
  vq::Params p;
  int rc = vq::make_params(desc, &p);
  if (rc != VQ_OK) return rc;
  if (!W) return VQ_ERR_NULL;
  if (ldw < p.in_features) return VQ_ERR_SHAPE;
  if (!aligned(W, 2)) return VQ_ERR_ALIGNMENT;
  return vq::launch_dequant(p, static_cast<__half *>(W), ldw, static_cast<hipStream_t>(hip_stream));
}

extern "C" int vq_gemv(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch,
                       void *y, int64_t ldy, void *hip_stream) {
  vq::read_switches();
  vq::Params p;
  int rc = vq::make_params(desc, &p);
  if (rc != VQ_OK) return rc;
  if (!x || !y) return VQ_ERR_NULL;
  if (batch < 1 || batch > 16 || ldx < p.in_features || ldy < p.out_features) return VQ_ERR_SHAPE;
  if (!aligned(x, 2) || !aligned(y, 2)) return VQ_ERR_ALIGNMENT;
  return vq::launch_gemv(p, static_cast<const __half *>(x), ldx, batch, static_cast<__half *>(y), ldy,
                         static_cast<hipStream_t>(hip_stream));
}

extern "C" size_t vq_gemv_workspace_bytes(const vq_layer_desc *desc, int32_t batch) {
  vq::read_switches();
  vq::Params p;
  if (vq::make_params(desc, &p) != VQ_OK || batch < 1 || batch > 16) return 0;
  // the size does not depend on x; the fast kernels' conditions on x are checked again at the call
  return vq::gemv_workspace_bytes(p, nullptr, p.in_features + (p.in_features & 1), batch);
}

extern "C" int vq_gemv_with_workspace(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch, void *y, int64_t ldy,
                                      void *workspace, size_t workspace_bytes, void *hip_stream) {
  vq::read_switches();
  vq::Params p;
  int rc = vq::make_params(desc, &p);
  if (rc != VQ_OK) return rc;
  if (!x || !y) return VQ_ERR_NULL;
  if (batch < 1 || batch > 16 || ldx < p.in_features || ldy < p.out_features) return VQ_ERR_SHAPE;
  if (!aligned(x, 2) || !aligned(y, 2)) return VQ_ERR_ALIGNMENT;
  if (workspace && workspace_bytes && !aligned(workspace, 256)) return VQ_ERR_ALIGNMENT;
  return vq::launch_gemv_ws(p, static_cast<const __half *>(x), ldx, batch, static_cast<__half *>(y), ldy, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream));
}

// ---- vq_gemv_with_workspace for callers that cannot allocate: the workspace is a device array of this library.
// In host code the array's name is only a handle for hipGetSymbolAddress; what kernels and the launchers get is the
// device address that call returns, looked up once per device (every device holds its own copy of the array).
namespace vq {
static __device__ __align__(256) unsigned char scratch[VQ_GEMV_STATIC_WORKSPACE_BYTES];
namespace {
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

int static_workspace(void **ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return VQ_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return VQ_ERR_HIP;
    g_scratch_ptr[dev] = q;
  }
  *ptr = g_scratch_ptr[dev];
  return VQ_OK;
}
}  // namespace
}  // namespace vq

extern "C" int vq_gemv_static_workspace(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch, void *y, int64_t ldy,
                                        void *hip_stream) {
  vq::read_switches();
  vq::Params p;
  int rc = vq::make_params(desc, &p);
  if (rc != VQ_OK) return rc;
  if (!x || !y) return VQ_ERR_NULL;
  if (batch < 1 || batch > 16 || ldx < p.in_features || ldy < p.out_features) return VQ_ERR_SHAPE;
  if (!aligned(x, 2) || !aligned(y, 2)) return VQ_ERR_ALIGNMENT;
  const size_t need = vq::gemv_workspace_bytes(p, static_cast<const __half *>(x), ldx, batch);
  if (need > (size_t)VQ_GEMV_STATIC_WORKSPACE_BYTES) return VQ_ERR_WORKSPACE;
  void *ws = nullptr;
  if (need) {
    rc = vq::static_workspace(&ws);
    if (rc != VQ_OK) return rc;
  }
  return vq::launch_gemv_ws(p, static_cast<const __half *>(x), ldx, batch, static_cast<__half *>(y), ldy, ws, need,
                            static_cast<hipStream_t>(hip_stream));
}

extern "C" int vq_gemv_multi(const vq_layer_desc *const *descs, int32_t n_layers, const void *x, int64_t ldx, int32_t batch,
                             void *const *y, const int64_t *ldy, void *hip_stream) {
  vq::read_switches();
  constexpr int MAX_LAYERS = 8;
  if (!descs || !y || !ldy || !x) return VQ_ERR_NULL;
  if (n_layers < 1 || n_layers > MAX_LAYERS || batch < 1 || batch > 16) return VQ_ERR_SHAPE;
  vq::Params p[MAX_LAYERS];
  __half *ys[MAX_LAYERS];
  long long ldys[MAX_LAYERS];
  for (int i = 0; i < n_layers; ++i) {
    const int rc = vq::make_params(descs[i], &p[i]);
    if (rc != VQ_OK) return rc;
    if (!y[i]) return VQ_ERR_NULL;
    if (p[i].in_features != p[0].in_features || ldx < p[i].in_features || ldy[i] < p[i].out_features) return VQ_ERR_SHAPE;
    if (!aligned(x, 2) || !aligned(y[i], 2)) return VQ_ERR_ALIGNMENT;
    ys[i] = static_cast<__half *>(y[i]); ldys[i] = ldy[i];
  }
  return vq::launch_gemv_multi(p, n_layers, static_cast<const __half *>(x), ldx, batch, ys, ldys, static_cast<hipStream_t>(hip_stream));
}

extern "C" size_t vq_gemm_workspace_bytes(const vq_layer_desc *desc, int32_t tokens) {
  vq::read_switches();
  vq::Params p;
  if (vq::make_params(desc, &p) != VQ_OK || tokens < 1) return 0;
  return vq::gemm_workspace_bytes(p, tokens);
}

extern "C" size_t vq_gemm_fast_workspace_bytes(const vq_layer_desc *desc, int32_t tokens) {
  vq::read_switches();
  vq::Params p;
  if (vq::make_params(desc, &p) != VQ_OK || tokens < 1) return 0;
  return vq::gemm_fast_workspace_bytes(p, tokens);
}

extern "C" int vq_gemm(const vq_layer_desc *desc, const void *X, int64_t ldx, int32_t tokens,
                       void *Y, int64_t ldy, void *workspace, size_t workspace_bytes, void *hip_stream) {
  vq::read_switches();
  vq::Params p;
  int rc = vq::make_params(desc, &p);
  if (rc != VQ_OK) return rc;
  if (!X || !Y) return VQ_ERR_NULL;
  if (tokens < 1 || tokens > (1 << 24) || ldx < p.in_features || ldy < p.out_features) return VQ_ERR_SHAPE;
  if (!aligned(X, 16) || (ldx & 7) || !aligned(Y, 2)) return VQ_ERR_ALIGNMENT;
  const size_t need = vq::gemm_workspace_bytes(p, tokens);
  if (need && (!workspace || workspace_bytes < need)) return VQ_ERR_WORKSPACE;
  if (workspace && workspace_bytes && !aligned(workspace, 16)) return VQ_ERR_ALIGNMENT;
  return vq::launch_gemm(p, static_cast<const __half *>(X), ldx, tokens, static_cast<__half *>(Y), ldy,
                         workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

extern "C" int vq_assign(const void *W, const void *B, int64_t ld, int32_t rows, int32_t cols, const void *codebook, int32_t v, int32_t k,
                         void *idx, int64_t idx_row_stride, void *hip_stream) {
  if (!W || !codebook || !idx) return VQ_ERR_NULL;
  const int lim = 1 << 24;
  if (rows < 1 || rows > lim || cols < 1 || cols > lim || ld < cols || v < 1 || v > 16 || k < 2 || k > 65536) return VQ_ERR_SHAPE;
  const long long P = ((long long)cols + v - 1) / v;
  const long long need = ((P * vq::index_bits(k) + 31) / 32) * 4;             // whole dwords
  if (idx_row_stride < need) return VQ_ERR_SHAPE;
  if (!aligned(W, 2) || (B && !aligned(B, 2)) || !aligned(codebook, 2)) return VQ_ERR_ALIGNMENT;
  if (!aligned(idx, 16) || idx_row_stride % 16 != 0) return VQ_ERR_ALIGNMENT;
  return vq::launch_assign(static_cast<const __half *>(W), static_cast<const __half *>(B), ld, rows, cols,
                           static_cast<const __half *>(codebook), v, k, static_cast<unsigned char *>(idx), idx_row_stride,
                           static_cast<hipStream_t>(hip_stream));
}

extern "C" int vq_assign_down(const void *W, const void *B, int64_t ld, int32_t rows, int32_t cols, const void *codebook, int32_t v,
                              int32_t k, void *idx, int64_t idx_row_stride, void *hip_stream) {
  if (!W || !codebook || !idx) return VQ_ERR_NULL;
  const int lim = 1 << 24;
  if (rows < 1 || rows > lim || cols < 1 || cols > lim || ld < cols || v < 1 || v > 16 || k < 2 || k > 65536) return VQ_ERR_SHAPE;
  const long long need = (((long long)cols * vq::index_bits(k) + 31) / 32) * 4;             // whole dwords
  if (idx_row_stride < need) return VQ_ERR_SHAPE;
  if (!aligned(W, 2) || (B && !aligned(B, 2)) || !aligned(codebook, 2)) return VQ_ERR_ALIGNMENT;
  if (!aligned(idx, 16) || idx_row_stride % 16 != 0) return VQ_ERR_ALIGNMENT;
  return vq::launch_assign_down(static_cast<const __half *>(W), static_cast<const __half *>(B), ld, rows, cols,
                                static_cast<const __half *>(codebook), v, k, static_cast<unsigned char *>(idx), idx_row_stride,
                                static_cast<hipStream_t>(hip_stream));
}

extern "C" size_t vq_quantize_columns_workspace_bytes(int32_t rows, int32_t v, int32_t k, int32_t k_res) {
  if (rows < 1 || rows > (1 << 24) || v < 1 || v > 16 || k < 2 || k > 65536 || (k_res != 0 && (k_res < 2 || k_res > 65536))) return 0;
  return vq::quantize_columns_workspace_bytes(rows, v, k, k_res);
}

extern "C" int vq_quantize_columns(void *W, int64_t ldw, int32_t rows, int32_t cols, const void *Hinv, int64_t ldh, const void *codebook,
                                   int32_t v, int32_t k, const void *codebook_res, int32_t k_res, int32_t block, void *idx,
                                   int64_t idx_row_stride, void *idx_res, int64_t idx_res_row_stride, void *T, int64_t ldt, void *workspace,
                                   size_t workspace_bytes, void *hip_stream) {
  if (!W || !Hinv || !codebook || !idx) return VQ_ERR_NULL;
  const int lim = 1 << 24;
  if (rows < 1 || rows > lim || cols < 1 || cols > lim || ldw < cols || ldh < cols || v < 1 || v > 16 || k < 2 || k > 65536) return VQ_ERR_SHAPE;
  if (k_res != 0 && (k_res < 2 || k_res > 65536)) return VQ_ERR_SHAPE;
  if (k_res && (!codebook_res || !idx_res)) return VQ_ERR_NULL;
  if (block < 1 || block > 128 || (T && ldt < cols)) return VQ_ERR_SHAPE;
  if (idx_row_stride < (((long long)cols * vq::index_bits(k) + 31) / 32) * 4) return VQ_ERR_SHAPE;
  if (k_res && idx_res_row_stride < (((long long)cols * vq::index_bits(k_res) + 31) / 32) * 4) return VQ_ERR_SHAPE;
  if (!aligned(W, 4) || !aligned(Hinv, 4) || (T && !aligned(T, 4)) || !aligned(codebook, 2) || (k_res && !aligned(codebook_res, 2))) return VQ_ERR_ALIGNMENT;
  if (!aligned(idx, 16) || idx_row_stride % 16 != 0 || (k_res && (!aligned(idx_res, 16) || idx_res_row_stride % 16 != 0))) return VQ_ERR_ALIGNMENT;
  const size_t need = vq::quantize_columns_workspace_bytes(rows, v, k, k_res);
  if (!workspace || workspace_bytes < need) return VQ_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return VQ_ERR_ALIGNMENT;
  return vq::launch_quantize_columns(static_cast<float *>(W), ldw, rows, cols, static_cast<const float *>(Hinv), ldh,
                                     static_cast<const __half *>(codebook), v, k, static_cast<const __half *>(codebook_res), k_res, block,
                                     static_cast<unsigned char *>(idx), idx_row_stride, static_cast<unsigned char *>(idx_res),
                                     idx_res_row_stride, static_cast<float *>(T), ldt, workspace, static_cast<hipStream_t>(hip_stream));
}

extern "C" const char *vq_status_string(int status) {
  switch (status) {
    case VQ_OK: return "ok";
    case VQ_ERR_NULL: return "a required pointer is NULL";
    case VQ_ERR_SHAPE: return "size, stride or leading dimension out of range";
    case VQ_ERR_ALIGNMENT: return "pointer or stride misaligned";
    case VQ_ERR_UNSUPPORTED: return "no kernel handles this layer";
    case VQ_ERR_HIP: return "HIP launch error";
    case VQ_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
  }
}

extern "C" int vq_version(void) { return 100; }
