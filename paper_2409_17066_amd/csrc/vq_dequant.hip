// vq_dequant: restore the FP16 weight matrix (paper Sec. 2.2 lookup; Sec. 3.2.2 residual sum;
// Sec. 3.2.3 outlier columns; App. "Our Dequantization Implementation", first phase).
#include "vq_common.hpp"

namespace vq {

// Where stored column c of a row goes (Sec. 3.2.3: the stored order of the columns may be a permutation of the layer's).
// Entries outside the row are dropped.
__device__ __forceinline__ void store_col(const Params &p, __half *wrow, int c, __half value) {
  const int t = p.perm ? p.perm[c] : c;
  if ((unsigned)t < (unsigned)p.in_features) wrow[t] = value;
}

// Any (v, k, residual, outlier) combination: one thread restores one vector.  Consecutive threads
// take consecutive vectors of one row, so a wave's stores cover one contiguous span of the row (of its stored order).
__global__ __launch_bounds__(256) void dequant_generic_kernel(Params p, __half *W, long long ldw, int blocks_per_row) {
  const int o = blockIdx.x / blocks_per_row;
  const int slot = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  if (slot >= p.Q + p.P) return;
  const float s = p.scale ? __half2float(p.scale[o]) : 1.0f;
  const float b = p.bias ? __half2float(p.bias[o]) : 0.0f;
  __half *wrow = W + (long long)o * ldw;
  if (slot < p.Q) {
    unsigned i = load_index(p.idx_out + (long long)o * p.stride_out, slot, p.bits_out);
    i = min(i, (unsigned)p.k_out - 1u);
    const __half *e = p.cb_out + (long long)i * p.v_out;
    const int c0 = slot * p.v_out;
    for (int j = 0; j < p.v_out; ++j) store_col(p, wrow, c0 + j, restore(__half2float(e[j]), s, b));
  } else {
    const int pp = slot - p.Q;
    unsigned i = load_index(p.idx + (long long)o * p.stride, pp, p.bits);
    i = min(i, (unsigned)p.k - 1u);
    const long long group = pp / p.Pg;                          // this vector's tables
    const __half *e = p.cb + (group * p.k + i) * p.v;
    const __half *er = nullptr;
    if (p.k_res) {
      unsigned r = load_index(p.idx_res + (long long)o * p.stride_res, pp, p.bits_res);
      r = min(r, (unsigned)p.k_res - 1u);
      er = p.cb_res + (group * p.k_res + r) * p.v;
    }
    const int c0 = p.n_out + pp * p.v;
    for (int j = 0; j < p.v; ++j) {
      if (c0 + j >= p.in_features) break;
      float d = __half2float(e[j]);
      if (er) d = __fadd_rn(d, __half2float(er[j]));
      store_col(p, wrow, c0 + j, restore(d, s, b));
    }
  }
}

// Orientation 1 (vectors down the output dimension; Sec. 3.1, Algorithm 1): one thread restores one vector, i.e. v
// consecutive rows of one column.  Consecutive threads take consecutive columns of one stream, so each of the v stores
// of a wave covers one contiguous span of a row.  Blocks [0, main_blocks) take the main streams, the rest the outlier ones.
__global__ __launch_bounds__(256) void dequant_down_kernel(Params p, __half *W, long long ldw, int bps_main, long long main_blocks, int bps_out) {
  const bool main = (long long)blockIdx.x < main_blocks;
  const long long blk = main ? (long long)blockIdx.x : (long long)blockIdx.x - main_blocks;
  const int bps = main ? bps_main : bps_out;
  const int stream = (int)(blk / bps);
  const int t = (int)(blk % bps) * 256 + threadIdx.x;
  if (t >= (main ? p.P : p.Q)) return;
  const int v = main ? p.v : p.v_out;
  const __half *e, *er = nullptr;
  if (main) {
    unsigned i = min(load_index(p.idx + (long long)stream * p.stride, t, p.bits), (unsigned)p.k - 1u);
    const long long group = t / p.Pg;
    e = p.cb + (group * p.k + i) * p.v;
    if (p.k_res) {
      unsigned r = min(load_index(p.idx_res + (long long)stream * p.stride_res, t, p.bits_res), (unsigned)p.k_res - 1u);
      er = p.cb_res + (group * p.k_res + r) * p.v;
    }
  } else {
    unsigned i = min(load_index(p.idx_out + (long long)stream * p.stride_out, t, p.bits_out), (unsigned)p.k_out - 1u);
    e = p.cb_out + (long long)i * p.v_out;
  }
  const int c = main ? p.n_out + t : t;
  for (int j = 0; j < v; ++j) {
    const int o = stream * v + j;
    if (o >= p.out_features) break;
    float d = __half2float(e[j]);
    if (er) d = __fadd_rn(d, __half2float(er[j]));
    store_col(p, W + (long long)o * ldw, c, restore(d, p.scale ? __half2float(p.scale[o]) : 1.0f, p.bias ? __half2float(p.bias[o]) : 0.0f));
  }
}

// The outlier columns of a row-wise layer only (the main columns were restored by a fast kernel).
int launch_dequant_outliers(const Params &p, __half *W, long long ldw, hipStream_t s) {
  Params q = p;
  q.P = 0;                                   // the generic kernel's slots are outlier vectors first, then main vectors
  const int blocks_per_row = (q.Q + 255) / 256;
  const long long blocks = (long long)blocks_per_row * q.out_features;
  if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(dequant_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, q, W, ldw, blocks_per_row);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

int launch_dequant_fast(const Params &p, __half *W, long long ldw, hipStream_t s);
int launch_dequant_down_fast(const Params &p, __half *W, long long ldw, hipStream_t s);
int launch_dequant_lds(const Params &p, __half *W, long long ldw, hipStream_t s);
int launch_dequant_down_lds(const Params &p, __half *W, long long ldw, hipStream_t s);

int launch_dequant(const Params &p, __half *W, long long ldw, hipStream_t s) {
  if (p.perm && switches().dequant != 'g') {
    // Permuted column order: restore in stored order with whatever kernel takes the layer, then move every row's values to
    // their columns, in place, through LDS.  (Rows too long for LDS: the generic kernels below, which scatter their stores.)
    Params q = p;
    q.perm = nullptr;
    if ((long long)p.in_features * 2 <= 160 * 1024) {
      const int rc = launch_dequant(q, W, ldw, s);
      return rc == VQ_OK ? launch_place_cols(W, ldw, p.out_features, p.in_features, p.perm, s) : rc;
    }
  }
  if (p.orientation == 1) {
    const int bps_main = (p.P + 255) / 256, bps_out = p.Q ? (p.Q + 255) / 256 : 1;
    long long main_blocks = (long long)bps_main * p.S;
    int rc = p.perm ? VQ_ERR_UNSUPPORTED : launch_dequant_down_fast(p, W, ldw, s);          // the main columns, when a fast kernel takes them
    if (rc == VQ_ERR_UNSUPPORTED && !p.perm) rc = launch_dequant_down_lds(p, W, ldw, s);      // (the other settings: tables in LDS)
    if (rc == VQ_OK) {
      if (!p.Q) return VQ_OK;
      main_blocks = 0;                                               // the generic kernel below: outlier streams only
    } else if (rc != VQ_ERR_UNSUPPORTED) {
      return rc;
    }
    const long long blocks = main_blocks + (long long)bps_out * p.S_out;
    if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(dequant_down_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, W, ldw, bps_main, main_blocks, bps_out);
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  const int rc = p.perm ? VQ_ERR_UNSUPPORTED : launch_dequant_fast(p, W, ldw, s);
  if (rc != VQ_ERR_UNSUPPORTED) return rc;
  if (!p.perm) {
    // the other (v, k) settings: main columns with the tables in LDS, the few outlier columns by the generic kernel
    const int rl = launch_dequant_lds(p, W, ldw, s);
    if (rl == VQ_OK) return p.Q ? launch_dequant_outliers(p, W, ldw, s) : VQ_OK;
    if (rl != VQ_ERR_UNSUPPORTED) return rl;
  }
  const int slots = p.P + p.Q;
  const int blocks_per_row = (slots + 255) / 256;
  const long long blocks = (long long)blocks_per_row * p.out_features;
  if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(dequant_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, W, ldw, blocks_per_row);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace vq
