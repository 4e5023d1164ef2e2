// vq_quantize_columns: the column loop of the quantizer (Algorithm 1, Sec. 3.1 "VPTQ Algorithm"; error update: the
// Delta W equation of that section).  Columns are quantized one at a time -- every column a stack of length-v vectors
// that each take their nearest centroid (Eq. 2; with a residual codebook a second one for what the first leaves, Sec.
// 3.2.2) -- and the column's error, divided by the diagonal entry of the matrix the algorithm calls H^-1, is spread over
// the later columns: inside a block of B columns at once, over the rest of the matrix at the end of the block.
//
// The rows of the matrix never meet in this loop: a vector's v rows only ever read their own weights and rows of H^-1.
// So one wave owns one stack position (v rows) for a whole block of columns and keeps its v x B tile of running weights
// in registers (lane l holds columns l and l + 64 of the block); the 64 lanes split the centroids of the nearest-centroid
// search, which is where the time goes (2 v + 3 vector-ALU instructions per centroid, as in vq_assign, whose distance
// arithmetic this follows).  The end-of-block update W[:, rest] -= E * Hinv[block, rest] is a dense binary32 product and
// runs on the matrix cores (v_mfma_f32_32x32x2_f32) from LDS tiles.
#include "vq_common.hpp"

namespace vq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int QW = 4;            // waves (stack positions) per workgroup of the column kernel
constexpr int QB = 128;          // most columns per block: two per lane
constexpr int CPL = QB / 64;

constexpr int entry_halfs(int v) { return v <= 4 ? 4 : v <= 8 ? 8 : 16; }     // table entries padded to 8, 16 or 32 bytes

struct QArgs {
  float *W; long long ldw; int rows, cols;
  const float *Hinv; long long ldh;
  const __half *cb; int k; const __half *cb_res; int k_res;
  int s, s_end;
  unsigned *idx; long long idx_dwords; int bits;             // streams as dwords: stride in dwords
  unsigned *idx_res; long long idx_res_dwords; int bits_res;
  float *T; long long ldt;
  float *E;                                                   // [rows][QB]: the block's scaled errors
};

// smaller distance, else smaller index: the rule by which the lanes' candidates meet
__device__ __forceinline__ void wave_arg_min(float &d, unsigned &i) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float d2 = __shfl_xor(d, o, 64);
    const unsigned i2 = (unsigned)__shfl_xor((int)i, o, 64);
    if (d2 < d || (d2 == d && i2 < i)) { d = d2; i = i2; }
  }
}

// Nearest of `count` centroids to t[0 .. len): lane l takes centroids l, l + 64, ... in ascending order (strict "less"
// keeps the lowest index of equal distances among its own).  Distance: binary32, one subtraction and one fused
// multiply-add per element into a sum that starts at +0, elements ascending.  Entries are EH halfs apart.
template <int V, int EH, class TablePtr>
__device__ __forceinline__ unsigned nearest(TablePtr table, int count, const float (&t)[V], int len, int lane) {
  float best = __builtin_inff();
  unsigned arg = 0xFFFFFFFFu;                                 // a lane without centroids never wins
  constexpr int UN = 4;                                       // centroids in flight per lane: their sums do not depend on each other
  for (int i0 = lane; i0 < count; i0 += 64 * UN) {
    float d[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int i = min(i0 + 64 * u, count - 1);              // (past the end: the last entry again, never taken below)
      __half c[EH];
      if constexpr (EH == 4) *reinterpret_cast<uint2 *>(c) = *reinterpret_cast<const uint2 *>(table + (long long)i * EH);
      else {
#pragma unroll
        for (int q = 0; q < EH / 8; ++q) *reinterpret_cast<uint4 *>(c + 8 * q) = *reinterpret_cast<const uint4 *>(table + (long long)i * EH + 8 * q);
      }
      d[u] = 0.0f;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        if (j < len) {
          const float diff = __fsub_rn(t[j], __half2float(c[j]));
          d[u] = __fmaf_rn(diff, diff, d[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u)
      if (i0 + 64 * u < count && d[u] < best) { best = d[u]; arg = (unsigned)(i0 + 64 * u); }
  }
  wave_arg_min(best, arg);
  return arg;
}

template <int V, bool IN_LDS>
__global__ __launch_bounds__(QW * 64) void qcol_block_kernel(QArgs a) {
  constexpr int EH = entry_halfs(V);
  extern __shared__ __attribute__((aligned(16))) __half tables[];          // [k][EH] then [k_res][EH] when IN_LDS
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // tables as padded entries: in LDS when they fit, else where the caller of the launcher put them (a padded copy in the workspace)
  const __half *tab = a.cb, *tab_res = a.cb_res;
  if constexpr (IN_LDS) {
    const int n16 = ((a.k + a.k_res) * EH + 7) / 8;                        // both tables are one contiguous padded array (its end rounded up)
    for (int e = threadIdx.x; e < n16; e += QW * 64) reinterpret_cast<uint4 *>(tables)[e] = reinterpret_cast<const uint4 *>(a.cb)[e];
    __syncthreads();
  }
  const int p = blockIdx.x * QW + wave;
  const int m0 = p * V;
  if (m0 >= a.rows) return;
  const int len = min(V, a.rows - m0);
  const int nb = a.s_end - a.s;

  float w[CPL][V];
#pragma unroll
  for (int i = 0; i < CPL; ++i)
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int c = a.s + lane + 64 * i;
      w[i][j] = (c < a.s_end && j < len) ? a.W[(long long)(m0 + j) * a.ldw + c] : 0.0f;
    }
  unsigned code[CPL] = {0u, 0u}, code_res[CPL] = {0u, 0u};
  float h[CPL];
#pragma unroll
  for (int i = 0; i < CPL; ++i) h[i] = (a.s + lane + 64 * i < a.s_end) ? a.Hinv[(long long)a.s * a.ldh + a.s + lane + 64 * i] : 0.0f;

  for (int nn = 0; nn < nb; ++nn) {
    const int n = a.s + nn;
    const int src = nn & 63, slot = nn >> 6;                                // the lane and register that hold column n
    // the next column's row of H^-1 goes out before the search
    float h_next[CPL];
#pragma unroll
    for (int i = 0; i < CPL; ++i) h_next[i] = (nn + 1 < nb && a.s + lane + 64 * i < a.s_end) ? a.Hinv[(long long)(n + 1) * a.ldh + a.s + lane + 64 * i] : 0.0f;
    const float hd = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(slot ? h[1] : h[0]), src));     // Hinv[n][n]
    float t[V];
#pragma unroll
    for (int j = 0; j < V; ++j) t[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(slot ? w[1][j] : w[0][j]), src));
    unsigned best, best_res = 0u;
    float q[V];
    if constexpr (IN_LDS) best = nearest<V, EH>(static_cast<const __half *>(tables), a.k, t, len, lane);
    else best = nearest<V, EH>(tab, a.k, t, len, lane);
    {
      __half c[EH];
      const __half *e = (IN_LDS ? static_cast<const __half *>(tables) : tab) + (long long)best * EH;
#pragma unroll
      for (int j = 0; j < V; ++j) c[j] = e[j];
#pragma unroll
      for (int j = 0; j < V; ++j) q[j] = __half2float(c[j]);
    }
    if (a.k_res) {
      float r[V];
#pragma unroll
      for (int j = 0; j < V; ++j) r[j] = __fsub_rn(t[j], q[j]);
      const __half *rt = IN_LDS ? static_cast<const __half *>(tables) + (long long)a.k * EH : tab_res;
      best_res = nearest<V, EH>(rt, a.k_res, r, len, lane);
#pragma unroll
      for (int j = 0; j < V; ++j) {
        // what inference restores: the binary32 sum of the two centroids, rounded to binary16 (Sec. 3.2.2)
        float sum = __fadd_rn(q[j], __half2float(rt[(long long)best_res * EH + j]));
        asm volatile("" : "+v"(sum));
        q[j] = __half2float(__float2half_rn(sum));
      }
    }
    float e[V];
#pragma unroll
    for (int j = 0; j < V; ++j) e[j] = j < len ? __fdiv_rn(__fsub_rn(t[j], q[j]), hd) : 0.0f;
    // spread over the block's later columns; column n itself becomes its quantized value
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int col = lane + 64 * i;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        if (col > nn) w[i][j] = __fmaf_rn(-e[j], h[i], w[i][j]);
        else if (col == nn) w[i][j] = q[j];
      }
      if (col == nn) { code[i] = best; code_res[i] = best_res; }
    }
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < V; ++j)
        if (j < len) {
          if (a.T) a.T[(long long)(m0 + j) * a.ldt + n] = t[j];
          a.E[(long long)(m0 + j) * QB + nn] = e[j];
        }
    }
#pragma unroll
    for (int i = 0; i < CPL; ++i) h[i] = h_next[i];
  }

  // the block's quantized columns, and their indices into the packed streams (one per column: stream p, position n;
  // the streams were cleared beforehand and no other wave touches stream p)
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = a.s + lane + 64 * i;
    if (c < a.s_end) {
#pragma unroll
      for (int j = 0; j < V; ++j)
        if (j < len) a.W[(long long)(m0 + j) * a.ldw + c] = w[i][j];
      {
        const unsigned long long bit = (unsigned long long)c * (unsigned)a.bits;
        unsigned *row = a.idx + (long long)p * a.idx_dwords + (bit >> 5);
        const unsigned sh = (unsigned)(bit & 31u);
        atomicOr(row, code[i] << sh);
        if (sh + a.bits > 32) atomicOr(row + 1, code[i] >> (32u - sh));
      }
      if (a.k_res) {
        const unsigned long long bit = (unsigned long long)c * (unsigned)a.bits_res;
        unsigned *row = a.idx_res + (long long)p * a.idx_res_dwords + (bit >> 5);
        const unsigned sh = (unsigned)(bit & 31u);
        atomicOr(row, code_res[i] << sh);
        if (sh + a.bits_res > 32) atomicOr(row + 1, code_res[i] >> (32u - sh));
      }
    }
  }
}

// Tables as padded entries, main then residual, one array (what the column kernel copies into LDS or reads in place).
__global__ __launch_bounds__(256) void pad_tables_kernel(const __half *__restrict__ cb, int k, const __half *__restrict__ cb_res, int k_res, int v, int eh,
                                                         __half *__restrict__ out) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= (k + k_res) * eh) return;
  const int entry = e / eh, j = e - entry * eh;
  __half val = __float2half_rn(0.0f);
  if (j < v) val = entry < k ? cb[(long long)entry * v + j] : cb_res[(long long)(entry - k) * v + j];
  out[e] = val;
}

__global__ __launch_bounds__(256) void clear_dwords_kernel(unsigned *p, long long stride_dwords, int dwords_per_row, int rows) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * dwords_per_row) return;
  const long long r = e / dwords_per_row;
  p[r * stride_dwords + (e - r * dwords_per_row)] = 0u;
}

// W[:, c0 ...] -= E[:, 0 .. nb) * Hinv[s .. s + nb, c0 ...]: one workgroup per 64 x 64 tile of W, a wave per 32 x 32 quarter,
// both operands through LDS, v_mfma_f32_32x32x2_f32 (lane l gives A[l & 31][l >> 5] and B[l >> 5][l & 31]; it gets back
// column l & 31 and, in register r, row 8 (r >> 2) + 4 (l >> 5) + (r & 3)).
__global__ __launch_bounds__(256) void qcol_trailing_kernel(float *__restrict__ W, long long ldw, int rows, int cols, const float *__restrict__ E,
                                                            const float *__restrict__ Hinv, long long ldh, int s, int nb, int c_first) {
  extern __shared__ __attribute__((aligned(16))) float tiles[];
  float (*As)[QB + 1] = reinterpret_cast<float (*)[QB + 1]>(tiles);                  // [64][QB + 1]
  float (*Bs)[64] = reinterpret_cast<float (*)[64]>(tiles + 64 * (QB + 1));         // [QB][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = blockIdx.y * 64, c0 = c_first + blockIdx.x * 64;
  for (int e = threadIdx.x; e < 64 * QB; e += 256) {
    const int r = e / QB, kk = e - r * QB;
    As[r][kk] = (r0 + r < rows && kk < nb) ? E[(long long)(r0 + r) * QB + kk] : 0.0f;
  }
  for (int e = threadIdx.x; e < QB * 64; e += 256) {
    const int kk = e >> 6, c = e & 63;
    Bs[kk][c] = (kk < nb && c0 + c < cols) ? Hinv[(long long)(s + kk) * ldh + c0 + c] : 0.0f;
  }
  __syncthreads();
  const int wr = (wave >> 1) * 32, wc = (wave & 1) * 32;
  float16v acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const int kmax = (nb + 1) & ~1;
  for (int kk = 0; kk < kmax; kk += 2)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[wr + (lane & 31)][kk + (lane >> 5)], Bs[kk + (lane >> 5)][wc + (lane & 31)], acc, 0, 0, 0);
  const int c = c0 + wc + (lane & 31);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = r0 + wr + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (row < rows && c < cols) W[(long long)row * ldw + c] -= acc[r];
  }
}

template <int V>
int launch_block(const QArgs &a, bool in_lds, unsigned lds_bytes, hipStream_t st) {
  const unsigned grid = (unsigned)(((a.rows + V - 1) / V + QW - 1) / QW);
  if (in_lds) {
    VQ_ALLOW_FULL_LDS((qcol_block_kernel<V, true>));
    hipLaunchKernelGGL((qcol_block_kernel<V, true>), dim3(grid), dim3(QW * 64), lds_bytes, st, a);
  } else {
    hipLaunchKernelGGL((qcol_block_kernel<V, false>), dim3(grid), dim3(QW * 64), 0, st, a);
  }
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Workspace: the block's errors E [rows][128] binary32, then both tables as padded entries.
size_t quantize_columns_workspace_bytes(int rows, int v, int k, int k_res) {
  const size_t e = ((size_t)rows * QB * sizeof(float) + 255) / 256 * 256;
  return e + ((size_t)(k + k_res) * entry_halfs(v) * sizeof(__half) + 255) / 256 * 256;
}

int launch_quantize_columns(float *W, long long ldw, int rows, int cols, const float *Hinv, long long ldh, const __half *cb, int v, int k,
                            const __half *cb_res, int k_res, int block, unsigned char *idx, long long idx_stride, unsigned char *idx_res,
                            long long idx_res_stride, float *T, long long ldt, void *workspace, hipStream_t st) {
  const int eh = entry_halfs(v);
  const int bits = index_bits(k), bits_res = k_res ? index_bits(k_res) : 0;
  const int S = (rows + v - 1) / v;
  float *E = static_cast<float *>(workspace);
  __half *padded = reinterpret_cast<__half *>(static_cast<unsigned char *>(workspace) + ((size_t)rows * QB * sizeof(float) + 255) / 256 * 256);
  const int n_pad = (k + k_res) * eh;
  hipLaunchKernelGGL(pad_tables_kernel, dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st, cb, k, cb_res, k_res, v, eh, padded);
  // every dword that holds one of a stream's cols * bits bits starts at zero (the column kernel ORs its indices in)
  const int dw = (int)(((long long)cols * bits + 31) / 32), dw_res = (int)(((long long)cols * bits_res + 31) / 32);
  hipLaunchKernelGGL(clear_dwords_kernel, dim3((unsigned)(((long long)S * dw + 255) / 256)), dim3(256), 0, st, reinterpret_cast<unsigned *>(idx),
                     idx_stride / 4, dw, S);
  if (k_res)
    hipLaunchKernelGGL(clear_dwords_kernel, dim3((unsigned)(((long long)S * dw_res + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<unsigned *>(idx_res), idx_res_stride / 4, dw_res, S);
  if (hipGetLastError() != hipSuccess) return VQ_ERR_HIP;
  const size_t table_bytes = (size_t)n_pad * sizeof(__half);
  const bool in_lds = table_bytes <= 150 * 1024;
  QArgs a{};
  a.W = W; a.ldw = ldw; a.rows = rows; a.cols = cols; a.Hinv = Hinv; a.ldh = ldh;
  a.cb = padded; a.k = k; a.cb_res = padded + (size_t)k * eh; a.k_res = k_res;
  a.idx = reinterpret_cast<unsigned *>(idx); a.idx_dwords = idx_stride / 4; a.bits = bits;
  a.idx_res = reinterpret_cast<unsigned *>(idx_res); a.idx_res_dwords = idx_res_stride / 4; a.bits_res = bits_res;
  a.T = T; a.ldt = ldt; a.E = E;
  for (int s = 0; s < cols; s += block) {
    a.s = s; a.s_end = s + block < cols ? s + block : cols;
    int rc = VQ_ERR_UNSUPPORTED;
    switch (v) {
#define VQ_CASE(V) case V: rc = launch_block<V>(a, in_lds, (unsigned)table_bytes, st); break;
      VQ_CASE(1) VQ_CASE(2) VQ_CASE(3) VQ_CASE(4) VQ_CASE(5) VQ_CASE(6) VQ_CASE(7) VQ_CASE(8)
      VQ_CASE(9) VQ_CASE(10) VQ_CASE(11) VQ_CASE(12) VQ_CASE(13) VQ_CASE(14) VQ_CASE(15) VQ_CASE(16)
#undef VQ_CASE
    }
    if (rc != VQ_OK) return rc;
    if (a.s_end < cols) {
      const unsigned gx = (unsigned)((cols - a.s_end + 63) / 64), gy = (unsigned)((rows + 63) / 64);
      if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
      VQ_ALLOW_FULL_LDS(qcol_trailing_kernel);
      hipLaunchKernelGGL(qcol_trailing_kernel, dim3(gx, gy), dim3(256), (64 * (QB + 1) + QB * 64) * sizeof(float), st, W, ldw, rows, cols, E, Hinv,
                         ldh, s, a.s_end - s, a.s_end);
      if (hipGetLastError() != hipSuccess) return VQ_ERR_HIP;
    }
  }
  return VQ_OK;
}

}  // namespace vq
