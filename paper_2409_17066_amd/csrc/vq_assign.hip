// vq_assign: the encode side of the lookup -- index of the nearest centroid of every length-v vector along the
// rows of a weight matrix (Eq. 2 of Sec. 2.2; with a base matrix, the residual stage's equation of Sec. 3.2.2),
// written as the packed index streams that vq_dequant / vq_gemv / vq_gemm read.
//
// The distance decides an integer, so its arithmetic is fixed (include/vq.h): binary32, t_j = W - B as one
// subtraction, per element one subtraction and one fused multiply-add into a sum that starts at +0, elements in
// ascending order, the first of equal distances wins.  That is 2 v + 3 vector-ALU instructions per (vector,
// centroid) pair and nothing else in the inner loop: the kernel is bound by the vector ALUs.
//
// Work split: a lane owns `seg` consecutive vectors of a row, seg = 8, 16 or 32 chosen so that they fill whole dwords of
// the row's index stream (lanes never share an output dword), and takes them VB at a time against the whole table, which sits in LDS as
// binary32 and is read with wave-uniform addresses (one broadcast read feeds VB x 64 distances).  Tables larger than
// the LDS chunk (k = 65536) are walked chunk by chunk with the running minimum kept in registers.  A row's last
// vector, when the row length is not a multiple of v, is compared over its own elements only; those few vectors
// go through a second, plain kernel (a wave per row) that inserts their bits into the stream afterwards.
#include "vq_common.hpp"

namespace vq {
namespace {

constexpr int AT = 1024;                 // threads per workgroup
constexpr unsigned LDS_TABLE_BYTES = 128u * 1024u;

constexpr int table_stride(int v) { return v <= 2 ? v : v <= 4 ? 4 : v <= 8 ? 8 : 16; }

template <int V, int VB>
__global__ __launch_bounds__(AT) void assign_kernel(const __half *__restrict__ W, const __half *__restrict__ B, long long ld, int rows,
                                                    int p_full, int p_all, const __half *__restrict__ codebook, int k, int bits,
                                                    int chunk, int seg_len, unsigned char *__restrict__ idx, long long idx_stride, int down_rows) {
  extern __shared__ __attribute__((aligned(16))) float table[];       // [chunk][TS]: rows padded to 16-byte reads
  constexpr int TS = table_stride(V);
  const int segs = (p_all + seg_len - 1) / seg_len;
  const long long item = (long long)blockIdx.x * AT + threadIdx.x;
  const bool live = item < (long long)rows * segs;
  const int o = live ? (int)(item / segs) : 0;
  const int seg = live ? (int)(item - (long long)o * segs) : 0;
  // down_rows > 0: the vectors run down the columns of a matrix of down_rows rows (Sec. 3.1, Algorithm 1).  "Row" o is then
  // the index stream of rows [o V, o V + V), its vector u is column u, element j of it sits in row o V + j; a stream whose
  // block of rows is cut off at the end of the matrix is left to the second kernel as a whole.
  const bool whole = down_rows == 0 || (o + 1) * V <= down_rows;
  unsigned *out = reinterpret_cast<unsigned *>(idx + (long long)o * idx_stride) + (long long)seg * (seg_len * bits / 32);
  unsigned long long buf = 0;
  int fill = 0;
  const int n_chunks = (k + chunk - 1) / chunk;
  auto stage = [&](int c0) {             // centroids [c0, c0 + chunk) as binary32; past k: never read
    const int n = min(chunk, k - c0) * V;
    for (int e = threadIdx.x; e < n; e += AT) table[(e / V) * TS + e % V] = __half2float(codebook[(long long)c0 * V + e]);
  };
  if (n_chunks == 1) { stage(0); __syncthreads(); }
  for (int r = 0; r < seg_len / VB; ++r) {                   // every lane walks every round: the barriers below need all of them
    const int p0 = seg * seg_len + r * VB;
    float t[VB][V], best[VB];
    int arg[VB];
#pragma unroll
    for (int u = 0; u < VB; ++u) {
      best[u] = __builtin_inff(); arg[u] = 0;
      const bool on = live && whole && p0 + u < p_full;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        const long long c = down_rows ? ((long long)o * V + j) * ld + (p0 + u) : (long long)o * ld + (long long)(p0 + u) * V + j;
        float x = on ? __half2float(W[c]) : 0.0f;
        if (on && B) x = __fsub_rn(x, __half2float(B[c]));
        t[u][j] = x;
      }
    }
    for (int ch = 0; ch < n_chunks; ++ch) {
      if (n_chunks > 1) { __syncthreads(); stage(ch * chunk); __syncthreads(); }
      const int n = min(chunk, k - ch * chunk);
#pragma unroll 2
      for (int i = 0; i < n; ++i) {
        float c[V];
#pragma unroll
        for (int j = 0; j < V; ++j) c[j] = table[i * TS + j];
#pragma unroll
        for (int u = 0; u < VB; ++u) {
          float d = 0.0f;
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float diff = __fsub_rn(t[u][j], c[j]);
            d = __fmaf_rn(diff, diff, d);
          }
          if (d < best[u]) { best[u] = d; arg[u] = ch * chunk + i; }
        }
      }
    }
    // append the round's indices to the lane's bit stream; a row's cut-off last vector gets zero bits here
#pragma unroll
    for (int u = 0; u < VB; ++u) {
      if (live && p0 + u < p_all) {
        const unsigned code = whole && p0 + u < p_full ? (unsigned)arg[u] : 0u;
        buf |= (unsigned long long)code << fill;
        fill += bits;
        if (fill >= 32) { *out++ = (unsigned)buf; buf >>= 32; fill -= 32; }
      }
    }
  }
  if (live && fill > 0) *out = (unsigned)buf;              // the row's last, partly filled dword: upper bits zero
}

// The cut-off last vector of every row (row length not a multiple of v): distance over its `len` elements only.
// One wave per row: lane l takes centroids l, l + 64, ... in ascending order (strict "less" keeps the lowest index of
// equal distances among its own), then the lanes meet with the same rule -- smaller distance, else smaller index.
// Runs after assign_kernel on the same stream and sets the vector's bits, which that kernel left zero.
__global__ __launch_bounds__(256) void assign_tail_kernel(const __half *__restrict__ W, const __half *__restrict__ B, long long ld, int rows,
                                                          int p_full, int v, int len, const __half *__restrict__ codebook, int k, int bits,
                                                          unsigned char *__restrict__ idx, long long idx_stride) {
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (o >= rows) return;
  float t[16];
  for (int j = 0; j < len; ++j) {
    const long long c = (long long)o * ld + (long long)p_full * v + j;
    float x = __half2float(W[c]);
    if (B) x = __fsub_rn(x, __half2float(B[c]));
    t[j] = x;
  }
  float best = __builtin_inff();
  unsigned arg = 0xFFFFFFFFu;                                // a lane without centroids (k < 64) never wins
  for (int i = lane; i < k; i += 64) {
    float d = 0.0f;
    for (int j = 0; j < len; ++j) {
      const float diff = __fsub_rn(t[j], __half2float(codebook[(long long)i * v + j]));
      d = __fmaf_rn(diff, diff, d);
    }
    if (d < best || arg == 0xFFFFFFFFu) { best = d; arg = (unsigned)i; }
  }
  for (int s = 32; s > 0; s >>= 1) {
    const float od = __shfl_xor(best, s, 64);
    const unsigned oa = __shfl_xor(arg, s, 64);
    if (oa != 0xFFFFFFFFu && (arg == 0xFFFFFFFFu || od < best || (od == best && oa < arg))) { best = od; arg = oa; }
  }
  if (lane != 0) return;
  unsigned *row = reinterpret_cast<unsigned *>(idx + (long long)o * idx_stride);
  const long long bit = (long long)p_full * bits;
  const int sh = (int)(bit & 31);
  row[bit >> 5] |= arg << sh;
  if (sh + bits > 32) row[(bit >> 5) + 1] |= arg >> (32 - sh);
}

// The cut-off last block of rows when the vectors run down the columns: every vector of the last index stream has only
// `len` elements.  One wave per column, as above; the streams' bits are set with an atomic OR because neighbouring columns
// share dwords (integer, so the result does not depend on the order).
__global__ __launch_bounds__(256) void assign_tail_down_kernel(const __half *__restrict__ W, const __half *__restrict__ B, long long ld, int cols,
                                                               int row0, int v, int len, const __half *__restrict__ codebook, int k, int bits,
                                                               unsigned *__restrict__ stream) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= cols) return;
  float t[16];
  for (int j = 0; j < len; ++j) {
    const long long c = (long long)(row0 + j) * ld + n;
    float x = __half2float(W[c]);
    if (B) x = __fsub_rn(x, __half2float(B[c]));
    t[j] = x;
  }
  float best = __builtin_inff();
  unsigned arg = 0xFFFFFFFFu;
  for (int i = lane; i < k; i += 64) {
    float d = 0.0f;
    for (int j = 0; j < len; ++j) {
      const float diff = __fsub_rn(t[j], __half2float(codebook[(long long)i * v + j]));
      d = __fmaf_rn(diff, diff, d);
    }
    if (d < best || arg == 0xFFFFFFFFu) { best = d; arg = (unsigned)i; }
  }
  for (int s = 32; s > 0; s >>= 1) {
    const float od = __shfl_xor(best, s, 64);
    const unsigned oa = __shfl_xor(arg, s, 64);
    if (oa != 0xFFFFFFFFu && (arg == 0xFFFFFFFFu || od < best || (od == best && oa < arg))) { best = od; arg = oa; }
  }
  if (lane != 0) return;
  const long long bit = (long long)n * bits;
  const int sh = (int)(bit & 31);
  atomicOr(stream + (bit >> 5), arg << sh);
  if (sh + bits > 32) atomicOr(stream + (bit >> 5) + 1, arg >> (32 - sh));
}

template <int V>
int launch_v(const __half *W, const __half *B, long long ld, int rows, int p_full, int p_all, const __half *codebook, int k, int bits,
             unsigned char *idx, long long idx_stride, hipStream_t s, int down_rows = 0) {
  constexpr int VB = V <= 8 ? 8 : 4;       // vectors a lane holds at once: each centroid read from LDS serves VB x 64 distances
  auto kernel = assign_kernel<V, VB>;
  VQ_ALLOW_FULL_LDS(kernel);
  const int chunk = min(k, (int)(LDS_TABLE_BYTES / (table_stride(V) * sizeof(float))));
  // vectors per lane: the fewest (most lanes) whose bits fill whole dwords
  const int seg_len = bits % 4 == 0 ? 8 : bits % 2 == 0 ? 16 : 32;
  const long long items = (long long)rows * ((p_all + seg_len - 1) / seg_len);
  const long long blocks = (items + AT - 1) / AT;
  if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(AT), (size_t)chunk * table_stride(V) * sizeof(float), s, W, B, ld, rows, p_full, p_all,
                     codebook, k, bits, chunk, seg_len, idx, idx_stride, down_rows);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

int launch_assign(const __half *W, const __half *B, long long ld, int rows, int cols, const __half *codebook, int v, int k,
                  unsigned char *idx, long long idx_stride, hipStream_t s) {
  const int bits = index_bits(k);
  const int p_full = cols / v, p_all = (cols + v - 1) / v;
  int rc = VQ_ERR_UNSUPPORTED;
  switch (v) {
#define VQ_V(N) case N: rc = launch_v<N>(W, B, ld, rows, p_full, p_all, codebook, k, bits, idx, idx_stride, s); break;
    VQ_V(1) VQ_V(2) VQ_V(3) VQ_V(4) VQ_V(5) VQ_V(6) VQ_V(7) VQ_V(8) VQ_V(9) VQ_V(10) VQ_V(11) VQ_V(12) VQ_V(13) VQ_V(14) VQ_V(15) VQ_V(16)
#undef VQ_V
    default: break;
  }
  if (rc != VQ_OK || p_all == p_full) return rc;
  hipLaunchKernelGGL(assign_tail_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, W, B, ld, rows, p_full, v, cols - p_full * v,
                     codebook, k, bits, idx, idx_stride);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// Vectors down the columns of W [rows][ld]: index streams [ceil(rows / v)][idx_stride], one index per column.
int launch_assign_down(const __half *W, const __half *B, long long ld, int rows, int cols, const __half *codebook, int v, int k,
                       unsigned char *idx, long long idx_stride, hipStream_t s) {
  const int bits = index_bits(k);
  const int streams = (rows + v - 1) / v;
  int rc = VQ_ERR_UNSUPPORTED;
  switch (v) {
#define VQ_V(N) case N: rc = launch_v<N>(W, B, ld, streams, cols, cols, codebook, k, bits, idx, idx_stride, s, rows); break;
    VQ_V(1) VQ_V(2) VQ_V(3) VQ_V(4) VQ_V(5) VQ_V(6) VQ_V(7) VQ_V(8) VQ_V(9) VQ_V(10) VQ_V(11) VQ_V(12) VQ_V(13) VQ_V(14) VQ_V(15) VQ_V(16)
#undef VQ_V
    default: break;
  }
  if (rc != VQ_OK || rows % v == 0) return rc;
  hipLaunchKernelGGL(assign_tail_down_kernel, dim3((unsigned)((cols + 3) / 4)), dim3(256), 0, s, W, B, ld, cols, (streams - 1) * v, v,
                     rows - (streams - 1) * v, codebook, k, bits, reinterpret_cast<unsigned *>(idx + (long long)(streams - 1) * idx_stride));
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace vq
