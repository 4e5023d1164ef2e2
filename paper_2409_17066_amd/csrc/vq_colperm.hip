// Column order of a layer whose stored columns are a permutation of its own (Sec. 3.2.3 "Outlier Elimination": the columns
// that get the outlier codebook are picked by the Hessian's diagonal and stored first; Algorithm 2's outlier step): the two
// data movements that let every other kernel of the library work in stored order.
#include "vq_common.hpp"

namespace vq {

namespace {

typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// dst[t][c] = src[t][perm[c]]: the activations in the stored order of the columns.  One thread per pair of columns;
// entries of perm outside the row read as zero; the pad columns [cols, ld_dst) of dst are cleared when ld_dst - cols < 8.
__global__ __launch_bounds__(256) void gather_cols_kernel(const __half *__restrict__ src, long long ld_src, int cols, const int *__restrict__ perm,
                                                          __half *__restrict__ dst, long long ld_dst, int dst_cols) {
  const int c = (blockIdx.x * 256 + threadIdx.x) * 2;
  if (c >= dst_cols) return;
  const __half *srow = src + (long long)blockIdx.y * ld_src;
  unsigned short h[2] = {0, 0};
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if (c + j < cols) {
      const int t = perm[c + j];
      if ((unsigned)t < (unsigned)cols) h[j] = __half_as_ushort(srow[t]);
    }
  }
  // dst rows start 4-byte aligned and c is even
  *reinterpret_cast<unsigned *>(dst + (long long)blockIdx.y * ld_dst + c) = (unsigned)h[0] | ((unsigned)h[1] << 16);
}

// W[o][perm[c]] = W[o][c] for every c < cols, one workgroup per row: the row goes to its new places in LDS, and comes
// back in order.  wide: W 16-byte aligned and ldw % 8 == 0, so rows move in 16-byte pieces (the tail in single elements).
__global__ __launch_bounds__(1024) void place_cols_kernel(__half *__restrict__ W, long long ldw, int cols, const int *__restrict__ perm, int wide) {
  extern __shared__ __attribute__((aligned(16))) __half row[];
  __half *w = W + (long long)blockIdx.x * ldw;
  const int body = wide ? cols & ~7 : 0;
  for (int c = (int)threadIdx.x * 8; c < body; c += 1024 * 8) {
    const uint4v v = *reinterpret_cast<const uint4v *>(w + c);
    const uint4v t0 = *reinterpret_cast<const uint4v *>(perm + c), t1 = *reinterpret_cast<const uint4v *>(perm + c + 4);
    const unsigned t[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
    const unsigned d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (t[j] < (unsigned)cols) row[t[j]] = __ushort_as_half((unsigned short)(d[j >> 1] >> ((j & 1) * 16)));
  }
  for (int c = body + (int)threadIdx.x; c < cols; c += 1024) {
    const unsigned t = (unsigned)perm[c];
    if (t < (unsigned)cols) row[t] = w[c];
  }
  __syncthreads();
  for (int c = (int)threadIdx.x * 8; c < body; c += 1024 * 8) *reinterpret_cast<uint4v *>(w + c) = *reinterpret_cast<const uint4v *>(row + c);
  for (int c = body + (int)threadIdx.x; c < cols; c += 1024) w[c] = row[c];
}

}  // namespace

int launch_gather_cols(const __half *src, long long ld_src, int rows, int cols, const int *perm, __half *dst, long long ld_dst, hipStream_t s) {
  if (rows < 1 || rows > 65535 || (ld_dst & 1) || (reinterpret_cast<uintptr_t>(dst) & 3)) return VQ_ERR_UNSUPPORTED;
  const int dst_cols = ld_dst - cols < 8 ? (int)ld_dst : cols + (cols & 1);     // whole pairs; the pad of a row rounded up to 8
  if (dst_cols > ld_dst) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(gather_cols_kernel, dim3((unsigned)((dst_cols + 511) / 512), (unsigned)rows), dim3(256), 0, s, src, ld_src, cols, perm, dst,
                     ld_dst, dst_cols);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

int launch_place_cols(__half *W, long long ldw, int rows, int cols, const int *perm, hipStream_t s) {
  const unsigned lds = (unsigned)(((long long)cols * 2 + 15) & ~15LL);
  if ((long long)cols * 2 > 160 * 1024) return VQ_ERR_UNSUPPORTED;
  VQ_ALLOW_FULL_LDS(place_cols_kernel);
  const int wide = (reinterpret_cast<uintptr_t>(W) & 15) == 0 && (ldw & 7) == 0 && (reinterpret_cast<uintptr_t>(perm) & 15) == 0;
  hipLaunchKernelGGL(place_cols_kernel, dim3((unsigned)rows), dim3(1024), lds, s, W, ldw, cols, perm, wide);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace vq
