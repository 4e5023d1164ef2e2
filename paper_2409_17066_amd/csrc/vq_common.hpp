// Shared host/device declarations of the gfx950 VQ linear-layer library (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include "../../include/vq.h"

namespace vq {

// Layer parameters in the form kernels take by value.
struct Params {
  int out_features, in_features;
  int v, k, bits;
  int k_res, bits_res;
  int n_out, v_out, k_out, bits_out;
  int P, Q;                      // main / outlier vectors per row
  int Pg, n_groups;              // vectors per codebook group (P if there is one group), groups; tables are [group][k][v]
  int orientation;               // 0: a vector covers v input columns of one row; 1: v output rows of one column
  int S, S_out;                  // index streams (main / outlier): out_features, or ceil(out_features / v) with orientation 1;
                                 // P and Q are then the indices per stream (main columns / outlier columns)
  const __half *cb, *cb_res, *cb_out;
  const uint8_t *idx, *idx_res, *idx_out;
  long long stride, stride_res, stride_out;   // bytes per row of each stream
  const __half *scale, *bias;
  const int *perm;               // stored column c is column perm[c] of the layer (Sec. 3.2.3); nullptr: the identity
};

// Lets a kernel use the whole 160 KB of LDS: once per kernel and process (a function-local static: thread-safe).
#define VQ_ALLOW_FULL_LDS(kernel)                                                                                        \
  do {                                                                                                                   \
    static const hipError_t vq_cfg_ = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),                        \
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);       \
    if (vq_cfg_ != hipSuccess) return VQ_ERR_HIP;                                                                        \
  } while (0)

// Compute units of the current device (looked up once; 256 when the runtime does not say).
int cu_count();

// Test and measurement switches, all in the environment variable VQ_SWITCHES as name=value pairs separated by commas; read
// once at the start of every entry-point call (one getenv), so that one process can walk through all of them:
//   gemv=g|m|d   generic kernels only / the matrix-core kernels wherever they take the layer / the dot-product kernels
//   groups=loop  layers with codebook groups: every workgroup walks all groups even when a workspace is there
//   multi=0      vq_gemv_multi as one vq_gemv after the other
//   gemm=g|f|w|r|6 vq_gemm: generic tile kernel / no restore-then-multiply / restore-then-multiply whenever a workspace is
//                there / rows through vq_gemv / the on-the-fly kernel for v = 6 layers at every token count
//   dense=0|1    the dense product of the restore-then-multiply route: never / always the 256 x 256 tile kernel
//   dequant=g|s  vq_dequant: generic kernel / never the wide-store kernel (v = 6); two passes with a read-back instead of residual
//                entries from memory where two tables do not fit LDS together (the other settings)
struct Switches {
  char gemv = 0, gemm = 0, dequant = 0;
  bool groups_loop = false, multi_off = false;
  int dense = -1;
};
const Switches &switches();
void read_switches();

inline int index_bits(int k) { int b = 1; while ((1 << b) < k) ++b; return b; }

// Host-side validation shared by the entry points; fills `p` on success.
int make_params(const vq_layer_desc *d, Params *p);

// Kernel launchers (each returns a vq_status).
int launch_dequant(const Params &p, __half *W, long long ldw, hipStream_t s);
int launch_dequant_outliers(const Params &p, __half *W, long long ldw, hipStream_t s);   // generic kernel, outlier columns of a row-wise layer only
int launch_gemv(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
bool gemv_has_fast_kernel(const Params &p, const __half *x, long long ldx);
size_t gemv_workspace_bytes(const Params &p, const __half *x, long long ldx, int batch);
int launch_gemv_ws(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, void *workspace,
                   size_t workspace_bytes, hipStream_t s);
int launch_gemv_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys, const long long *ldys,
                      hipStream_t s);
int launch_gemm(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy,
                void *workspace, size_t workspace_bytes, hipStream_t s);
int launch_assign(const __half *W, const __half *B, long long ld, int rows, int cols, const __half *codebook, int v, int k,
                  unsigned char *idx, long long idx_stride, hipStream_t s);
int launch_assign_down(const __half *W, const __half *B, long long ld, int rows, int cols, const __half *codebook, int v, int k,
                       unsigned char *idx, long long idx_stride, hipStream_t s);
// Column order (Sec. 3.2.3): dst[t][c] = src[t][perm[c]] for c < cols (entries outside [0, cols) give zero), dst rows
// ld_dst halfs apart; and the inverse on a matrix restored in stored order: W[o][perm[c]] = W_stored[o][c], row by row
// through LDS, in place (VQ_ERR_UNSUPPORTED when a row does not fit LDS).
int launch_gather_cols(const __half *src, long long ld_src, int rows, int cols, const int *perm, __half *dst, long long ld_dst, hipStream_t s);
int launch_place_cols(__half *W, long long ldw, int rows, int cols, const int *perm, hipStream_t s);
size_t quantize_columns_workspace_bytes(int rows, int v, int k, int k_res);
int launch_quantize_columns(float *W, long long ldw, int rows, int cols, const float *Hinv, long long ldh, const __half *cb, int v, int k,
                            const __half *cb_res, int k_res, int block, unsigned char *idx, long long idx_stride, unsigned char *idx_res,
                            long long idx_res_stride, float *T, long long ldt, void *workspace, hipStream_t st);
size_t gemm_workspace_bytes(const Params &p, int tokens);
size_t gemm_fast_workspace_bytes(const Params &p, int tokens);

#ifdef __HIPCC__
// Index p of a row's little-endian bitstream (bits <= 16).  `row` is 4-byte aligned and the row's
// stride covers every dword that holds one of its P*bits bits, so both loads stay inside the row.
__device__ __forceinline__ unsigned load_index(const uint8_t *row, long long p, int bits) {
  const long long bit = p * bits;
  const unsigned *w = reinterpret_cast<const unsigned *>(row) + (bit >> 5);
  const int sh = (int)(bit & 31);
  unsigned lo = w[0] >> sh;
  if (sh + bits > 32) lo |= w[1] << (32 - sh);
  return lo & ((1u << bits) - 1u);
}

// The bit-exact restore of one weight: binary32 add of centroids happens at the caller, then one
// binary32 fma and one round-to-nearest-even conversion to binary16 (Sec. 2.2 lookup, Sec. 3.2.2 sum
// of tables).  The empty asm keeps the compiler from merging fma and conversion into the mixed-
// precision fma (v_fma_mixlo_f16), which rounds the exact result once, straight to binary16, and so
// differs from the two-step definition on double-rounding cases.
__device__ __forceinline__ __half restore(float d, float scale, float bias) {
  float w32 = __fmaf_rn(scale, d, bias);
  asm volatile("" : "+v"(w32));
  return __float2half_rn(w32);
}

// Touch the first `LINES` 64-byte lines of the kernel-argument segment with independent scalar loads.  The
// compiler loads arguments lazily, a few at a time, each group waiting for its own miss in the scalar cache
// (the segment is written by the host just before the launch); issuing one load per line up front overlaps
// those misses, and the later argument loads hit.
template <int LINES = 4>
__device__ __forceinline__ void warm_kernel_arguments() {      // the first LINES (4 or 5) lines of 64 bytes
#if defined(__HIP_DEVICE_COMPILE__)
  const auto ka = __builtin_amdgcn_kernarg_segment_ptr();
  unsigned a, b, c, d, e;
  if constexpr (LINES >= 5) asm volatile("s_load_dword %0, %1, 0x100" : "=&s"(e) : "s"(ka) : "memory");
  asm volatile("s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %4, 0x40\n\ts_load_dword %2, %4, 0x80\n\t"
               "s_load_dword %3, %4, 0xc0\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(a), "=&s"(b), "=&s"(c), "=&s"(d) : "s"(ka) : "memory");
#endif
}

// Sum over the 64 lanes of a wave, in every lane: DPP adds (within quads, half rows, rows, then across rows into lane 63)
// and one broadcast -- a sixth of what the same butterfly costs through ds_bpermute.  All 64 lanes must be active.
__device__ __forceinline__ float wave_sum(float x) {
#define VQ_DPP_ADD(CTRL, ROWS) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROWS, 0xF, false))
  VQ_DPP_ADD(0xB1, 0xF);     // quad_perm [1,0,3,2]
  VQ_DPP_ADD(0x4E, 0xF);     // quad_perm [2,3,0,1]
  VQ_DPP_ADD(0x141, 0xF);    // row_half_mirror
  VQ_DPP_ADD(0x140, 0xF);    // row_mirror
  VQ_DPP_ADD(0x142, 0xA);    // row_bcast15 into rows 1 and 3
  VQ_DPP_ADD(0x143, 0xC);    // row_bcast31 into rows 2 and 3
#undef VQ_DPP_ADD
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
#endif

}  // namespace vq
