// vq_gemv fast path for the paper's main decode setting: v = 6, 12-bit indices (k <= 4096), optional
// residual codebook with 12- or 8-bit indices, optional outlier columns with v = 4 and 12-bit indices
// (App. "Parameter Description"; Table "Quantization parameters").  Batch 1, 2 or 4 per launch.
//
// One workgroup of 16 waves per compute unit keeps every codebook in LDS (entries padded to 16 bytes so
// one ds_read_b128 fetches a centroid).  A wave owns a fixed column slice of the layer: each lane keeps
// the activations of its U consecutive vectors in registers for the whole kernel and walks down the
// rows.  Per row a lane loads its 12*U index bits as one unaligned dword window (bounds-checked buffer
// loads), funnel-shifts it to bit 0, extracts the indices, gathers the centroids from LDS and
// accumulates with v_dot2_f32_f16.  Row sums are reduced across the wave with DPP and across slices
// through a small LDS array; scale and bias are applied once per row as y = s * sum(d x) + b * sum(x).
#include "vq_common.hpp"

namespace vq {

namespace {

constexpr int NW = 16;           // waves per workgroup
constexpr int RC = 32;           // rows per reduction chunk
constexpr int MAX_SLICES = 16;
constexpr int NDW = 8;           // dwords in an index window

struct GemvPlan {
  int W, U;                      // main slices per row, vectors per lane
  int Wo, Uo;                    // outlier slices per row, outlier vectors per lane
  int RS;                        // row streams (rows in flight) for the main waves
  int rows_per_wg;
  unsigned lds_res, lds_out, lds_part, lds_xsum;   // byte offsets into dynamic LDS (main table at 0)
};

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dot2(unsigned a, unsigned b, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b), c, false);
}

__device__ __forceinline__ float dpp_add(float v, const int ctrl, const int row_mask) {
  // v + (lane-permuted v); lanes whose row is masked out add 0
  int moved;
  switch (ctrl) {   // the builtin wants literal control words
    case 0xB1: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false); break;
    case 0x4E: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false); break;
    case 0x141: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false); break;
    case 0x140: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false); break;
    case 0x142: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false); break;
    default: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false); break;
  }
  (void)row_mask;
  return v + __builtin_bit_cast(float, moved);
}

// Sum over the 64 lanes of a wave; the total lands in lane 63.
__device__ __forceinline__ float wave_reduce_to_lane63(float v) {
  v = dpp_add(v, 0xB1, 0xF);    // quad_perm [1,0,3,2]
  v = dpp_add(v, 0x4E, 0xF);    // quad_perm [2,3,0,1]
  v = dpp_add(v, 0x141, 0xF);   // row_half_mirror
  v = dpp_add(v, 0x140, 0xF);   // row_mirror: every lane of a 16-lane row now holds the row's sum
  v = dpp_add(v, 0x142, 0xA);   // row_bcast15 into rows 1 and 3
  v = dpp_add(v, 0x143, 0xC);   // row_bcast31 into rows 2 and 3
  return v;
}

// Index window of one lane: NDW dwords starting at dword `dw` of the row at byte offset `row_off`.
struct Window { unsigned w[NDW]; };

__device__ __forceinline__ Window load_window(__amdgpu_buffer_rsrc_t rsrc, unsigned row_off, unsigned dw) {
  Window r;
  const unsigned off = row_off + dw * 4u;
  uint4v a = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
  uint4v b = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off + 16u, 0, 0);
  r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z; r.w[3] = a.w;
  r.w[4] = b.x; r.w[5] = b.y; r.w[6] = b.z; r.w[7] = b.w;
  return r;
}

// Shift the window right by `sh` bits (0..31) so that the lane's first index starts at bit 0.
__device__ __forceinline__ void normalize(Window &win, unsigned sh) {
#pragma unroll
  for (int i = 0; i < NDW - 1; ++i) win.w[i] = __builtin_amdgcn_alignbit(win.w[i + 1], win.w[i], sh);
  win.w[NDW - 1] >>= sh;
}

// Byte offset (index * 16 or index * 8) of field u of a normalized window of BITS-bit fields.
template <int BITS, int SHIFT>
__device__ __forceinline__ unsigned field_offset(const Window &win, int u) {
  const int bit = u * BITS, i = bit >> 5, o = bit & 31;
  unsigned v = (o + BITS <= 32) ? (win.w[i] >> o) : __builtin_amdgcn_alignbit(win.w[i + 1], win.w[i], o);
  return (v & ((1u << BITS) - 1u)) << SHIFT;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// Copy a table of `k` entries of V halfs (V = 6 -> 16-byte LDS entries, V = 4 -> 8-byte entries).
template <int V>
__device__ __forceinline__ void stage_table(const __half *src, int k, int k_alloc, unsigned char *dst) {
  const unsigned *s = reinterpret_cast<const unsigned *>(src);
  for (int e = threadIdx.x; e < k_alloc; e += NW * 64) {
    if (V == 6) {
      uint4 val = make_uint4(0, 0, 0, 0);
      if (e < k) { val.x = s[e * 3]; val.y = s[e * 3 + 1]; val.z = s[e * 3 + 2]; }
      *reinterpret_cast<uint4 *>(dst + e * 16) = val;
    } else {
      uint2 val = make_uint2(0, 0);
      if (e < k) { val.x = s[e * 2]; val.y = s[e * 2 + 1]; }
      *reinterpret_cast<uint2 *>(dst + e * 8) = val;
    }
  }
}

// Activations of `n` halfs starting at column c as packed pairs; columns >= in_features read as zero.
__device__ __forceinline__ unsigned load_x_pair(const __half *xrow, int c, int in_features) {
  if (c + 1 < in_features) return *reinterpret_cast<const unsigned *>(xrow + c);
  if (c < in_features) return (unsigned)__half_as_ushort(xrow[c]);
  return 0u;
}

template <int RES_BITS, int B, int UMAX>
__global__ __launch_bounds__(NW * 64) void gemv_v6_kernel(Params p, GemvPlan plan, const __half *__restrict__ x, long long ldx,
                                                          __half *__restrict__ y, long long ldy) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = blockIdx.x * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const int Wt = plan.W + plan.Wo;
  float *part = reinterpret_cast<float *>(lds + plan.lds_part);     // [RC][Wt][B]
  float *xsum = reinterpret_cast<float *>(lds + plan.lds_xsum);     // [B]

  // ---- stage codebooks, sum activations
  stage_table<6>(p.cb, p.k, 4096, lds);
  if (RES_BITS) stage_table<6>(p.cb_res, p.k_res, 1 << RES_BITS, lds + plan.lds_res);
  if (plan.Wo) stage_table<4>(p.cb_out, p.k_out, 4096, lds + plan.lds_out);
  if (wv < B) {
    float s = 0.0f;
    for (int c = lane; c < p.in_features; c += 64) s += __half2float(x[wv * ldx + c]);
    s = wave_reduce_to_lane63(s);
    if (lane == 63) xsum[wv] = s;
  }

  // ---- role of this wave
  const int n_main = plan.RS * plan.W;
  const bool is_main = wv < n_main;
  const bool is_out = !is_main && (wv - n_main) < plan.Wo;
  const int slice = is_main ? wv % plan.W : wv - n_main;
  const int stream = is_main ? wv / plan.W : 0;
  const int step = is_main ? plan.RS : 1;
  const int U = is_main ? plan.U : plan.Uo;

  // ---- activations of this lane's vectors, kept for the whole kernel
  unsigned xr[B][UMAX][3];
  const int first_vec = (slice * 64 + lane) * U;
#pragma unroll
  for (int u = 0; u < UMAX; ++u)
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
      for (int h = 0; h < 3; ++h) xr[b][u][h] = 0u;
  if (is_main) {
#pragma unroll
    for (int u = 0; u < UMAX; ++u)
      if (u < U && first_vec + u < p.P) {
        const int c = p.n_out + (first_vec + u) * 6;
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
          for (int h = 0; h < 3; ++h) xr[b][u][h] = load_x_pair(x + b * ldx, c + 2 * h, p.in_features);
      }
  } else if (is_out) {
#pragma unroll
    for (int u = 0; u < UMAX; ++u)
      if (u < U && first_vec + u < p.Q) {
        const int c = (first_vec + u) * 4;
#pragma unroll
        for (int b = 0; b < B; ++b)
#pragma unroll
          for (int h = 0; h < 2; ++h) xr[b][u][h] = load_x_pair(x + b * ldx, c + 2 * h, p.in_features);
      }
  }
  __syncthreads();

  // ---- index stream geometry of this lane
  const unsigned rows_here = (unsigned)(row1 - row0);
  const unsigned char *lds_res = lds + plan.lds_res;
  const unsigned char *lds_out = lds + plan.lds_out;
  const unsigned bit0 = (unsigned)first_vec * 12u;
  const unsigned dw_main = bit0 >> 5, sh_main = bit0 & 31u;
  const unsigned bitr = (unsigned)first_vec * (unsigned)(RES_BITS ? RES_BITS : 1);
  const unsigned dw_res = bitr >> 5, sh_res = bitr & 31u;
  const __amdgpu_buffer_rsrc_t r_main = make_rsrc(p.idx + (long long)row0 * p.stride, rows_here * (unsigned)p.stride);
  const __amdgpu_buffer_rsrc_t r_res = make_rsrc(RES_BITS ? p.idx_res + (long long)row0 * p.stride_res : p.idx,
                                                 RES_BITS ? rows_here * (unsigned)p.stride_res : 0u);
  const __amdgpu_buffer_rsrc_t r_out = make_rsrc(plan.Wo ? p.idx_out + (long long)row0 * p.stride_out : p.idx,
                                                 plan.Wo ? rows_here * (unsigned)p.stride_out : 0u);

  for (int chunk0 = 0; chunk0 < (int)rows_here; chunk0 += RC) {
    const int rows_chunk = min(RC, (int)rows_here - chunk0);
    if (is_main) {
      for (int rl = stream; rl < rows_chunk; rl += step) {
        const unsigned r = (unsigned)(chunk0 + rl);
        Window wm = load_window(r_main, r * (unsigned)p.stride, dw_main);
        Window wr;
        if (RES_BITS) wr = load_window(r_res, r * (unsigned)p.stride_res, dw_res);
        normalize(wm, sh_main);
        if (RES_BITS) normalize(wr, sh_res);
        float acc[B];
#pragma unroll
        for (int b = 0; b < B; ++b) acc[b] = 0.0f;
#pragma unroll
        for (int u = 0; u < UMAX; ++u) {
          if (u < U) {
            const uint4 e = *reinterpret_cast<const uint4 *>(lds + field_offset<12, 4>(wm, u));
#pragma unroll
            for (int b = 0; b < B; ++b) {
              acc[b] = dot2(e.x, xr[b][u][0], acc[b]);
              acc[b] = dot2(e.y, xr[b][u][1], acc[b]);
              acc[b] = dot2(e.z, xr[b][u][2], acc[b]);
            }
            if (RES_BITS) {
              const uint4 f = *reinterpret_cast<const uint4 *>(lds_res + field_offset<(RES_BITS ? RES_BITS : 8), 4>(wr, u));
#pragma unroll
              for (int b = 0; b < B; ++b) {
                acc[b] = dot2(f.x, xr[b][u][0], acc[b]);
                acc[b] = dot2(f.y, xr[b][u][1], acc[b]);
                acc[b] = dot2(f.z, xr[b][u][2], acc[b]);
              }
            }
          }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
          const float s = wave_reduce_to_lane63(acc[b]);
          if (lane == 63) part[(rl * Wt + slice) * B + b] = s;
        }
      }
    } else if (is_out) {
      for (int rl = 0; rl < rows_chunk; ++rl) {
        const unsigned r = (unsigned)(chunk0 + rl);
        Window wo = load_window(r_out, r * (unsigned)p.stride_out, dw_main);
        normalize(wo, sh_main);
        float acc[B];
#pragma unroll
        for (int b = 0; b < B; ++b) acc[b] = 0.0f;
#pragma unroll
        for (int u = 0; u < UMAX; ++u) {
          if (u < U) {
            const uint2 e = *reinterpret_cast<const uint2 *>(lds_out + field_offset<12, 3>(wo, u));
#pragma unroll
            for (int b = 0; b < B; ++b) {
              acc[b] = dot2(e.x, xr[b][u][0], acc[b]);
              acc[b] = dot2(e.y, xr[b][u][1], acc[b]);
            }
          }
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
          const float s = wave_reduce_to_lane63(acc[b]);
          if (lane == 63) part[(rl * Wt + plan.W + slice) * B + b] = s;
        }
      }
    }
    __syncthreads();
    // ---- combine slices, apply scale and bias, store
    for (int t = threadIdx.x; t < rows_chunk * B; t += NW * 64) {
      const int rl = t / B, b = t - rl * B;
      const int o = row0 + chunk0 + rl;
      float s = 0.0f;
      for (int w = 0; w < Wt; ++w) s += part[(rl * Wt + w) * B + b];
      const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f;
      const float bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
      y[b * ldy + o] = __float2half_rn(__fmaf_rn(sc, s, bi * xsum[b]));
    }
    __syncthreads();
  }
}

int g_cu_count = 0;

int cu_count() {
  if (g_cu_count == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    g_cu_count = n;
  }
  return g_cu_count;
}

template <int RES_BITS, int B, int UMAX>
int launch_one(const Params &p, const GemvPlan &plan, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx,
               __half *y, long long ldy, hipStream_t s) {
  static bool configured = false;
  auto kernel = gemv_v6_kernel<RES_BITS, B, UMAX>;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return VQ_ERR_HIP;
    configured = true;
  }
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds_bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Whether the fast kernels take this layer and these buffers.
bool gemv_fast_applicable(const Params &p, const __half *x, long long ldx) {
  if (p.v != 6 || p.bits != 12) return false;
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return false;
  if (p.n_out && (p.v_out != 4 || p.bits_out != 12)) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 3) || (ldx & 1)) return false;
  if (p.Q > 64 * 16 * 4) return false;
  const long long max_stride = p.stride > p.stride_res ? p.stride : p.stride_res;
  if (max_stride > (1 << 24)) return false;
  return true;
}

// Launch for one group of 1, 2 or 4 batch rows.
int launch_gemv_fast(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  const int umax = batch == 1 ? 16 : batch == 2 ? 8 : 4;
  GemvPlan plan{};
  const int ncu = cu_count();
  plan.Uo = 0; plan.Wo = 0;
  if (p.Q) {
    plan.Wo = (p.Q + 64 * umax - 1) / (64 * umax);
    plan.Uo = (p.Q + 64 * plan.Wo - 1) / (64 * plan.Wo);
  }
  unsigned grid = (unsigned)min(ncu, p.out_features);
  plan.rows_per_wg = (p.out_features + (int)grid - 1) / (int)grid;
  grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  // pick the number of main slices: fill lanes, keep waves busy, balance rows over streams
  double best = -1.0;
  for (int W = 1; W <= NW - plan.Wo && W <= MAX_SLICES - plan.Wo; ++W) {
    const int U = (p.P + 64 * W - 1) / (64 * W);
    if (U > umax) continue;
    const int RS = (NW - plan.Wo) / W;
    const int iters = (plan.rows_per_wg + RS - 1) / RS;
    const double eff = (double)p.P / (64.0 * W * U) * (double)(RS * W) / NW * (double)plan.rows_per_wg / ((double)iters * RS);
    if (eff > best) { best = eff; plan.W = W; plan.U = U; plan.RS = RS; }
  }
  if (best < 0.0) return VQ_ERR_UNSUPPORTED;
  const long long max_stride = max(p.stride, max(p.stride_res, p.stride_out));
  if ((long long)plan.rows_per_wg * max_stride >= (1LL << 31)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  unsigned off = 4096u * 16u;
  plan.lds_res = off; off += p.k_res ? (1u << p.bits_res) * 16u : 0u;
  plan.lds_out = off; off += p.Q ? 4096u * 8u : 0u;
  plan.lds_part = off; off += (unsigned)(RC * (plan.W + plan.Wo) * batch) * 4u;
  plan.lds_xsum = off; off += 16u;
  if (off > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  const int rb = p.k_res ? p.bits_res : 0;
#define VQ_CASE(R, BB, UM) if (rb == R && batch == BB) return launch_one<R, BB, UM>(p, plan, off, grid, x, ldx, y, ldy, s);
  VQ_CASE(0, 1, 16) VQ_CASE(12, 1, 16) VQ_CASE(8, 1, 16)
  VQ_CASE(0, 2, 8) VQ_CASE(12, 2, 8) VQ_CASE(8, 2, 8)
  VQ_CASE(0, 4, 4) VQ_CASE(12, 4, 4) VQ_CASE(8, 4, 4)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
