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
#include "vq_v6.hpp"
#include <cstdlib>

namespace vq {


namespace {

using namespace v6;

constexpr int NW = 16;           // waves per workgroup
constexpr int RC_MAX = 64;       // most rows per reduction chunk
constexpr int MAX_SLICES = 16;

struct GemvPlan {
  int W, U;                      // main slices per row, vectors per lane
  int Wo, Uo;                    // outlier slices per row, outlier vectors per lane
  int RS;                        // row streams (rows in flight) for the main waves
  int rows_per_wg;
  unsigned lds_out, lds_part, lds_xsum;            // byte offsets into dynamic LDS (the v=6 tables start at 0)
  unsigned lds_x;                                  // activation rows in LDS: x_regions regions of x_bytes each
  int x_regions;                                   // batch rows staged at a time (1 .. B)
  unsigned x_bytes;                                // bytes of one staged activation row (multiple of 1024)
  int rc;                                          // rows per reduction chunk
  unsigned role[16];                               // per wave: slice | first row << 8 | main << 16 | outlier << 17
};

// Codebook staging: all loads of all tables first, then the LDS writes.  Each thread takes four consecutive 12-byte entries (v = 6: three aligned
// 16-byte loads) or two 16-byte chunks of 8-byte entries (v = 4).  Range-checked loads give zeros past the
// table's k entries, so the LDS copy is zero up to its power-of-two size.
struct TableRegs { uint4v m[3], r[3], o[2]; };

template <int RES_BITS>
__device__ __forceinline__ void tables_load(TableRegs &t, const Params &p, bool has_out) {
  const __amdgpu_buffer_rsrc_t rm = make_rsrc(p.cb, (unsigned)p.k * 12u);
#pragma unroll
  for (int i = 0; i < 3; ++i) t.m[i] = __builtin_amdgcn_raw_buffer_load_b128(rm, threadIdx.x * 48u + i * 16u, 0, 0);
  if (RES_BITS) {
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(p.cb_res, (unsigned)p.k_res * 12u);
#pragma unroll
    for (int i = 0; i < 3; ++i) t.r[i] = __builtin_amdgcn_raw_buffer_load_b128(rr, threadIdx.x * 48u + i * 16u, 0, 0);
  }
  if (has_out) {
    const __amdgpu_buffer_rsrc_t ro = make_rsrc(p.cb_out, (unsigned)p.k_out * 8u);
#pragma unroll
    for (int i = 0; i < 2; ++i) t.o[i] = __builtin_amdgcn_raw_buffer_load_b128(ro, (threadIdx.x + i * NW * 64) * 16u, 0, 0);
  }
}

template <unsigned OFF, unsigned SH>
__device__ __forceinline__ void store_padded4(unsigned char *lds, const uint4v (&v)[3]) {
  // 12 dwords = 4 entries of 3 dwords -> 4 slots of 4 dwords (last one zero)
  const unsigned d[12] = {v[0].x, v[0].y, v[0].z, v[0].w, v[1].x, v[1].y, v[1].z, v[1].w, v[2].x, v[2].y, v[2].z, v[2].w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint4v e; e.x = d[3 * i]; e.y = d[3 * i + 1]; e.z = d[3 * i + 2]; e.w = 0u;
    *reinterpret_cast<uint4v *>(lds + OFF + ((threadIdx.x * 4 + i) << SH)) = e;
  }
}

template <int RES_BITS>
__device__ __forceinline__ void tables_store(const TableRegs &t, unsigned char *lds, const GemvPlan &plan, bool has_out) {
  typedef Layout<RES_BITS> L;
  store_padded4<L::MAIN_OFF, L::MAIN_SH>(lds, t.m);                          // 1024 threads x 4 = 4096 entries
  if (RES_BITS == 12) store_padded4<L::RES_OFF, L::RES_SH>(lds + L::RES_ADD, t.r);
  if (RES_BITS == 8 && threadIdx.x < 64) store_padded4<L::RES_OFF, L::RES_SH>(lds, t.r);   // 256 entries
  if (has_out) {
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4v *>(lds + plan.lds_out + (threadIdx.x + i * NW * 64) * 16) = t.o[i];
  }
}

constexpr int window_dwords(int bits, int u) { return (32 - 4 + bits * u + 31) / 32; }   // worst start bit is 28 (12-bit) or 24 (8-bit)

// U: vectors per lane (compile time, so the lookups of a row carry no branches and overlap freely).
// `wg`: the workgroup's number within its layer (a launch may hold the workgroups of several layers).
template <int RES_BITS, int B, int U>
__device__ __forceinline__ void gemv_v6_body(const Params &p, const GemvPlan &plan, const __half *__restrict__ x, long long ldx,
                                             __half *__restrict__ y, long long ldy, int wg) {
  // rows of index windows a wave keeps in flight, and copies of the row body in the unrolled loop.  Measured on the
  // 11008 x 4096 layer (9 rows a wave), one row of activations: 2 / 3 / 4 / 5 / 8 in flight -> 7.9 / 7.8 / 8.1 / 8.6 / 9.6 us;
  // what is in flight beyond the latency of HBM buys nothing, and a body copy that the last round does not use costs.
  // With a residual stream (two windows a row, a longer row body) two rows are enough: 4096 x 4096 8.1 -> 7.9 us,
  // 11008 x 4096 12.9 -> 12.7 us, 8192 x 28672 37.0 -> 36.4 us.  (Seven other layer shapes without a residual stream, one
  // row: three in flight are 3-7 % ahead of four on every one, two are level with three; more rows per launch: three
  // are 1-2 % ahead of four.)
  constexpr int DEPTH = (RES_BITS && B == 1) ? 2 : 3;
  constexpr int NM = window_dwords(12, U);
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  constexpr int NR = window_dwords(RB, U);
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = wg * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const int rows_here = row1 - row0;
  const int Wt = plan.W + plan.Wo;
  float *part = reinterpret_cast<float *>(lds + plan.lds_part);     // [rc][Wt][B]
  float *xsum = reinterpret_cast<float *>(lds + plan.lds_xsum);     // [B][NW]
  typedef Layout<RES_BITS> LY;
  const unsigned a_out = lds_address(lds) + plan.lds_out;

  // ---- role of this wave: main slice `slice` of row stream `start`, or outlier slice, or idle
  const unsigned role = plan.role[wv];          // worked out on the host: no divisions here
  const bool is_main = (role >> 16) & 1u, is_out = (role >> 17) & 1u;
  const int slice = (int)(role & 0xFFu);
  const int start = (int)((role >> 8) & 0xFFu);
  const int step = is_main ? plan.RS : 1;
  const int first_vec = (slice * 64 + lane) * U;

  // ---- index stream geometry of this lane
  const unsigned bit0 = (unsigned)first_vec * 12u;
  const unsigned dw_main = bit0 >> 5, sh_main = bit0 & 31u;
  const unsigned bitr = (unsigned)first_vec * (unsigned)RB;
  const unsigned dw_res = bitr >> 5, sh_res = bitr & 31u;
  const unsigned st_main = (unsigned)(is_out ? p.stride_out : p.stride), st_res = (unsigned)p.stride_res;
  const __amdgpu_buffer_rsrc_t r_main =
      is_out ? make_rsrc(p.idx_out + (long long)row0 * p.stride_out, (unsigned)rows_here * st_main)
             : make_rsrc(p.idx + (long long)row0 * p.stride, (unsigned)rows_here * st_main);
  const __amdgpu_buffer_rsrc_t r_res = make_rsrc(RES_BITS ? p.idx_res + (long long)row0 * p.stride_res : p.idx,
                                                 RES_BITS ? (unsigned)rows_here * st_res : 0u);
  const __amdgpu_buffer_rsrc_t r_cbres = make_rsrc(RES_BITS ? (const void *)p.cb_res : (const void *)p.cb, RES_BITS ? (unsigned)p.k_res * 12u : 0u);

  unsigned xr[B][U][3];
  Window<NM> wm[DEPTH];
  Window<NR> wr[DEPTH];
  const int c0 = is_main ? p.n_out + first_vec * 6 : first_vec * 4;

  // the codebook loads go out first: they are hits in L2 (for all but the first workgroups) and, as loads return in order,
  // can be stored as soon as they are back, while the index rows asked for after them are still on their way from HBM
  // ---- put the first DEPTH rows of a chunk's index windows in flight
  auto first_rows = [&](int chunk0) {
    const int row_end = (is_main || is_out) ? min(plan.rc, rows_here - chunk0) : 0;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      if (start + d * step < row_end) {
        const unsigned r = (unsigned)(chunk0 + start + d * step);
        load_window(wm[d], r_main, r * st_main, dw_main);
        if (RES_BITS && is_main) load_window(wr[d], r_res, r * st_res, dw_res);
      }
  };
  // The same for the first chunk, with every load issued whatever the wave's role and rows (a row past the wave's last one
  // is replaced by the workgroup's last row: the load stays an ordinary one that returns in order): the start-up below
  // waits for "all but the last FIRST_LOADS loads", which must be exactly these.
  constexpr int FIRST_LOADS = DEPTH * (RES_BITS ? 2 : 1);
  static_assert(NM <= 4 && NR <= 4, "one load instruction per window");
  auto first_rows_all = [&]() {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const unsigned r = (unsigned)min(start + d * step, rows_here - 1);
      load_window(wm[d], r_main, r * st_main, dw_main);
      if (RES_BITS) load_window(wr[d], r_res, r * st_res, dw_res);
    }
  };
  TableRegs tabs;
  tables_load<RES_BITS>(tabs, p, plan.Wo != 0);

  // ---- activations: batch rows are copied into LDS by asynchronous, range-checked 16-byte loads that write
  // LDS directly (zeros past in_features, which is even here, so padded vectors and idle lanes multiply by
  // zero); wave w copies 1 KB pieces w, w+16, ...  plan.x_regions rows fit at a time (all of them when LDS
  // allows); each lane then moves its own vectors to registers, where they stay for the whole kernel.
#pragma unroll
  for (int b0 = 0; b0 < B; ++b0) {
    const int region = b0 % plan.x_regions;
    if (region == 0) {
      if (b0 != 0) __syncthreads();                       // everyone has read the previous group of rows
#pragma unroll
      for (int bb = 0; bb < B; ++bb) {
        if (bb >= b0 && bb < b0 + plan.x_regions) {
          const __amdgpu_buffer_rsrc_t rx = make_rsrc(x + bb * ldx, (unsigned)p.in_features * 2u);
          if (p.perm) {
            // permuted column order (Sec. 3.2.3): stored column c meets x[perm[c]]; a thread gathers two columns at a time
            // (ordinary loads, which the compiler waits for before the LDS write; entries outside the row count as zero)
            const __amdgpu_buffer_rsrc_t rp = make_rsrc(p.perm, (unsigned)p.in_features * 4u);
            for (unsigned c = threadIdx.x * 2u; c < plan.x_bytes / 2u; c += NW * 128u) {
              const uint2v t = __builtin_amdgcn_raw_buffer_load_b64(rp, c * 4u, 0, 0);
              const unsigned lo = c < (unsigned)p.in_features && t.x < (unsigned)p.in_features ? (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rx, t.x * 2u, 0, 0) : 0u;
              const unsigned hi = c + 1u < (unsigned)p.in_features && t.y < (unsigned)p.in_features ? (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rx, t.y * 2u, 0, 0) : 0u;
              *reinterpret_cast<unsigned *>(lds + plan.lds_x + (bb - b0) * plan.x_bytes + c * 2u) = lo | (hi << 16);
            }
          } else {
          for (unsigned piece = (unsigned)wv * 1024u; piece < plan.x_bytes; piece += NW * 1024u)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void *)(lds + plan.lds_x + (bb - b0) * plan.x_bytes + piece),
                                                     16, piece + lane * 16u, 0, 0, 0);
          }
        }
      }
      if (b0 == 0) {
        // The first index rows go out behind the codebooks and the first activation rows -- those are hits in L2 -- and
        // are not waited for here: the rest of the start-up runs while they are on their way from HBM.  (Loads return
        // in order; the empty statements keep the compiler from moving the index loads across them.)
        asm volatile("" ::: "memory");
        first_rows_all();
        asm volatile("" ::: "memory");
        tables_store<RES_BITS>(tabs, lds, plan, plan.Wo != 0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FIRST_LOADS) : "memory");   // codebooks and direct-to-LDS copies have landed
        lds_barrier();                                   // (a full barrier would wait for the index rows as well)
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the direct-to-LDS copies have landed
        __syncthreads();
      }
    }
    const int b = b0;
    const unsigned char *xl = lds + plan.lds_x + region * plan.x_bytes;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (is_main) {
#pragma unroll
        for (int h = 0; h < 3; ++h) xr[b][u][h] = *reinterpret_cast<const unsigned *>(xl + (c0 + u * 6 + h * 2) * 2);
      } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int c = c0 + u * 4 + h * 2;
          const unsigned v = *reinterpret_cast<const unsigned *>(xl + (is_out ? c : 0) * 2);
          xr[b][u][h] = (is_out && c < p.n_out) ? v : 0u;      // outlier lanes past the last outlier vector
        }
        xr[b][u][2] = 0u;
      }
    }
    float s0 = 0.0f;
    for (unsigned o = threadIdx.x * 16u; o < plan.x_bytes; o += NW * 64 * 16u) {
      const uint4v v = *reinterpret_cast<const uint4v *>(xl + o);
      s0 += half_pair_sum(v.x) + half_pair_sum(v.y) + half_pair_sum(v.z) + half_pair_sum(v.w);
    }
    const float s = wave_reduce_to_lane63(s0);
    if (lane == 63) xsum[b * NW + wv] = s;
  }

  for (int chunk0 = 0; chunk0 < rows_here; chunk0 += plan.rc) {
    const int rows_chunk = min(plan.rc, rows_here - chunk0);
    const int row_end = (is_main || is_out) ? rows_chunk : 0;     // rows start, start+step, ... below row_end are this wave's
    if (chunk0 != 0) first_rows(chunk0);

    // scale and bias of the row this thread finishes at the end of the chunk
    const int ep_rl = (int)threadIdx.x / B, ep_b = (int)threadIdx.x - ep_rl * B;
    const bool ep_on = (int)threadIdx.x < rows_chunk * B;
    const int ep_o = row0 + chunk0 + ep_rl;
    const float ep_scale = (ep_on && p.scale) ? __half2float(p.scale[ep_o]) : 1.0f;
    const float ep_bias = (ep_on && p.bias) ? __half2float(p.bias[ep_o]) : 0.0f;


    for (int rl0 = start; rl0 < row_end; rl0 += DEPTH * step) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        const int rl = rl0 + d * step;
        if (rl < row_end) {
          Window<NM> cm;
          Window<NR> cr;
          normalize_from(cm, wm[d], sh_main);
          if (RES_BITS && is_main) normalize_from(cr, wr[d], sh_res);
          if (rl + DEPTH * step < row_end) {  // refill this slot with the row DEPTH steps ahead
            const unsigned r = (unsigned)(chunk0 + rl + DEPTH * step);
            load_window(wm[d], r_main, r * st_main, dw_main);
            if (RES_BITS && is_main) load_window(wr[d], r_res, r * st_res, dw_res);
          }
          float acc[B];
#pragma unroll
          for (int b = 0; b < B; ++b) acc[b] = 0.0f;
          if (is_main) {
            // main lookups, then (second phase, reusing the registers) the LDS-side residual lookups
            {
              uint4v e[U];
#pragma unroll
              for (int u = 0; u < U; ++u) lds_gather16<LY::MAIN_OFF>(e[u], field_addr<12, LY::MAIN_SH>(cm, u));
              lds_gather_wait();
#pragma unroll
              for (int u = 0; u < U; ++u) settle(e[u]);
#pragma unroll
              for (int u = 0; u < U; ++u)
#pragma unroll
                for (int b = 0; b < B; ++b) {
                  acc[b] = dot2(e[u].x, xr[b][u][0], acc[b]);
                  acc[b] = dot2(e[u].y, xr[b][u][1], acc[b]);
                  acc[b] = dot2(e[u].z, xr[b][u][2], acc[b]);
                }
            }
            if (RES_BITS) {
              uint4v f[U];
#pragma unroll
              for (int u = 0; u < U; ++u) lds_gather16<LY::RES_OFF>(f[u], field_addr<RB, LY::RES_SH>(cr, u) + LY::RES_ADD);
              lds_gather_wait();
#pragma unroll
              for (int u = 0; u < U; ++u) settle(f[u]);
#pragma unroll
              for (int u = 0; u < U; ++u)
#pragma unroll
                for (int b = 0; b < B; ++b) {
                  acc[b] = dot2(f[u].x, xr[b][u][0], acc[b]);
                  acc[b] = dot2(f[u].y, xr[b][u][1], acc[b]);
                  acc[b] = dot2(f[u].z, xr[b][u][2], acc[b]);
                }
            }
          } else {
            uint2v e[U];
#pragma unroll
            for (int u = 0; u < U; ++u) lds_gather8(e[u], field_addr<12, 3>(cm, u) + a_out);
            lds_gather_wait();
#pragma unroll
            for (int u = 0; u < U; ++u) settle(e[u]);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
              for (int b = 0; b < B; ++b) {
                acc[b] = dot2(e[u].x, xr[b][u][0], acc[b]);
                acc[b] = dot2(e[u].y, xr[b][u][1], acc[b]);
              }
          }
          const int col = is_main ? slice : plan.W + slice;
#pragma unroll
          for (int b = 0; b < B; ++b) {
            const float s = wave_reduce_to_lane63(acc[b]);
            if (lane == 63) part[(rl * Wt + col) * B + b] = s;
          }
        }
      }
    }
    __syncthreads();
    // ---- combine slices, apply scale and bias, store
    if (ep_on) {
      float s = 0.0f;
      for (int w = 0; w < Wt; ++w) s += part[(ep_rl * Wt + w) * B + ep_b];
      float xs = 0.0f;
      for (int w = 0; w < NW; ++w) xs += xsum[ep_b * NW + w];
      y[ep_b * ldy + ep_o] = __float2half_rn(__fmaf_rn(ep_scale, s, ep_bias * xs));
    }
    __syncthreads();
  }
}

template <int RES_BITS, int B, int U>
__global__ __launch_bounds__(NW * 64) void gemv_v6_kernel(Params p, GemvPlan plan, const __half *__restrict__ x, long long ldx,
                                                          __half *__restrict__ y, long long ldy) {
  warm_kernel_arguments();                      // Params + GemvPlan + four scalars: about 250 bytes
  gemv_v6_body<RES_BITS, B, U>(p, plan, x, ldx, y, ldy, (int)blockIdx.x);
}

// Several layers on one activation row in one launch (the query, key and value projections; gate and up): every
// workgroup belongs to one layer and runs the body above on it.  Batch 1 only: this is the kernel that a single
// decode step runs, where the launch and start-up cost weighs most.
constexpr int MULTI_MAX = 8;
struct MultiLayer {
  Params p;
  GemvPlan plan;
  __half *y;
};
struct MultiArgs {
  int n;
  int first_wg[MULTI_MAX + 1];             // layer i owns workgroups [first_wg[i], first_wg[i + 1])
  MultiLayer layer[MULTI_MAX];
};

template <int RES_BITS, int U>
__global__ __launch_bounds__(NW * 64) void gemv_v6_multi_kernel(MultiArgs a, const __half *__restrict__ x) {
  warm_kernel_arguments();
  int i = 0;
  while (i + 1 < a.n && (int)blockIdx.x >= a.first_wg[i + 1]) ++i;
  const MultiLayer &l = a.layer[i];
  gemv_v6_body<RES_BITS, 1, U>(l.p, l.plan, x, 0, l.y, 0, (int)blockIdx.x - a.first_wg[i]);
}

template <int RES_BITS, int B, int U>
int launch_one(const Params &p, const GemvPlan &plan, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx,
               __half *y, long long ldy, hipStream_t s) {
  auto kernel = gemv_v6_kernel<RES_BITS, B, U>;
  VQ_ALLOW_FULL_LDS(kernel);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds_bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int RES_BITS, int B>
int launch_u(int U, const Params &p, const GemvPlan &plan, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx,
             __half *y, long long ldy, hipStream_t s) {
  if (U == 4) return launch_one<RES_BITS, B, 4>(p, plan, lds_bytes, grid, x, ldx, y, ldy, s);
  // (the combinations u_allowed() admits, no others: each costs build time and library size)
  if constexpr (B <= 2) {
    if (U == 5) return launch_one<RES_BITS, B, 5>(p, plan, lds_bytes, grid, x, ldx, y, ldy, s);
  }
  if constexpr (B == 1) {
    if (U == 6) return launch_one<RES_BITS, B, 6>(p, plan, lds_bytes, grid, x, ldx, y, ldy, s);
  }
  if constexpr (B == 1 && RES_BITS == 0) {
    if (U == 8) return launch_one<0, 1, 8>(p, plan, lds_bytes, grid, x, ldx, y, ldy, s);
  }
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace


// Whether the fast kernels take this layer and these buffers.
bool gemv_fast_applicable(const Params &p, const __half *x, long long ldx) {
  if (p.orientation != 0 || p.v != 6 || p.bits != 12) return false;
  if (p.n_groups > 1 && (p.Pg & 7)) return false;           // a group starts on a dword of the index streams
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return false;
  if (p.n_out && (p.v_out != 4 || p.bits_out != 12)) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 3) || (ldx & 1) || (p.in_features & 1)) return false;
  const long long max_stride = p.stride > p.stride_res ? p.stride : p.stride_res;
  if (max_stride > (1 << 24)) return false;
  return true;
}

// Vectors per lane the kernels are built for, by batch group and residual use (register budget of 128).
static bool u_allowed(int U, int batch, bool res) {
  if (batch == 1) return res ? (U == 4 || U == 5 || U == 6) : (U == 4 || U == 5 || U == 6 || U == 8);
  if (batch == 2) return res ? (U == 4 || U == 5) : (U == 4 || U == 5);
  return U == 4;
}

namespace {

// Work split and LDS layout of one layer.  rows_per_wg == 0: one workgroup per compute unit; u_force > 0: that many
// vectors per lane or nothing (several layers in one launch share one kernel instantiation).
int make_plan(const Params &p, int batch, int rows_per_wg, int u_force, GemvPlan *out, unsigned *lds_bytes, unsigned *grid_out) {
  static const int kU[] = {4, 5, 6, 8};
  GemvPlan plan{};
  // LDS: tables first (main at 0); the activation rows, partial sums and activation sums follow once the
  // slicing is known
  const int rb = p.k_res ? p.bits_res : 0;
  unsigned off = rb == 0 ? Layout<0>::BYTES : rb == 8 ? Layout<8>::BYTES : Layout<12>::BYTES;
  plan.lds_out = off; off += p.Q ? 4096u * 8u : 0u;
  if (off > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  if (rows_per_wg > 0) {
    plan.rows_per_wg = rows_per_wg;
  } else {
    const unsigned g = (unsigned)min(cu_count(), p.out_features);
    plan.rows_per_wg = (p.out_features + (int)g - 1) / (int)g;
  }
  *grid_out = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  const long long max_stride = max(p.stride, max(p.stride_res, p.stride_out));
  if ((long long)plan.rows_per_wg * max_stride >= (1LL << 31)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  // vectors per lane U and main slices W: fill lanes, keep waves busy, balance rows over the row streams
  double best = -1.0;
  for (int U : kU) {
    if (!u_allowed(U, batch, p.k_res != 0) || (u_force > 0 && U != u_force)) continue;
    const int Wo = p.Q ? (p.Q + 64 * U - 1) / (64 * U) : 0;
    if (Wo >= NW) continue;
    const int W = (p.P + 64 * U - 1) / (64 * U);
    if (W + Wo > NW || W + Wo > MAX_SLICES) continue;
    const int RS = (NW - Wo) / W;
    const int rows = min(plan.rows_per_wg, RC_MAX);
    const int iters = (rows + RS - 1) / RS;
    const double eff = (double)p.P / (64.0 * W * U) * (double)(RS * W) / NW * (double)rows / ((double)iters * RS);
    if (eff > best) { best = eff; plan.W = W; plan.U = U; plan.RS = RS; plan.Wo = Wo; plan.Uo = U; }
  }
  if (best < 0.0) return VQ_ERR_UNSUPPORTED;
  for (int w = 0; w < NW; ++w) {
    const int n_main = plan.RS * plan.W;
    if (w < n_main) plan.role[w] = (unsigned)(w % plan.W) | ((unsigned)(w / plan.W) << 8) | (1u << 16);
    else if (w - n_main < plan.Wo) plan.role[w] = (unsigned)(w - n_main) | (1u << 17);
    else plan.role[w] = 0u;
  }
  // one activation row, up to the last column any lane touches, in 1 KB pieces
  const long long x_cols = max((long long)p.n_out + 6LL * plan.W * 64 * plan.U, 4LL * plan.Wo * 64 * plan.U);
  plan.x_bytes = (unsigned)((x_cols * 2 + 1023) / 1024 * 1024);
  const int per_row = (plan.W + plan.Wo) * batch * 4;
  const unsigned fixed = off + (unsigned)(NW * batch) * 4u + (unsigned)(plan.RS * per_row);   // tables, sums, fewest partial rows
  if (fixed + plan.x_bytes > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  plan.x_regions = (int)min((unsigned)batch, (160u * 1024u - fixed) / plan.x_bytes);
  if (plan.x_regions == 3) plan.x_regions = 2;                 // groups of equal size
  plan.lds_x = off; off += plan.x_bytes * (unsigned)plan.x_regions;
  plan.lds_xsum = off; off += (unsigned)(NW * batch) * 4u;
  plan.lds_part = off;
  if (off >= 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  plan.rc = min(RC_MAX, (int)((160u * 1024u - off) / (unsigned)per_row));
  if (plan.rc < plan.RS || plan.rc < 1) return VQ_ERR_UNSUPPORTED;
  off += (unsigned)(plan.rc * per_row);
  *out = plan; *lds_bytes = off;
  return VQ_OK;
}

template <int RES_BITS, int U>
int launch_multi(const MultiArgs &a, unsigned lds_bytes, unsigned grid, const __half *x, hipStream_t s) {
  auto kernel = gemv_v6_multi_kernel<RES_BITS, U>;
  VQ_ALLOW_FULL_LDS(kernel);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds_bytes, s, a, x);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Launch for one group of 1, 2 or 4 batch rows.
int launch_gemv_fast(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (p.n_groups > 1) return VQ_ERR_UNSUPPORTED;          // one table set per workgroup: layers with codebook groups go elsewhere
  GemvPlan plan;
  unsigned off = 0, grid = 0;
  const int rc = make_plan(p, batch, 0, 0, &plan, &off, &grid);
  if (rc != VQ_OK) return rc;
  const int rb = p.k_res ? p.bits_res : 0;
#define VQ_CASE(R, BB) if (rb == R && batch == BB) return launch_u<R, BB>(plan.U, p, plan, off, grid, x, ldx, y, ldy, s);
  VQ_CASE(0, 1) VQ_CASE(12, 1) VQ_CASE(8, 1)
  VQ_CASE(0, 2) VQ_CASE(12, 2) VQ_CASE(8, 2)
  VQ_CASE(0, 4) VQ_CASE(12, 4) VQ_CASE(8, 4)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

// n layers (2 .. MULTI_MAX) on the same single activation row in one launch.  VQ_ERR_UNSUPPORTED when the layers do not
// fit one kernel instantiation (different residual kinds or vectors per lane, codebook groups, different in_features).
// The caller has checked gemv_fast_applicable() for each.
int launch_gemv_fast_multi(const Params *ps, int n, const __half *x, __half *const *ys, hipStream_t s) {
  if (n < 2 || n > MULTI_MAX) return VQ_ERR_UNSUPPORTED;
  const int cus = cu_count();
  long long rows_all = 0;
  for (int i = 0; i < n; ++i) {
    if (ps[i].in_features != ps[0].in_features || ps[i].n_groups > 1) return VQ_ERR_UNSUPPORTED;
    if ((ps[i].k_res ? ps[i].bits_res : 0) != (ps[0].k_res ? ps[0].bits_res : 0)) return VQ_ERR_UNSUPPORTED;
    rows_all += ps[i].out_features;
  }
  // every workgroup takes the same number of rows of one layer: the smallest number with which all the workgroups run
  // at once, one per compute unit
  int r = (int)((rows_all + cus - 1) / cus);
  for (;; ++r) {
    long long wgs = 0;
    for (int i = 0; i < n; ++i) wgs += (ps[i].out_features + r - 1) / r;
    if (wgs <= cus) break;
  }
  MultiArgs a{};
  unsigned lds_bytes = 0;
  int U = 0;
  a.n = n;
  for (int i = 0; i < n; ++i) {
    unsigned off = 0, grid = 0;
    const int rc = make_plan(ps[i], 1, r, U, &a.layer[i].plan, &off, &grid);
    if (rc != VQ_OK) return rc;
    U = a.layer[i].plan.U;                               // the first layer's choice binds the others
    a.layer[i].p = ps[i]; a.layer[i].y = ys[i];
    a.first_wg[i + 1] = a.first_wg[i] + (int)grid;
    lds_bytes = max(lds_bytes, off);
  }
  const unsigned grid = (unsigned)a.first_wg[n];
  const int rb = ps[0].k_res ? ps[0].bits_res : 0;
#define VQ_CASE(R, UU) if (rb == R && U == UU) return launch_multi<R, UU>(a, lds_bytes, grid, x, s);
  VQ_CASE(0, 4) VQ_CASE(0, 5) VQ_CASE(0, 6) VQ_CASE(0, 8)
  VQ_CASE(12, 4) VQ_CASE(12, 5) VQ_CASE(12, 6)
  VQ_CASE(8, 4) VQ_CASE(8, 5) VQ_CASE(8, 6)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
