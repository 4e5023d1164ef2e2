// vq_gemv for layers stored in the paper's own orientation (Sec. 3.1, Algorithm 1: a vector covers v output rows of one input
// column) in the settings that have no kernel of their own there -- v = 12 with two 4096-entry tables, codebook groups, 1 %
// outlier columns of v = 4 (Table "Quantization parameters"), v = 4 / k = 256, ... -- with one table in LDS at a time, as the
// pass kernel of the other orientation does (vq_gemv_lds.hip).
//
// A workgroup owns a block of index streams (a stream is v output rows) and walks the passes: (codebook group, main or
// residual table), then the outlier table.  In a pass the (stream, 64 windows of the stream) items are dealt to the sixteen
// waves in order; a lane takes a window of its stream's indices (consecutive columns), looks every centroid up in LDS and adds
// centroid[j] * x[column] to the sum of row j; at the end of a stream's items a wave reduces its v sums over the lanes and
// leaves them in LDS, where the waves' parts of a stream are added in ascending order (the same bits every run) to the sums of
// the passes before.  Activations are staged in stored column order (gathered by col_perm), with zeros outside the pass's
// group, so that windows that straddle two groups need no masks.  y = scale * (sum of the passes) + bias * sum(x).
#include "vq_lds_tables.hpp"

namespace vq {

namespace {

using namespace lds_tables;

constexpr int LW = 16;           // waves per workgroup

struct DownPlan {
  unsigned off_x, off_xo, off_xsum, off_part, off_ypart, bytes;   // byte offsets in dynamic LDS (the pass's table at 0)
  unsigned x_pitch, xo_pitch;                                     // bytes per staged row of main / outlier columns
  int streams_per_wg;
  // With a workspace on loan a workgroup takes one codebook group (the first group's workgroups also the outlier streams) and
  // a block of streams, and leaves its sums in the workspace for the kernel that adds the groups up:
  int n_slots, batch_total;                                       // 0: every workgroup walks all passes and writes y
  float *gpart, *gpart_xs;                                        // [n_slots][batch_total][out_features] sums, [n_slots][16] activation sums
};

__device__ __forceinline__ float lo_half(unsigned w) { return __half2float(__ushort_as_half((unsigned short)(w & 0xFFFFu))); }
__device__ __forceinline__ float hi_half(unsigned w) { return __half2float(__ushort_as_half((unsigned short)(w >> 16))); }

template <int V, int BITS, int B>
__global__ __launch_bounds__(LW * 64) void gemv_down_lds_kernel(Params p, DownPlan plan, const __half *__restrict__ x, long long ldx,
                                                                __half *__restrict__ y, long long ldy) {
  constexpr int U = win_vectors(BITS), ND = U * BITS / 32, NW = ND < 2 ? 2 : ND, EH = entry_halfs(V), ED = EH / 2, VD = V / 2;
  constexpr int AM = V > 4 ? V : 4;                       // sums a lane keeps: v rows of a stream, or the 4 of an outlier stream
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  float *xsum = reinterpret_cast<float *>(lds + plan.off_xsum);          // [B], then the waves' parts [B][LW]
  float *xpart = xsum + B;
  float *part = reinterpret_cast<float *>(lds + plan.off_part);          // [unit][wave][AM][B]: a wave's sums of a stream in this pass
  float *ypart = reinterpret_cast<float *>(lds + plan.off_ypart);        // [row of the workgroup][B]: the passes so far
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const bool slots = plan.n_slots != 0;
  const int slot = slots ? (int)blockIdx.x % plan.n_slots : 0;
  const int s0 = (slots ? (int)blockIdx.x / plan.n_slots : (int)blockIdx.x) * plan.streams_per_wg, s1 = min(p.S, s0 + plan.streams_per_wg);
  const int row_base = s0 * V, n_rows = min(p.out_features, s1 * V) - row_base;      // (row_base is a multiple of 4 when there are outlier columns)
  const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.S * p.stride), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.k_res ? p.idx_res : p.idx), 0,
                                                                       p.k_res ? (unsigned)((long long)p.S * p.stride_res) : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_o = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.Q ? p.idx_out : p.idx), 0,
                                                                       p.Q ? (unsigned)((long long)p.S_out * p.stride_out) : 0u, 0x00020000);
  auto x_at = [&](int t, int c) {                         // activation of stored column c (Sec. 3.2.3), zero outside the row
    int src = c;
    if (p.perm) src = p.perm[c];
    return (unsigned)src < (unsigned)p.in_features ? x[(long long)t * ldx + src] : __float2half_rn(0.0f);
  };

  // ---- once: the activations of the outlier columns and their sum (with slots: the first slot's workgroups only); the main
  // columns are added to the sums as the passes restage them
  const int once_cols = slot == 0 ? p.n_out : 0;
#pragma unroll
  for (int t = 0; t < B; ++t) {
    __half *xo = reinterpret_cast<__half *>(lds + plan.off_xo + t * plan.xo_pitch);
    float sum = 0.0f;
    for (int c = threadIdx.x; c < once_cols; c += LW * 64) {
      const __half v = x_at(t, c);
      if (c < p.n_out) xo[c] = v;
      sum += __half2float(v);
    }
    sum = wave_sum(sum);
    if (lane == 0) xpart[t * LW + wv] = sum;
  }

  const int tables_per_group = p.k_res ? 2 : 1;
  const int table_passes = p.n_groups * tables_per_group;
  const int pass_begin = slots ? slot * tables_per_group : 0;
  const int my_table_passes = slots ? tables_per_group : table_passes;
  const int my_passes = my_table_passes + (p.Q && slot == 0 ? 1 : 0);
  for (int ip = 0; ip < my_passes; ++ip) {
    const int pass = ip < my_table_passes ? pass_begin + ip : table_passes;
    const bool outlier = pass == table_passes;
    const int g = pass / tables_per_group;
    const bool second = !outlier && pass - g * tables_per_group == 1;
    // the pass's stream positions [p_lo, p_hi) (columns), its windows [w_lo, w_hi) (outlier pass: an index per "window")
    const int p_lo = outlier ? 0 : g * p.Pg, p_hi = outlier ? p.Q : min(p.P, p_lo + p.Pg);
    const int w_lo = outlier ? 0 : p_lo / U, w_hi = outlier ? p.Q : (p_hi + U - 1) / U;
    const int rounds = max((w_hi - w_lo + 63) >> 6, 1);
    const int VA = outlier ? 4 : V;                       // rows of a unit: a main stream's v, an outlier stream's 4
    const int units = outlier ? (n_rows + 3) / 4 : s1 - s0;
    const int unit0 = outlier ? row_base / 4 : s0;        // the first unit's stream
    const int n_items = units * rounds, ipw = (n_items + LW - 1) / LW;
    const int i_lo = min(wv * ipw, n_items), i_hi = min(n_items, i_lo + ipw);         // this wave's items: (unit, round), unit-major
    const int k_a = outlier ? p.k_out : second ? p.k_res : p.k;
    const __half *cb_a = outlier ? p.cb_out : second ? p.cb_res + (long long)g * p.k_res * V : p.cb + (long long)g * p.k * V;
    const __amdgpu_buffer_rsrc_t r_a = outlier ? r_o : second ? r_r : r_i;
    const unsigned stride_a = (unsigned)(outlier ? p.stride_out : second ? p.stride_res : p.stride);
    auto load_round = [&](unsigned (&w)[NW], int item) {
      const int unit = item / rounds, wdx = w_lo + lane + (item - unit * rounds) * 64;
      unsigned off = 0xFFFFFFF0u;                         // past the buffer: zeros, never looked at
      if (item < i_hi && wdx < w_hi)
        off = (unsigned)(unit0 + unit) * stride_a + (outlier ? (((unsigned)wdx * (unsigned)p.bits_out) >> 5) * 4u : (unsigned)wdx * (ND * 4u));
      if (outlier) {
        const uint2v a = __builtin_amdgcn_raw_buffer_load_b64(r_a, off, 0, 0);
        w[0] = a.x; w[1] = a.y;
      } else {
        unsigned v[ND];
        load_window<ND>(v, r_a, off);
#pragma unroll
        for (int d = 0; d < ND; ++d) w[d] = v[d];
      }
    };
    unsigned wm[NW];
    load_round(wm, i_lo);                                 // the first item's words go out ahead of the staging

    __syncthreads();                                      // every wave has left the table, rows and parts of the pass before
    // ---- the pass's table into LDS: padded entries, an entry per thread and round (outlier entries: 8 bytes as they are)
    if (outlier) {
      for (int en = threadIdx.x; en < k_a; en += LW * 64)
        *reinterpret_cast<uint2v *>(lds + (unsigned)en * 8u) = *reinterpret_cast<const uint2v *>(cb_a + (long long)en * 4);
    } else {
#pragma unroll 4
      for (int en = threadIdx.x; en < k_a; en += LW * 64) stage_entry<V>(lds, cb_a, en);
    }
    // ---- the activations of the pass's windows: a new group's, with zeros outside the group (and past the row)
    if (!outlier && !second) {
#pragma unroll
      for (int t = 0; t < B; ++t) {
        __half *xs = reinterpret_cast<__half *>(lds + plan.off_x + t * plan.x_pitch);
        float sum = 0.0f;
        for (int pos = w_lo * U + (int)threadIdx.x; pos < w_hi * U; pos += LW * 64) {
          const __half v = pos >= p_lo && pos < p_hi ? x_at(t, p.n_out + pos) : __float2half_rn(0.0f);
          xs[pos] = v;
          sum += __half2float(v);
        }
        sum = wave_sum(sum);                              // the group's share of sum(x)
        if (lane == 0) xpart[t * LW + wv] += sum;
      }
    }
    __syncthreads();

    // ---- this wave's items
    float acc[AM][B];
#pragma unroll
    for (int j = 0; j < AM; ++j)
#pragma unroll
      for (int t = 0; t < B; ++t) acc[j][t] = 0.0f;
    for (int item = i_lo; item < i_hi; ++item) {
      unsigned nm[NW];
      load_round(nm, item + 1);
      const int unit = item / rounds, wdx = w_lo + lane + (item - unit * rounds) * 64;
      if (wdx < w_hi) {
        if (outlier) {
          const unsigned sh = ((unsigned)wdx * (unsigned)p.bits_out) & 31u;
          unsigned i = wm[0] >> sh;
          if (sh + (unsigned)p.bits_out > 32u) i |= wm[1] << (32u - sh);
          i = min(i & ((1u << p.bits_out) - 1u), (unsigned)k_a - 1u);
          const uint2v e = *reinterpret_cast<const uint2v *>(lds + i * 8u);
#pragma unroll
          for (int t = 0; t < B; ++t) {
            const float xf = __half2float(*reinterpret_cast<const __half *>(lds + plan.off_xo + t * plan.xo_pitch + (unsigned)wdx * 2u));
            acc[0][t] = __fmaf_rn(lo_half(e.x), xf, acc[0][t]);
            acc[1][t] = __fmaf_rn(hi_half(e.x), xf, acc[1][t]);
            acc[2][t] = __fmaf_rn(lo_half(e.y), xf, acc[2][t]);
            acc[3][t] = __fmaf_rn(hi_half(e.y), xf, acc[3][t]);
          }
        } else {
          // the window's U activations per row of x: U halves in a row
          unsigned xw[B][U / 2];
#pragma unroll
          for (int t = 0; t < B; ++t)
#pragma unroll
            for (int q = 0; q < U / 2; ++q)
              xw[t][q] = *reinterpret_cast<const unsigned *>(lds + plan.off_x + t * plan.x_pitch + (unsigned)wdx * (U * 2u) + q * 4u);
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const unsigned i = min(window_field<BITS, NW>(wm, u), (unsigned)k_a - 1u);
            unsigned e[ED];
            read_entry<V>(e, lds, i);
#pragma unroll
            for (int t = 0; t < B; ++t) {
              const float xf = (u & 1) ? hi_half(xw[t][u / 2]) : lo_half(xw[t][u / 2]);
#pragma unroll
              for (int d = 0; d < VD; ++d) {
                acc[2 * d][t] = __fmaf_rn(lo_half(e[d]), xf, acc[2 * d][t]);
                acc[2 * d + 1][t] = __fmaf_rn(hi_half(e[d]), xf, acc[2 * d + 1][t]);
              }
            }
          }
        }
      }
      if (item + 1 == i_hi || (item + 1) / rounds != unit) {            // the wave's last item of this unit: its sums to LDS
#pragma unroll
        for (int j = 0; j < AM; ++j)
#pragma unroll
          for (int t = 0; t < B; ++t) {
            if (j < VA) {
              const float r = segment_sum_to_last(acc[j][t], 64);
              if (lane == 63) part[((unit * LW + wv) * AM + j) * B + t] = r;
            }
            acc[j][t] = 0.0f;
          }
      }
#pragma unroll
      for (int d = 0; d < NW; ++d) wm[d] = nm[d];
    }
    __syncthreads();
    // ---- the waves' parts of every unit, in ascending order, on top of the passes before
    for (int q = threadIdx.x; q < units * VA * B; q += LW * 64) {
      const int unit = q / (VA * B), rem = q - unit * (VA * B), j = rem / B, t = rem - j * B;
      const int w_first = (unit * rounds) / ipw, w_last = ((unit + 1) * rounds - 1) / ipw;
      float sum = 0.0f;
      for (int w = w_first; w <= w_last; ++w) sum += part[((unit * LW + w) * AM + j) * B + t];
      const int r = unit * VA + j;
      if (r < n_rows) ypart[r * B + t] = ip ? __fadd_rn(ypart[r * B + t], sum) : sum;
    }
  }
  // ---- scale, bias, store: a lane per row
  __syncthreads();
  if (threadIdx.x < B) {                                  // the waves' parts of sum(x) in a fixed order
    float sum = 0.0f;
    for (int w = 0; w < LW; ++w) sum += xpart[threadIdx.x * LW + w];
    xsum[threadIdx.x] = sum;
  }
  __syncthreads();
  if (slots) {
    for (int r = threadIdx.x; r < n_rows; r += LW * 64)
#pragma unroll
      for (int t = 0; t < B; ++t) plan.gpart[((long long)slot * plan.batch_total + t) * p.out_features + row_base + r] = ypart[r * B + t];
    if (s0 == 0 && threadIdx.x < B) plan.gpart_xs[slot * 16 + threadIdx.x] = xsum[threadIdx.x];
    return;
  }
  for (int r = threadIdx.x; r < n_rows; r += LW * 64) {
    const int o = row_base + r;
    const float s = p.scale ? __half2float(p.scale[o]) : 1.0f, b = p.bias ? __half2float(p.bias[o]) : 0.0f;
#pragma unroll
    for (int t = 0; t < B; ++t) y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(s, ypart[r * B + t], b * xsum[t]));
  }
}

bool pair_ok(const Params &p) {
  if ((p.k_res && p.bits_res != p.bits) || (p.Q && (p.v_out != 4 || p.bits_out > 16))) return false;
  return compiled_pair(p.v, p.bits, true);
}

bool make_down_plan(const Params &p, int batch, DownPlan *plan, int n_slots = 0) {
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  const int u = win_vectors(p.bits), eh = entry_halfs(p.v), am = p.v > 4 ? p.v : 4;
  size_t table = up16((size_t)p.k * eh * 2);
  if (up16((size_t)p.k_res * eh * 2) > table) table = up16((size_t)p.k_res * eh * 2);
  if (p.Q && up16((size_t)p.k_out * 8) > table) table = up16((size_t)p.k_out * 8);
  const size_t windows = ((size_t)p.P + u - 1) / u;
  const size_t pitch = up16(windows * u * 2), xo_pitch = up16((size_t)p.n_out * 2);
  const int wgs = n_slots ? (cu_count() / n_slots > 0 ? cu_count() / n_slots : 1) : cu_count();     // workgroups per slot
  plan->n_slots = n_slots; plan->batch_total = 0; plan->gpart = nullptr; plan->gpart_xs = nullptr;
  int spw = (p.S + wgs - 1) / wgs;
  if (spw < 1) spw = 1;
  if (p.Q && (p.v & 3)) spw = (spw + 1) & ~1;               // a workgroup's rows start on a multiple of 4, the outlier streams' height
  plan->streams_per_wg = spw;
  const size_t units = (size_t)spw > ((size_t)spw * p.v + 3) / 4 ? (size_t)spw : ((size_t)spw * p.v + 3) / 4;
  const size_t sums = up16(4 * 4 * (1 + LW));
  const size_t part = up16(units * LW * am * batch * 4), ypart = up16((size_t)spw * p.v * batch * 4);
  const size_t total = table + (pitch + xo_pitch) * batch + sums + part + ypart;
  if (total > 160 * 1024) return false;
  if ((long long)p.S * p.stride >= (1LL << 32) || (long long)p.S * p.stride_res >= (1LL << 32) || (long long)p.S_out * p.stride_out >= (1LL << 32)) return false;
  plan->off_x = (unsigned)table; plan->off_xo = (unsigned)(table + pitch * batch);
  plan->off_xsum = (unsigned)(table + (pitch + xo_pitch) * batch); plan->off_part = plan->off_xsum + (unsigned)sums;
  plan->off_ypart = plan->off_part + (unsigned)part; plan->bytes = (unsigned)total;
  plan->x_pitch = (unsigned)pitch; plan->xo_pitch = (unsigned)xo_pitch;
  return true;
}

template <int V, int BITS, int B>
int launch_one(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  DownPlan plan;
  if (!make_down_plan(p, B, &plan)) return VQ_ERR_UNSUPPORTED;
  auto kernel = gemv_down_lds_kernel<V, BITS, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned grid = (unsigned)((p.S + plan.streams_per_wg - 1) / plan.streams_per_wg);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int V, int BITS, int B>
int launch_one_slots(const Params &p, const __half *x, long long ldx, int batch_total, float *part, float *part_xs, hipStream_t s) {
  DownPlan plan;
  if (!make_down_plan(p, B, &plan, p.n_groups)) return VQ_ERR_UNSUPPORTED;
  plan.batch_total = batch_total; plan.gpart = part; plan.gpart_xs = part_xs;
  auto kernel = gemv_down_lds_kernel<V, BITS, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned grid = (unsigned)((p.S + plan.streams_per_wg - 1) / plan.streams_per_wg) * (unsigned)p.n_groups;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, static_cast<__half *>(nullptr), 0LL);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Vectors down the output dimension, a compiled (v, index width) pair, a table that fits LDS beside `batch` activation rows.
bool gemv_down_lds_applicable(const Params &p, int batch) {
  DownPlan plan;
  return p.orientation == 1 && pair_ok(p) && (batch == 1 || batch == 2 || batch == 4) && make_down_plan(p, batch, &plan);
}

// batch in {1, 2, 4}
int launch_gemv_down_lds(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (p.orientation != 1 || !pair_ok(p) || (batch != 1 && batch != 2 && batch != 4)) return VQ_ERR_UNSUPPORTED;
#define VQ_PAIR(V, BITS)                                                                                            \
  if (p.v == V && p.bits == BITS)                                                                                   \
    return batch == 1 ? launch_one<V, BITS, 1>(p, x, ldx, y, ldy, s) : batch == 2 ? launch_one<V, BITS, 2>(p, x, ldx, y, ldy, s) \
                                                                                  : launch_one<V, BITS, 4>(p, x, ldx, y, ldy, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(6, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

// Two codebook groups or more: with a workspace of groups x (batch x out_features + 16) binary32 sums every workgroup takes
// one group; 0 when that does not apply.
size_t gemv_down_lds_slots_workspace_bytes(const Params &p, int batch) {
  DownPlan plan;
  if (p.orientation != 1 || p.n_groups < 2 || p.n_groups > 64 || !pair_ok(p)) return 0;
  if (!make_down_plan(p, 1, &plan, p.n_groups)) return 0;
  return ((size_t)p.n_groups * ((size_t)batch * (size_t)p.out_features + 16) * sizeof(float) + 255) / 256 * 256;
}

// The groups' sums into part [groups][batch][out_features] and part_xs [groups][16]; the caller adds them up.
int launch_gemv_down_lds_slots(const Params &p, const __half *x, long long ldx, int batch, float *part, float *part_xs, hipStream_t s) {
  if (p.orientation != 1 || !pair_ok(p)) return VQ_ERR_UNSUPPORTED;
  int done = 0, g_max = 4;
  while (done < batch) {
    int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
    if (g > g_max) g = g_max;
    int rc = VQ_ERR_UNSUPPORTED;
    float *pt = part + (size_t)done * p.out_features, *px = part_xs + done;
    const __half *xd = x + done * ldx;
#define VQ_PAIR(V, BITS)                                                                                                  \
    if (p.v == V && p.bits == BITS)                                                                                       \
      rc = g == 1 ? launch_one_slots<V, BITS, 1>(p, xd, ldx, batch, pt, px, s) : g == 2 ? launch_one_slots<V, BITS, 2>(p, xd, ldx, batch, pt, px, s) \
                                                                                        : launch_one_slots<V, BITS, 4>(p, xd, ldx, batch, pt, px, s);
    VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(6, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
    if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
    if (rc != VQ_OK) return done ? VQ_ERR_HIP : rc;
    done += g;
  }
  return VQ_OK;
}

}  // namespace vq
