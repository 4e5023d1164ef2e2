// vq_gemv for layers whose vectors run down the output dimension (orientation 1: the paper's own layout, Sec. 3.1 --
// a quantized column is a stack of centroids -- and Algorithm 1), v = 6, 12-bit indices, optional 12- or 8-bit
// residual codebook, batch 1, 2 or 4 per launch (App. "Our Dequantization Implementation", second phase).
//
// Index stream p holds one index per input column and serves output rows 6p .. 6p+5: a gathered centroid meets ONE
// activation and feeds six sums, y[6p + j] += C[idx][j] * x[n].  That is six mixed-precision multiply-adds per gather
// and token (v_fma_mix_f32: fp16 operands, binary32 sum) against three dot products in the row-wise layout, and still
// about nine vector instructions per gather at batch 1 -- under the dozen that keep the LDS gathers (the bound of all
// these kernels) busy.  There is nothing to sum across lanes until a stream ends: a lane keeps its six (times batch)
// sums over all the columns it visits.
//
// Work split: a pass of a wave covers 512 columns of one stream, eight per lane (their 96 index bits are three
// aligned dwords, their activations one 16-byte LDS read per token).  A stream's passes go to WS = 1, 2, 4 or 8 waves of
// a workgroup (chosen on the host so that the workgroups fill the chip); a workgroup holds the tables and the
// activation rows in LDS and takes several groups of 8 / WS streams in turn.  Index words run DEPTH passes ahead in a
// register ring.  A stream ends with a wave-wide sum of the 6 x batch values, a meeting of the WS waves in LDS when
// WS > 1, and y = scale * sum + bias * sum(x) per output row.
//
// Outlier columns (Sec. 3.2.3; their streams belong to blocks of v_out rows, any v_out and k_out) are few: before the
// main loop each wave works out, for a share of the workgroup's output rows, the row's sum over the outlier columns --
// lanes over the columns, index and centroid element straight from memory -- and leaves it in LDS for the row's end.
//
// Codebook groups (Sec. 3.1: ranges of columns with tables of their own) run when the caller lends a workspace: workgroups
// [g w, (g + 1) w) see group g as a layer of its own -- its tables, its part of every index stream (a group of 8 n columns
// starts on a dword), its columns of x, the outlier columns with group 0 -- and leave binary32 sums without scale and bias
// in the workspace [group][token][row]; the kernel that adds the groups up is the row-wise layers' (vq_gemv_mfma.hip).
// The outlier columns then are one more "group" of the workspace, and every workgroup of the launch works out its share
// of rows of it (a workgroup that owned all the rows of one group of columns would spend longer on them than on its own).
#include "vq_common.hpp"
#include "vq_v6.hpp"

namespace vq {
namespace {

using namespace v6;

constexpr int DW = 8;            // waves per workgroup
constexpr int DEPTH = 4;         // passes whose index words are in flight or in registers
constexpr int VPL = 8;           // vectors (columns) per lane and pass

struct DownPlan {
  int ws_log2;                   // waves per stream
  int passes;                    // 512-column passes per stream
  int ppw;                       // passes per wave and stream
  int iters;                     // groups of DW >> ws_log2 streams per workgroup
  unsigned lds_x, lds_xsum, lds_part;
  unsigned lds_osum;             // sums over the outlier columns: [workgroup's rows][batch], then [batch] activation sums
  unsigned x_row_bytes;          // one staged activation row: passes * 1024 bytes, zero past the last column
  // codebook groups (0 workgroups per group: none): where the sums go instead of y
  int wgs_per_group, part_batch; // tokens of the whole call: the workspace is [group][part_batch][out_features]
  float *part, *part_xs;         // already moved to this launch's first token
};

// The halves of a dword as binary32 (the compiler folds these conversions into v_fma_mix_f32's operand selects).  The
// dwords are taken as scalars on purpose: a bit cast of a component of a four-wide vector has been miscompiled by this
// hipcc inside unrolled loops (every use read component 0).
// Sum over the wave, the same value in every lane: six DPP steps into lane 63 and a broadcast through a scalar register
// (the shuffle-based wave_sum goes through the LDS crossbar six times, one after the other; a stream ends with 6 x batch sums).
__device__ __forceinline__ float wave_total(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_reduce_to_lane63(v)), 63));
}

__device__ __forceinline__ float half_lo(unsigned w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xFFFFu)); }
__device__ __forceinline__ float half_hi(unsigned w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16)); }

// acc[j] += e_j * x for the six values of one table entry (three dwords) and one activation
__device__ __forceinline__ void mac6(float (&acc)[6], unsigned e0, unsigned e1, unsigned e2, float xf) {
  acc[0] = __builtin_fmaf(half_lo(e0), xf, acc[0]);
  acc[1] = __builtin_fmaf(half_hi(e0), xf, acc[1]);
  acc[2] = __builtin_fmaf(half_lo(e1), xf, acc[2]);
  acc[3] = __builtin_fmaf(half_hi(e1), xf, acc[3]);
  acc[4] = __builtin_fmaf(half_lo(e2), xf, acc[4]);
  acc[5] = __builtin_fmaf(half_hi(e2), xf, acc[5]);
}

template <int RES_BITS, int B>
__global__ __launch_bounds__(DW * 64) void gemv_down_v6_kernel(Params p, DownPlan plan, const __half *__restrict__ x, long long ldx,
                                                               __half *__restrict__ y, long long ldy) {
  typedef Layout<RES_BITS> LY;
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  constexpr int NR = RES_BITS == 12 ? 3 : 2;             // dwords of a lane's residual indices
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int wg = (int)blockIdx.x, n_wg = (int)gridDim.x, grp = 0, col0 = p.n_out;    // col0: column of x that meets stream position 0
  unsigned idx_left = (unsigned)p.S * (unsigned)p.stride, res_left = RES_BITS ? (unsigned)p.S * (unsigned)p.stride_res : 0u;
  if (plan.wgs_per_group > 0) {
    grp = wg / plan.wgs_per_group; wg -= grp * plan.wgs_per_group; n_wg = plan.wgs_per_group;
    const int v_lo = grp * p.Pg;
    p.P = min(p.Pg, p.P - v_lo);
    col0 += v_lo;
    p.cb += (long long)grp * p.k * 6;
    if (RES_BITS) p.cb_res += (long long)grp * p.k_res * 6;
    const unsigned skip = (unsigned)(v_lo >> 3) * 12u, skip_res = (unsigned)(v_lo >> 3) * (unsigned)RES_BITS;
    p.idx += skip; idx_left -= skip;
    if (RES_BITS) { p.idx_res += skip_res; res_left -= skip_res; }
    plan.passes = (p.P + 511) >> 9;
    plan.ppw = (plan.passes + (1 << plan.ws_log2) - 1) >> plan.ws_log2;
  }
  const int WS = 1 << plan.ws_log2, SPW = DW >> plan.ws_log2;      // waves per stream, streams per group
  const int ws_i = wv & (WS - 1), slot = wv >> plan.ws_log2;

  // ---- outlier columns, first half: rows of this workgroup in the order the main loop ends them, item
  // r = ((group it) * SPW + slot) * 6 + j.  A wave takes UNR rows at a time, lanes over the columns.  All loads are
  // unconditional (range-checked; a row past the end reads row 0 and counts as zero) so that they overlap, and the index
  // words of the first batch are asked for here, before the tables are staged, so that their trip to memory overlaps it.
  constexpr int UNR = 6;
  struct OutPre { unsigned w0[UNR], w1[UNR]; float xo[B]; };
  const bool out_ws = plan.wgs_per_group > 0 && p.Q > 0;   // grouped layer: outlier sums of rows [blockIdx * rpw, +rpw) into the workspace
  const bool out_lds = plan.wgs_per_group == 0 && p.Q > 0;
  const int rpw = ((p.out_features + (int)gridDim.x - 1) / (int)gridDim.x);
  const int items = out_ws ? rpw : plan.iters * SPW * 6;
  const __amdgpu_buffer_rsrc_t r_oidx = make_rsrc(p.Q ? p.idx_out : p.idx, p.Q ? (unsigned)p.S_out * (unsigned)p.stride_out : 0u);
  const __amdgpu_buffer_rsrc_t r_ocb = make_rsrc(p.Q ? p.cb_out : p.cb, p.Q ? (unsigned)(p.k_out * p.v_out) * 2u : 0u);
  const __amdgpu_buffer_rsrc_t r_xo = make_rsrc(x, (unsigned)(((long long)(B - 1) * ldx + p.Q) * 2));
  auto item_row = [&](int r) {                           // output row of item r, or -1
    if (out_ws) return r < items && (int)blockIdx.x * rpw + r < p.out_features ? (int)blockIdx.x * rpw + r : -1;
    const int grp_slot = r / 6, j = r - grp_slot * 6;
    const int it_r = grp_slot / SPW, slot_r = grp_slot - it_r * SPW;
    const int o = ((it_r * n_wg + wg) * SPW + slot_r) * 6 + j;
    return r < items && o < p.out_features ? o : -1;
  };
  auto out_issue = [&](int r0, int c, OutPre &pre) {
#pragma unroll
    for (int t = 0; t < B; ++t)
      pre.xo[t] = __half2float(__ushort_as_half((unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_xo, (unsigned)(t * ldx + c) * 2u, 0, 0)));
#pragma unroll
    for (int uu = 0; uu < UNR; ++uu) {
      const int o = max(item_row(r0 + uu * DW), 0);
      const unsigned bit = (unsigned)c * (unsigned)p.bits_out;
      const unsigned woff = (unsigned)(o / p.v_out) * (unsigned)p.stride_out + (bit >> 5) * 4u;
      pre.w0[uu] = __builtin_amdgcn_raw_buffer_load_b32(r_oidx, woff, 0, 0);
      pre.w1[uu] = __builtin_amdgcn_raw_buffer_load_b32(r_oidx, woff + 4u, 0, 0);
    }
  };
  auto out_finish = [&](int r0, int c, const OutPre &pre, float (&part_o)[UNR][B]) {
#pragma unroll
    for (int uu = 0; uu < UNR; ++uu) {
      const int o = item_row(r0 + uu * DW);
      const bool ok = o >= 0 && c < p.Q;
      const int oc = max(o, 0), jo = oc - (oc / p.v_out) * p.v_out;
      const unsigned bit = (unsigned)c * (unsigned)p.bits_out;
      const unsigned i = min(__builtin_amdgcn_alignbit(pre.w1[uu], pre.w0[uu], bit & 31u) & ((1u << p.bits_out) - 1u), (unsigned)p.k_out - 1u);
      const unsigned short wh = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_ocb, (i * (unsigned)p.v_out + (unsigned)jo) * 2u, 0, 0);
      const float w = ok ? __half2float(__ushort_as_half(wh)) : 0.0f;
#pragma unroll
      for (int t = 0; t < B; ++t) part_o[uu][t] = __fmaf_rn(w, pre.xo[t], part_o[uu][t]);
    }
  };
  // the table loads, all at once, before everything else of the start-up; stored at its end
  TableStage<RES_BITS, DW * 64> tables{};
  tables.issue(p, 0, false);                             // (p.cb and p.cb_res already point at this workgroup's group)
  OutPre pre0;
  if (p.Q) out_issue(wv, lane, pre0);

  // ---- tables into LDS (16-byte entries, zero past k), activation rows (zero past the last column), their sums
  {
    float *xsum = reinterpret_cast<float *>(lds + plan.lds_xsum);             // [B][DW]
#pragma unroll
    for (int t = 0; t < B; ++t) {
      const __half *xt = x + (long long)t * ldx + col0;                      // stream position n is column col0 + n
      const bool wide = (col0 & 7) == 0;                                     // then the 16-byte pieces are aligned (x is, on the host's word)
      float sum = 0.0f;
      for (int c = (int)threadIdx.x * 8; c < plan.passes * 512; c += DW * 64 * 8) {
        uint4v val = {0u, 0u, 0u, 0u};
        if (wide && c + 8 <= p.P) {
          val = *reinterpret_cast<const uint4v *>(xt + c);
        } else if (c < p.P) {
          unsigned short h[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) h[i] = c + i < p.P ? __half_as_ushort(xt[c + i]) : (unsigned short)0;
          val.x = h[0] | ((unsigned)h[1] << 16); val.y = h[2] | ((unsigned)h[3] << 16);
          val.z = h[4] | ((unsigned)h[5] << 16); val.w = h[6] | ((unsigned)h[7] << 16);
        }
        *reinterpret_cast<uint4v *>(lds + plan.lds_x + (unsigned)t * plan.x_row_bytes + (unsigned)c * 2u) = val;
        sum += half_pair_sum(val.x) + half_pair_sum(val.y) + half_pair_sum(val.z) + half_pair_sum(val.w);
      }
      sum = wave_sum(sum);
      if (lane == 0) xsum[t * DW + wv] = sum;
    }
  }
  if (p.Q) {
    float *osum = reinterpret_cast<float *>(lds + plan.lds_osum);
    for (int r0 = wv; r0 < items; r0 += DW * UNR) {
      float part_o[UNR][B];
#pragma unroll
      for (int uu = 0; uu < UNR; ++uu)
#pragma unroll
        for (int t = 0; t < B; ++t) part_o[uu][t] = 0.0f;
      for (int c0 = 0; c0 < p.Q; c0 += 64) {
        if (r0 == wv && c0 == 0) {
          out_finish(r0, lane, pre0, part_o);          // the loads issued before the tables were staged
        } else {
          OutPre pre;
          out_issue(r0, c0 + lane, pre);
          out_finish(r0, c0 + lane, pre, part_o);
        }
      }
#pragma unroll
      for (int uu = 0; uu < UNR; ++uu)
#pragma unroll
        for (int t = 0; t < B; ++t) {
          const float tot = wave_total(part_o[uu][t]);
          const int o_ws = item_row(r0 + uu * DW);
          if (out_ws) {
            if (lane == 0 && o_ws >= 0) plan.part[((long long)p.n_groups * plan.part_batch + t) * p.out_features + o_ws] = tot;
          } else if (lane == 0 && r0 + uu * DW < items) {
            osum[(r0 + uu * DW) * B + t] = tot;
          }
        }
    }
    if (wv == 0) {                                       // activation sums over the outlier columns
#pragma unroll
      for (int t = 0; t < B; ++t) {
        float sx = 0.0f;
        for (int c = lane; c < p.Q; c += 64) sx += __half2float(x[(long long)t * ldx + c]);
        sx = wave_sum(sx);
        if (lane == 0) {
          if (out_ws) { if (blockIdx.x == 0) plan.part_xs[p.n_groups * 16 + t] = sx; }
          else osum[items * B + t] = sx;
        }
      }
    }
  }
  const unsigned st_main = (unsigned)p.stride, st_res = (unsigned)p.stride_res;
  const __amdgpu_buffer_rsrc_t r_main = make_rsrc(p.idx, idx_left);
  const __amdgpu_buffer_rsrc_t r_res = make_rsrc(RES_BITS ? p.idx_res : p.idx, res_left);
  const unsigned a_x = lds_address(lds) + plan.lds_x + (unsigned)lane * 16u;

  // The wave's work is one sequence of units, unit k = (group k / ppw of streams, pass k % ppw of this wave in the stream).
  // A unit past the end of the streams or of a stream's passes is walked like any other -- the barriers below need every
  // wave -- on the first stream's first pass, and its products are dropped.
  const int K = plan.iters * plan.ppw;
  auto unit_stream = [&](int it) { return (it * n_wg + wg) * SPW + slot; };
  int l_it = 0, l_i = 0;                               // the loader's position in the same sequence, DEPTH units ahead
  auto load_unit = [&](Window<3> &wm, Window<NR> &wr) {
    const int stream = unit_stream(l_it), q = ws_i + l_i * WS;
    const bool on = l_it < plan.iters && stream < p.S && q < plan.passes;
    if (++l_i == plan.ppw) { l_i = 0; ++l_it; }
    const unsigned s_off = on ? (unsigned)stream : 0u, q_off = on ? (unsigned)q : 0u;
    load_window(wm, r_main, s_off * st_main + q_off * 768u + (unsigned)lane * 12u, 0u);
    if (RES_BITS == 12) load_window(wr, r_res, s_off * st_res + q_off * 768u + (unsigned)lane * 12u, 0u);
    if (RES_BITS == 8) load_window(wr, r_res, s_off * st_res + q_off * 512u + (unsigned)lane * 8u, 0u);
  };

  Window<3> win[DEPTH];
  Window<NR> wres[DEPTH];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) load_unit(win[d], wres[d]);

  // The ring's loads (from HBM) have gone out behind everything else of the start-up and are not waited for here: loads
  // return in order, so "all but the ring's" means the tables are in, and the barrier waits for LDS traffic only.
  wait_vmem_at_most<DEPTH * (RES_BITS ? 2 : 1)>();
  tables.store(p, lds, 0u, false);
  lds_barrier();


  float acc[B][6];
#pragma unroll
  for (int t = 0; t < B; ++t)
#pragma unroll
    for (int j = 0; j < 6; ++j) acc[t][j] = 0.0f;
  float *part = reinterpret_cast<float *>(lds + plan.lds_part);               // [DW][B * 6]
  const float *osum = reinterpret_cast<const float *>(lds + plan.lds_osum);
  const float *xsum = reinterpret_cast<const float *>(lds + plan.lds_xsum);

  int it = 0, i = 0;                                   // group and pass-of-this-wave of the current unit
  for (int k0 = 0; k0 < K; k0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int k = k0 + d;
      if (k < K) {
        const int stream = unit_stream(it), q = ws_i + i * WS;
        const bool on = stream < p.S && q < plan.passes;
        const Window<3> cm = win[d];
        const Window<NR> cr = wres[d];
        load_unit(win[d], wres[d]);                    // refill the slot; the copies above are what this unit uses
        if (on) {
          uint4v e[VPL], f[VPL];
#pragma unroll
          for (int u = 0; u < VPL; ++u) lds_gather16<LY::MAIN_OFF>(e[u], field_addr<12, LY::MAIN_SH>(cm, u));
          if (RES_BITS) {
#pragma unroll
            for (int u = 0; u < VPL; ++u) lds_gather16<LY::RES_OFF>(f[u], field_addr<RB, LY::RES_SH>(cr, u) + LY::RES_ADD);
          }
          uint4v xv[B];
#pragma unroll
          for (int t = 0; t < B; ++t)
            asm volatile("ds_read_b128 %0, %1" : "=v"(xv[t]) : "v"(a_x + (unsigned)t * plan.x_row_bytes + (unsigned)q * 1024u));
          lds_gather_wait();
#pragma unroll
          for (int u = 0; u < VPL; ++u) { settle(e[u]); if (RES_BITS) settle(f[u]); }
#pragma unroll
          for (int t = 0; t < B; ++t) {
            settle(xv[t]);
            const unsigned xd[4] = {xv[t].x, xv[t].y, xv[t].z, xv[t].w};
#pragma unroll
            for (int u = 0; u < VPL; ++u) {
              const float xf = (u & 1) ? half_hi(xd[u >> 1]) : half_lo(xd[u >> 1]);
              mac6(acc[t], e[u].x, e[u].y, e[u].z, xf);
              if (RES_BITS) mac6(acc[t], f[u].x, f[u].y, f[u].z, xf);
            }
          }
        }
        if (i == plan.ppw - 1) {
          // ---- the stream ends for this wave: sum over the lanes, meet the other waves of the stream, store
          float mine = 0.0f;                           // lane l < 6 B keeps value (token l / 6, row l % 6)
#pragma unroll
          for (int t = 0; t < B; ++t)
#pragma unroll
            for (int j = 0; j < 6; ++j) {
              const float s = wave_total(acc[t][j]);
              if (lane == t * 6 + j) mine = s;
              acc[t][j] = 0.0f;
            }
          if (WS > 1) {
            if (lane < 6 * B) part[wv * (6 * B) + lane] = mine;
            lds_barrier();
            if (ws_i == 0 && lane < 6 * B) {
              mine = 0.0f;
              for (int w = 0; w < WS; ++w) mine += part[(wv + w) * (6 * B) + lane];
            }
          }
          if (ws_i == 0 && lane < 6 * B && stream < p.S) {
            const int t = lane / 6, o = stream * 6 + (lane - t * 6);
            if (o < p.out_features) {
              float xs = 0.0f;
#pragma unroll
              for (int w = 0; w < DW; ++w) xs += xsum[t * DW + w];
              if (out_lds) {
                mine += osum[((it * SPW + slot) * 6 + (lane - t * 6)) * B + t];
                xs += osum[plan.iters * SPW * 6 * B + t];
              }
              if (plan.part) {                          // one group of several: the sum as it is, for the kernel that adds the groups up
                plan.part[((long long)grp * plan.part_batch + t) * p.out_features + o] = mine;
                if (wg == 0 && slot == 0 && it == 0 && lane - t * 6 == 0) plan.part_xs[grp * 16 + t] = xs;
              } else {
                const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
                y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(sc, mine, bi * xs));
              }
            }
          }
          if (WS > 1) lds_barrier();                   // the partial sums are free again
          i = 0; ++it;
        } else {
          ++i;
        }
      }
    }
  }
}


template <int RES_BITS, int B>
int launch_one(const Params &p, const DownPlan &plan, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx, __half *y,
               long long ldy, hipStream_t s) {
  auto kernel = gemv_down_v6_kernel<RES_BITS, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(DW * 64), lds_bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Whether the kernel above takes this layer and these buffers.
bool gemv_down_applicable(const Params &p, const __half *x, long long ldx) {
  if (p.orientation != 1 || p.v != 6 || p.bits != 12) return false;
  if (p.n_groups > 1 && (p.Pg & 7)) return false;        // a group starts on a dword of the index streams (and needs a workspace)
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (ldx & 7)) return false;
  const long long max_stride = p.stride > p.stride_res ? p.stride : p.stride_res;
  return (long long)p.S * max_stride < (1LL << 31);                          // 32-bit buffer offsets
}

namespace {
// Work split and LDS layout for one group of `batch` rows; VQ_ERR_UNSUPPORTED when the rows do not fit LDS beside the tables.
int make_plan(const Params &p, int batch, float *part, float *part_xs, int part_batch, DownPlan *out, unsigned *lds_bytes, unsigned *grid_out) {
  DownPlan plan{};
  if ((p.n_groups > 1) != (part != nullptr)) return VQ_ERR_UNSUPPORTED;
  plan.part = part; plan.part_xs = part_xs; plan.part_batch = part_batch;
  const int rb = p.k_res ? p.bits_res : 0;
  unsigned off = rb == 0 ? Layout<0>::BYTES : rb == 8 ? Layout<8>::BYTES : Layout<12>::BYTES;
  plan.passes = (min(p.P, p.Pg) + 511) / 512;            // of the widest codebook group
  plan.x_row_bytes = (unsigned)plan.passes * 1024u;
  if ((unsigned long long)plan.x_row_bytes * (unsigned)batch > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  plan.lds_x = off; off += plan.x_row_bytes * (unsigned)batch;
  plan.lds_xsum = off; off += (unsigned)(batch * DW) * 4u;
  plan.lds_part = off; off += (unsigned)(DW * 6 * batch) * 4u;
  plan.lds_osum = off;                                   // sized below, once the groups per workgroup are known
  // waves per stream: the choice with the fewest passes on the busiest wave, a stream's end counted as a third of a pass
  // (half when waves have to meet)
  const int cus = part ? max(1, cu_count() / p.n_groups) : cu_count();      // workgroups one group of columns gets
  double best = 1e30;
  unsigned grid = 1;
  for (int l = 0; l <= 3; ++l) {
    const int WS = 1 << l, groups = (p.S + (DW >> l) - 1) / (DW >> l);
    const int iters = (groups + cus - 1) / cus, ppw = (plan.passes + WS - 1) / WS;
    const double cost = iters * (ppw + (l ? 0.5 : 0.33));
    if (cost < best) { best = cost; plan.ws_log2 = l; plan.ppw = ppw; plan.iters = iters; grid = (unsigned)((groups + iters - 1) / iters); }
  }
  off += p.Q ? (unsigned)((plan.iters * (DW >> plan.ws_log2) * 6 + 1) * batch) * 4u : 0u;
  if (off > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  if (part) { plan.wgs_per_group = (int)grid; grid *= (unsigned)p.n_groups; }
  *out = plan; *lds_bytes = off; *grid_out = grid;
  return VQ_OK;
}
}  // namespace

// Whether one row of a layer without codebook groups fits the kernel above (its activations beside the tables in LDS).
bool gemv_down_fits(const Params &p) {
  DownPlan plan;
  unsigned off, grid;
  return p.n_groups == 1 && make_plan(p, 1, nullptr, nullptr, 0, &plan, &off, &grid) == VQ_OK;
}

// Launch for one group of 1, 2 or 4 batch rows.  VQ_ERR_UNSUPPORTED when the rows do not fit LDS beside the tables.
// part != nullptr: a layer with codebook groups; the sums go to the workspace part[group][part_batch][out_features] (and
// part_xs[group * 16 + token]), both already moved to this launch's first token.
int launch_gemv_down(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s,
                     float *part, float *part_xs, int part_batch) {
  DownPlan plan;
  unsigned off, grid;
  const int rc = make_plan(p, batch, part, part_xs, part_batch, &plan, &off, &grid);
  if (rc != VQ_OK) return rc;
  const int rb = p.k_res ? p.bits_res : 0;
#define VQ_CASE(R, BB) if (rb == R && batch == BB) return launch_one<R, BB>(p, plan, off, grid, x, ldx, y, ldy, s);
  VQ_CASE(0, 1) VQ_CASE(12, 1) VQ_CASE(8, 1)
  VQ_CASE(0, 2) VQ_CASE(12, 2) VQ_CASE(8, 2)
  VQ_CASE(0, 4) VQ_CASE(12, 4) VQ_CASE(8, 4)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
