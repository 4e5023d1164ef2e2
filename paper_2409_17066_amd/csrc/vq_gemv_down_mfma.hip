// vq_gemv on the matrix cores for layers whose vectors run down the output dimension (orientation 1: the paper's own
// layout, Sec. 3.1 and Algorithm 1), v = 6, 12-bit indices, optional 12- or 8-bit residual codebook, outlier columns,
// any batch up to 16 in one launch (App. "Our Dequantization Implementation", second phase), one or more codebook groups.
//
// In this layout a gathered centroid meets ONE activation and feeds six output rows, y[6p + j] += C[I[p][n]][j] * x[n]:
// on the vector ALUs that is six multiply-adds per gather and token, and from four tokens on the kernel of
// vq_gemv_down.hip is bound by them.  One v_mfma_f32_16x16x32_f16 takes their place.  Its 32 "k" slots are four groups
// of eight; a group is one column n of the layer, and the eight slots are the six elements j' of the centroid of that
// column plus two zeros -- exactly the 16-byte table entry in LDS, as operand A of the stream (l & 15).  Operand B is
// built to match: its 16 columns are (token, j) pairs -- the 6 x batch pairs of a launch are dealt out 16 to an
// instruction, ceil(6 batch / 16) instructions per step -- and the value in slot (n, j') of column (t, j) is x[t][n] where
// j' = j and zero elsewhere.  The product then is D[stream][(t, j)] = sum over the four columns of
// C[I[stream][n]][j] * x[t][n]: 16 streams x 4 columns x 2 2/3 tokens per instruction, an eighth of its multiply-adds put
// to use, and still several times the rate of the vector ALUs.  A lane builds one B operand with three byte permutes
// (v_perm_b32 with per-lane selectors that place one half of an activation dword and zero the rest).
//
// Work split: a workgroup of eight waves owns one block of 16 index streams (96 output rows) and one part of the
// columns; wave w takes the part's windows w, w + 8, ... of 32 columns (eight per lane: 96 index bits, three aligned
// dwords; its eight activations per token are one 16-byte load, read straight from memory -- they are hits in L2 --
// with range-checked buffer loads).  Index words and activations run a few windows ahead in a register ring.  At the
// end the waves' 16 x 16 sums per token pair meet in LDS, in the space of the tables, which are no longer needed.
// With one part the workgroup applies y = scale * sum + bias * sum(x) itself; a block of 16 streams is a coarse unit,
// though (a 4096 x 4096 layer has 43 of them for 256 compute units), so when the caller lends a workspace the columns
// are cut into parts, every (block, part) is a workgroup, the binary32 sums go to the workspace [part][token][row] and
// the kernel that adds up codebook groups (vq_gemv_mfma.hip) adds up the parts.  Codebook groups (Sec. 3.1: ranges of
// columns with tables of their own) are parts by nature -- a part stages the tables of its group -- and are cut further
// the same way; without a workspace the workgroup of a block walks the groups one after the other, swapping the tables
// in LDS, with its sums running on.
#include "vq_common.hpp"
#include "vq_v6.hpp"

namespace vq {
namespace {

using namespace v6;

constexpr int MW = 8;            // waves per workgroup
constexpr int VPL = 8;           // columns per lane and window

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

struct DownMfmaPlan {
  int ksplit;                    // parts of the columns; grid = blocks of 16 streams x ksplit
  int sub;                       // parts per codebook group: ksplit = groups x sub
  int wpp;                       // 32-column windows per part
  int batch;
  unsigned x_bytes;              // from x[0][0] to the end of the last token's row
  float *part, *part_xs;         // workspace [part][batch][out_features], [part * 16 + token]; nullptr: one part, the kernel stores y
  // outlier columns: the workgroup's rows of them as a dense tile in LDS
  unsigned lds_o;                // [OROWS][o_pitch] dwords of weights, [16][o_pitch] of activations, [16][OROWS] sums, [16] activation sums
  int o_pitch;                   // dwords per tile row: ceil(Q / 2), made odd (rows then start in different banks)
  int o_rpw;                     // with a workspace: rows per workgroup (the rows are dealt out to all workgroups of the launch)
};

constexpr int OROWS = 96;        // rows of outlier sums a workgroup works out: its own block's, or its share of all rows (never more)

__device__ __forceinline__ float4v mfma16(uint4v a, uint4v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
}

// WALK: the instantiation for layers with codebook groups and no workspace, whose workgroups walk all groups; the others
// take one group (or the only one) and have no loop around the start-up (with the loop in every instantiation the
// single-group ones lost up to 4 us on a 4096 x 4096 layer in 16 groups: registers held across the loop edge).
// `wg` is the workgroup's number within its layer (a launch may hold the workgroups of several layers).
// NTP: instructions per step, each with 16 of the 6 x batch (token, row) pairs as operand columns.
template <int RES_BITS, int NTP, bool WALK>
__device__ __forceinline__ void gemv_down_mfma_body(const Params &p, const DownMfmaPlan &plan, const __half *__restrict__ x, long long ldx,
                                                    __half *__restrict__ y, long long ldy, int wg) {
  typedef Layout<RES_BITS> LY;
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  constexpr int NR = RES_BITS == 12 ? 3 : 2;             // dwords of a lane's residual indices
  // (measured: a ring deeper than this only adds start-up loads -- a wave of a column part has few windows -- and the
  // refill of a slot already runs a window ahead of its use; 4 deep -> 1 deep: 4096 x 4096 with residual and workspace,
  // batch 4, 14.1 -> 12.9 us; q+k+v fused, batch 4, 24.4 -> 22.1 us)
  constexpr int DEPTH = (NTP == 1 && RES_BITS == 0) ? 2 : 1;
  constexpr bool LATE_X = NTP >= 6;                      // registers: refill a slot's activations only after the window's last product
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;                // A: stream n of the block, column group g.  B and D: column n = (token, j)
  const int blk = wg / plan.ksplit, part_i = wg - blk * plan.ksplit;
  // A part belongs to one codebook group; without a workspace the workgroup walks all groups, one set of tables after the
  // other in LDS, and its sums simply keep running (the tables change with the column, the output rows do not).
  const int g_lo = plan.part ? part_i / plan.sub : 0, g_hi = WALK ? p.n_groups : g_lo + 1;
  const int sub_i = plan.part ? part_i - g_lo * plan.sub : 0;
  const bool need_xs = plan.part == nullptr || blk == 0;

  // ---- outlier columns (Sec. 3.2.3; any v_out and k_out; their index streams belong to blocks of v_out rows): few columns, so
  // the workgroup's rows of them are restored into a dense tile in LDS -- every (row, column) is independent: one trip to the
  // index streams, one to the table, for all of them at once -- and multiplied from there once the barrier below has passed.
  // Without a workspace the rows are the block's own and their sums wait in LDS for the end; with one, the outlier columns
  // are one more part of the workspace and every workgroup of the launch takes a share of ALL rows.
  const int o_row_lo = plan.part ? wg * plan.o_rpw : blk * OROWS;
  const int o_rows = p.Q ? max(0, min(plan.part ? plan.o_rpw : OROWS, p.out_features - o_row_lo)) : 0;
  const int Q2 = 2 * plan.o_pitch;                       // halves per tile row
  unsigned short *o_tile = reinterpret_cast<unsigned short *>(lds + plan.lds_o);
  unsigned short *o_x = o_tile + OROWS * Q2;
  float *o_sum = reinterpret_cast<float *>(o_x + 16 * Q2), *o_xs = o_sum + 16 * OROWS;
  // ---- this lane's side of operand B
  // (operand column n of instruction m is pair 16 m + n of the 6 x batch (token, row j) pairs: token (16 m + n) / 6, row
  // (16 m + n) % 6 = (n + 4 (m % 3)) % 6 -- three patterns of rows; pairs past the batch read zero activations)
  auto token_of = [&](int m) { return (16 * m + n) / 6; };
  auto row_of = [&](int m) { return (16 * m + n) % 6; };
  // byte selectors that move the low (even column) or high (odd column) half of an activation dword into half (j & 1) of
  // dword (j >> 1) of the operand, zeros (selector byte 0x0c) everywhere else
  constexpr int NPAT = NTP < 3 ? NTP : 3;
  unsigned sel[NPAT][3][2];
#pragma unroll
  for (int pm = 0; pm < NPAT; ++pm) {
    const int j = row_of(pm);
#pragma unroll
    for (int d = 0; d < 3; ++d) {
      const bool mine = d == (j >> 1);
      sel[pm][d][0] = !mine ? 0x0c0c0c0cu : (j & 1) ? 0x01000c0cu : 0x0c0c0100u;
      sel[pm][d][1] = !mine ? 0x0c0c0c0cu : (j & 1) ? 0x03020c0cu : 0x0c0c0302u;
    }
  }
  const unsigned st_main = (unsigned)p.stride, st_res = (unsigned)p.stride_res;
  const __amdgpu_buffer_rsrc_t r_main = make_rsrc(p.idx, (unsigned)p.S * st_main);
  const __amdgpu_buffer_rsrc_t r_res = make_rsrc(RES_BITS ? p.idx_res : p.idx, RES_BITS ? (unsigned)p.S * st_res : 0u);
  const __amdgpu_buffer_rsrc_t r_x = make_rsrc(x, plan.x_bytes);
  float4v acc[NTP];
  float xs[NTP];
#pragma unroll
  for (int tp = 0; tp < NTP; ++tp) { acc[tp] = float4v{0.0f, 0.0f, 0.0f, 0.0f}; xs[tp] = 0.0f; }

  for (int grp = g_lo; grp < g_hi; ++grp) {
    // the group's stream positions [pos_lo, pos_hi) -- pos_lo a multiple of 8, a dword boundary of the streams -- and the
    // part's windows, counted from pos_lo; a part past a short last group has none and leaves zeros
    const int pos_lo = grp * p.Pg, pos_hi = min(p.P, pos_lo + p.Pg);
    const int windows = (pos_hi - pos_lo + 31) >> 5;
    const int w_lo = sub_i * plan.wpp, w_hi = min(windows, w_lo + plan.wpp);
    const int my_n = w_hi - w_lo > wv ? (w_hi - w_lo - wv + MW - 1) / MW : 0;  // this wave's windows: w_lo + wv + i * MW
    if (WALK && grp > g_lo) __syncthreads();             // every wave is done with the tables of the group before

    // ---- tables into LDS: 16-byte entries, zero past k (an index past k, or read beyond a stream's end, meets zeros or a
    // finite entry and a zero activation).  All their loads are asked for here, at once; they are stored after everything
    // else of the start-up has been asked for as well (a loop of load-and-store rounds costs a trip to L2 per round).
    // (The thread id is made opaque in every round, or the table addresses derived from it would stay in registers
    // through the main loop for the next group.)
    unsigned tid = threadIdx.x;
    if (WALK) asm volatile("" : "+v"(tid));
    TableStage<RES_BITS, MW * 64> tables{};
    tables.issue(p, grp, false, tid);
    if (grp == g_lo && p.Q) {
      {
        const __amdgpu_buffer_rsrc_t r_oidx = make_rsrc(p.idx_out, (unsigned)p.S_out * (unsigned)p.stride_out);
        const __amdgpu_buffer_rsrc_t r_ocb = make_rsrc(p.cb_out, (unsigned)(p.k_out * p.v_out) * 2u);
        constexpr int OU = 4;                                // entries a thread has in flight
        const int total = o_rows * Q2;
        for (int e0 = (int)threadIdx.x; e0 < total; e0 += MW * 64 * OU) {
          unsigned w0[OU], w1[OU], sh[OU], jo[OU];
          bool ok[OU];
#pragma unroll
          for (int uu = 0; uu < OU; ++uu) {
            const int e = e0 + uu * MW * 64, r = e / Q2, c = e - r * Q2;
            ok[uu] = e < total && c < p.Q;
            const int o = o_row_lo + (ok[uu] ? r : 0), sq = o / p.v_out;
            const unsigned bit = (unsigned)(ok[uu] ? c : 0) * (unsigned)p.bits_out;
            const unsigned woff = (unsigned)sq * (unsigned)p.stride_out + (bit >> 5) * 4u;
            jo[uu] = (unsigned)(o - sq * p.v_out); sh[uu] = bit & 31u;
            w0[uu] = __builtin_amdgcn_raw_buffer_load_b32(r_oidx, woff, 0, 0);
            w1[uu] = __builtin_amdgcn_raw_buffer_load_b32(r_oidx, woff + 4u, 0, 0);
          }
#pragma unroll
          for (int uu = 0; uu < OU; ++uu) {
            const unsigned i = min(__builtin_amdgcn_alignbit(w1[uu], w0[uu], sh[uu]) & ((1u << p.bits_out) - 1u), (unsigned)p.k_out - 1u);
            const unsigned short wh = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_ocb, (i * (unsigned)p.v_out + jo[uu]) * 2u, 0, 0);
            const int e = e0 + uu * MW * 64;
            if (e < total) o_tile[e] = ok[uu] ? wh : (unsigned short)0;
          }
        }
        for (int e = (int)threadIdx.x; e < 16 * Q2; e += MW * 64) {
          const int t = e / Q2, c = e - t * Q2;
          o_x[e] = t < plan.batch && c < p.Q ? __half_as_ushort(x[(long long)t * ldx + c]) : (unsigned short)0;
        }
      }

    }

    // byte offset of this lane's first activation of window 0, per token pair; a token past the batch (and the idle columns)
    // reads out of range, i.e. zeros
    const int col0 = p.n_out + pos_lo;                     // column of x that meets the part's window 0
    unsigned xoff[NTP];
#pragma unroll
    for (int tp = 0; tp < NTP; ++tp) {
      const int t = token_of(tp);
      xoff[tp] = t < plan.batch ? (unsigned)(((long long)t * ldx + col0 + 8 * g) * 2) : 0x80000000u;
    }

    // a stream past the last one reads out of range: index 0, whose products land in rows that are never stored
    const unsigned srow_main = (unsigned)(blk * 16 + n) * st_main + (unsigned)(pos_lo >> 3) * 12u;
    const unsigned srow_res = (unsigned)(blk * 16 + n) * st_res + (unsigned)(pos_lo >> 3) * (unsigned)RB;

    // The loaders run DEPTH windows ahead of the consumer.  A slot's index words are refilled as soon as the gather
    // addresses have been formed from them; so are its activations, from a copy, except with 16 tokens, where the copy
    // would not fit the registers and the refill waits for the window's last product.
    int lw = w_lo + wv, lwx = w_lo + wv;
    auto load_idx = [&](Window<3> &wm, Window<NR> &wr) {
      const unsigned wq = (unsigned)(lw < w_hi ? lw : w_lo);                   // past the end: any window in range, never used
      lw += MW;
      load_window(wm, r_main, srow_main + (wq * 4u + (unsigned)g) * 12u, 0u);
      if (RES_BITS == 12) load_window(wr, r_res, srow_res + (wq * 4u + (unsigned)g) * 12u, 0u);
      if (RES_BITS == 8) load_window(wr, r_res, srow_res + (wq * 4u + (unsigned)g) * 8u, 0u);
    };
    auto load_x = [&](uint4v (&xx)[NTP]) {
      const unsigned wq = (unsigned)(lwx < w_hi ? lwx : w_lo);
      lwx += MW;
#pragma unroll
      for (int tp = 0; tp < NTP; ++tp) xx[tp] = __builtin_amdgcn_raw_buffer_load_b128(r_x, xoff[tp] + wq * 64u, 0, 0);
    };

    Window<3> win[DEPTH];
    Window<NR> wres[DEPTH];
    uint4v xr[DEPTH][NTP];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) { load_idx(win[d], wres[d]); load_x(xr[d]); }
    // the table loads are older than the ring's (loads return in order): at most the ring's may still be on their way
    wait_vmem_at_most<DEPTH * (1 + (RES_BITS ? 1 : 0) + NTP)>();
    tables.store(p, lds, 0u, false, tid);
    lds_barrier();                                       // the tables are in (a full barrier would also wait for the ring's loads from HBM)

    if (grp == g_lo && p.Q) {
      {                                                  // the outlier tile times the activations: a thread per (row, four tokens)
        const unsigned *wt = reinterpret_cast<const unsigned *>(o_tile), *xt = reinterpret_cast<const unsigned *>(o_x);
        const int ntg = (plan.batch + 3) >> 2;
        for (int i = (int)threadIdx.x; i < o_rows * ntg; i += MW * 64) {
          const int tg = i / o_rows, r = i - tg * o_rows;
          float a[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          for (int c2 = 0; c2 < plan.o_pitch; ++c2) {
            const unsigned wd = wt[r * plan.o_pitch + c2];
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) a[tt] = dot2(wd, xt[(tg * 4 + tt) * plan.o_pitch + c2], a[tt]);
          }
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) {
            const int t = tg * 4 + tt;
            if (t < plan.batch) {
              if (plan.part) plan.part[((long long)plan.ksplit * plan.batch + t) * p.out_features + o_row_lo + r] = a[tt];
              else o_sum[t * OROWS + r] = a[tt];
            }
          }
        }
        if ((int)threadIdx.x < plan.batch) {                 // activation sums over the outlier columns
          float sx = 0.0f;
          for (int c2 = 0; c2 < plan.o_pitch; ++c2) sx += half_pair_sum(xt[(int)threadIdx.x * plan.o_pitch + c2]);
          if (!plan.part) o_xs[threadIdx.x] = sx;
          else if (wg == 0) plan.part_xs[plan.ksplit * 16 + (int)threadIdx.x] = sx;
        }
      }

    }

    for (int k0 = 0; k0 < my_n; k0 += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        const int k = k0 + d;
        if (k < my_n) {
          const int w = w_lo + wv + k * MW;
          const Window<3> cm = win[d];
          const Window<NR> cr = wres[d];
          uint4v xv[NTP];
#pragma unroll
          for (int tp = 0; tp < NTP; ++tp) xv[tp] = xr[d][tp];
          load_idx(win[d], wres[d]);                     // refill the slot; the copies above are what this window uses
          if (!LATE_X) load_x(xr[d]);
          uint4v e[VPL], f[RES_BITS ? VPL : 1];
#pragma unroll
          for (int u = 0; u < VPL; ++u) lds_gather16<LY::MAIN_OFF>(e[u], field_addr<12, LY::MAIN_SH>(cm, u));
          if (RES_BITS) {
#pragma unroll
            for (int u = 0; u < VPL; ++u) lds_gather16<LY::RES_OFF>(f[u], field_addr<RB, LY::RES_SH>(cr, u) + LY::RES_ADD);
          }
          if (w == windows - 1) {                          // the window that holds the end of the stream or of the group: zero what lies past it
            const int left = pos_hi - pos_lo - (w * 32 + g * 8);               // of this lane's eight positions
#pragma unroll
            for (int tp = 0; tp < NTP; ++tp) {
              unsigned xd[4] = {xv[tp].x, xv[tp].y, xv[tp].z, xv[tp].w};
#pragma unroll
              for (int q = 0; q < 4; ++q) xd[q] = left >= 2 * q + 2 ? xd[q] : left == 2 * q + 1 ? xd[q] & 0xFFFFu : 0u;
              xv[tp].x = xd[0]; xv[tp].y = xd[1]; xv[tp].z = xd[2]; xv[tp].w = xd[3];
            }
          }
          if (need_xs) {
#pragma unroll
            for (int tp = 0; tp < NTP; ++tp)
              xs[tp] = dot2(xv[tp].x, 0x3C003C00u, dot2(xv[tp].y, 0x3C003C00u, dot2(xv[tp].z, 0x3C003C00u, dot2(xv[tp].w, 0x3C003C00u, xs[tp]))));
          }
          lds_gather_wait();
#pragma unroll
          for (int u = 0; u < VPL; ++u) { settle(e[u]); if (RES_BITS) settle(f[u]); }
#pragma unroll
          for (int u = 0; u < VPL; ++u) {
#pragma unroll
            for (int tp = 0; tp < NTP; ++tp) {
              const unsigned xd = (u >> 1) == 0 ? xv[tp].x : (u >> 1) == 1 ? xv[tp].y : (u >> 1) == 2 ? xv[tp].z : xv[tp].w;
              uint4v b;
              b.x = __builtin_amdgcn_perm(xd, xd, sel[tp % 3][0][u & 1]);
              b.y = __builtin_amdgcn_perm(xd, xd, sel[tp % 3][1][u & 1]);
              b.z = __builtin_amdgcn_perm(xd, xd, sel[tp % 3][2][u & 1]);
              b.w = 0u;
              acc[tp] = mfma16(e[u], b, acc[tp]);
              if (RES_BITS) acc[tp] = mfma16(f[u], b, acc[tp]);
            }
          }
          if (LATE_X) load_x(xr[d]);
        }
      }
    }

  }

  // ---- the waves meet: sums per token pair, 1 KB per wave and pair, in the space of the tables
  __syncthreads();
  float4v *pbuf = reinterpret_cast<float4v *>(lds);                           // [NTP][MW][64]
  float *xsb = reinterpret_cast<float *>(lds + NTP * MW * 1024);              // [MW][16 tokens][4]
#pragma unroll
  for (int tp = 0; tp < NTP; ++tp) {
    pbuf[(tp * MW + wv) * 64 + lane] = acc[tp];
    if (row_of(tp) == 0 && token_of(tp) < plan.batch) xsb[(wv * 16 + token_of(tp)) * 4 + g] = xs[tp];
  }
  __syncthreads();
  if (wv < NTP) {                                        // wave tp finishes token pair tp
    const int tp = wv, t = token_of(tp), j = row_of(tp);
    float4v s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int w = 0; w < MW; ++w) s += pbuf[(tp * MW + w) * 64 + lane];
    if (t < plan.batch) {
      float xsum = 0.0f;
      if (need_xs) {
#pragma unroll
        for (int w = 0; w < MW; ++w)
#pragma unroll
          for (int gg = 0; gg < 4; ++gg) xsum += xsb[(w * 16 + t) * 4 + gg];
      }
      float sv[4] = {s.x, s.y, s.z, s.w};
      if (p.Q && !plan.part) {                           // the block's own outlier sums, left in LDS before the main loop
        xsum += o_xs[t];
#pragma unroll
        for (int r = 0; r < 4; ++r) sv[r] += o_sum[t * OROWS + (4 * g + r) * 6 + j];
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int stream = blk * 16 + 4 * g + r, o = stream * 6 + j;
        if (stream < p.S && o < p.out_features) {
          if (plan.part) {
            plan.part[((long long)part_i * plan.batch + t) * p.out_features + o] = sv[r];
          } else {
            const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
            y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(sc, sv[r], bi * xsum));
          }
        }
      }
      if (plan.part && blk == 0 && g == 0 && j == 0) plan.part_xs[part_i * 16 + t] = xsum;
    }
  }
}

template <int RES_BITS, int NTP, bool WALK>
__global__ __launch_bounds__(MW * 64) void gemv_down_mfma_kernel(Params p, DownMfmaPlan plan, const __half *__restrict__ x, long long ldx,
                                                                 __half *__restrict__ y, long long ldy) {
  gemv_down_mfma_body<RES_BITS, NTP, WALK>(p, plan, x, ldx, y, ldy, (int)blockIdx.x);
}

// Several layers that read the same activations (the query, key and value projections of a decoder layer; its gate and up
// projections) in one launch: every workgroup belongs to one layer and runs the body above on one of its blocks of 16
// streams, over all columns.  This is where the coarse blocks stop hurting without a workspace: the blocks of all the
// layers are in flight together (three 4096 x 4096 layers: 129 workgroups instead of three times 43).
constexpr int DMULTI_MAX = 8;
struct DownMultiLayer {
  Params p;
  DownMfmaPlan plan;
  __half *y;
  long long ldy;
};
struct DownMultiArgs {
  int n;
  int first_wg[DMULTI_MAX + 1];                          // layer i owns workgroups [first_wg[i], first_wg[i + 1])
  DownMultiLayer layer[DMULTI_MAX];
};

template <int RES_BITS, int NTP>
__global__ __launch_bounds__(MW * 64) void gemv_down_mfma_multi_kernel(DownMultiArgs a, const __half *__restrict__ x, long long ldx) {
  int i = 0;
  while (i + 1 < a.n && (int)blockIdx.x >= a.first_wg[i + 1]) ++i;
  gemv_down_mfma_body<RES_BITS, NTP, false>(a.layer[i].p, a.layer[i].plan, x, ldx, a.layer[i].y, a.layer[i].ldy, (int)blockIdx.x - a.first_wg[i]);
}


// LDS of one layer: tables (or the meeting place of the waves, which takes their space at the end), then the outlier tile
template <int RES_BITS, int NTP>
unsigned place_lds(const Params &p, DownMfmaPlan &plan) {
  unsigned lds_bytes = Layout<RES_BITS>::BYTES;
  const unsigned meet = (unsigned)(NTP * MW) * 1024u + (unsigned)(MW * 16 * 4) * 4u;
  if (lds_bytes < meet) lds_bytes = meet;
  plan.lds_o = lds_bytes;
  if (p.Q) lds_bytes += (unsigned)((OROWS + 16) * plan.o_pitch + 16 * OROWS + 16) * 4u;
  return lds_bytes;
}

template <int RES_BITS, int NTP>
int launch_multi(DownMultiArgs &a, const __half *x, long long ldx, hipStream_t s) {
  auto kernel = gemv_down_mfma_multi_kernel<RES_BITS, NTP>;
  VQ_ALLOW_FULL_LDS(kernel);
  unsigned lds_bytes = 0;
  for (int i = 0; i < a.n; ++i) {
    const unsigned b = place_lds<RES_BITS, NTP>(a.layer[i].p, a.layer[i].plan);
    if (b > lds_bytes) lds_bytes = b;
  }
  if (lds_bytes > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)a.first_wg[a.n]), dim3(MW * 64), lds_bytes, s, a, x, ldx);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int RES_BITS, int NTP, bool WALK>
int launch_one(const Params &p, DownMfmaPlan &plan, unsigned grid, const __half *x, long long ldx, __half *y, long long ldy,
               hipStream_t s) {
  auto kernel = gemv_down_mfma_kernel<RES_BITS, NTP, WALK>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned lds_bytes = place_lds<RES_BITS, NTP>(p, plan);
  if (lds_bytes > 160u * 1024u) return VQ_ERR_UNSUPPORTED;                  // too many outlier columns to hold beside the tables
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(MW * 64), lds_bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Whether the kernel above takes this layer and these buffers (the caller has checked gemv_down_applicable()).
bool gemv_down_mfma_applicable(const Params &p, const __half *x, long long ldx, int batch) {
  if (p.orientation != 1 || p.v != 6 || p.bits != 12 || p.Q > 512) return false;
  if (p.Q && (long long)p.S_out * p.stride_out >= (1LL << 31)) return false;
  if (p.n_groups > 1 && ((p.Pg & 7) || p.n_groups > 256)) return false;     // a group starts on a dword of the index streams
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return false;
  if (batch < 1 || batch > 16) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 3) || (ldx & 1) || (p.n_out & 1)) return false;      // activation loads are dword-aligned
  if (((long long)(batch - 1) * ldx + p.in_features) * 2 >= (1LL << 31)) return false;       // 32-bit buffer offsets
  const long long max_stride = p.stride > p.stride_res ? p.stride : p.stride_res;
  return (long long)p.S * max_stride < (1LL << 31);
}

// Parts the columns are cut into when a workspace is there: enough for the (block, part) workgroups to fill the chip, each
// part at least one 32-column window per wave.  1: nothing to gain from a workspace.
// Codebook groups are parts by themselves (a part has one set of tables); each is cut further on the same terms.
static int parts_per_group(const Params &p) {
  const int blocks = (p.S + 15) / 16, windows = (min(p.P, p.Pg) + 31) / 32;
  int want = cu_count() / ((blocks > 0 ? blocks : 1) * p.n_groups);
  if (want > windows / MW) want = windows / MW;
  if (want > 16) want = 16;
  if (want < 2) return 1;
  const int wpp = (windows + want - 1) / want;
  return (windows + wpp - 1) / wpp;
}
int gemv_down_mfma_parts(const Params &p) { return p.n_groups * parts_per_group(p); }

static int make_plan(const Params &p, long long ldx, int batch, float *part, float *part_xs, int parts, DownMfmaPlan &plan, long long *grid_out) {
  const int blocks = (p.S + 15) / 16, windows = (min(p.P, p.Pg) + 31) / 32;                // windows of the widest group
  if (blocks < 1 || windows < 1) return VQ_ERR_UNSUPPORTED;
  plan.ksplit = part ? parts : 1;
  if (part && plan.ksplit % p.n_groups) return VQ_ERR_UNSUPPORTED;
  plan.sub = part ? plan.ksplit / p.n_groups : 1;      // without a workspace: one workgroup per block walks all groups and all windows
  plan.wpp = (windows + plan.sub - 1) / plan.sub;
  plan.batch = batch;
  // (a whole number of dwords: the buffer's range check drops a dword that straddles the end, and with it the last
  // column of the last row when in_features is odd; ldx is a multiple of 8 here, so the half after it is the caller's
  // padding, and the kernel masks it like every position past the stream's end)
  plan.x_bytes = (unsigned)((((long long)(batch - 1) * ldx + p.in_features) * 2 + 3) & ~3LL);
  plan.part = part; plan.part_xs = part_xs;
  plan.o_pitch = ((p.Q + 1) / 2) | 1;
  plan.o_rpw = (int)((p.out_features + (long long)blocks * plan.ksplit - 1) / ((long long)blocks * plan.ksplit));   // <= 96: a block has 96 rows
  const long long grid = (long long)blocks * plan.ksplit;
  if (grid > 0x7FFFFFFFLL) return VQ_ERR_UNSUPPORTED;
  *grid_out = grid;
  return VQ_OK;
}

// part == nullptr: one launch that stores y (a layer with codebook groups: every workgroup walks all of them).  Else
// parts = gemv_down_mfma_parts(p) > 1 and the sums go to part[parts][batch][out_features], part_xs[parts * 16]; the caller
// adds them up.
int launch_gemv_down_mfma(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s,
                          float *part, float *part_xs, int parts) {
  DownMfmaPlan plan{};
  long long grid = 0;
  const int rc_plan = make_plan(p, ldx, batch, part, part_xs, parts, plan, &grid);
  if (rc_plan != VQ_OK) return rc_plan;
  const int rb = p.k_res ? p.bits_res : 0;
  const int ntp = (6 * batch + 15) / 16;                // instructions whose 16 operand columns hold the 6 x batch (token, row) pairs
  const bool walk = !part && p.n_groups > 1;
#define VQ_CASE(R, N, LO) if (rb == R && ntp > LO && ntp <= N) \
    return walk ? launch_one<R, N, true>(p, plan, (unsigned)grid, x, ldx, y, ldy, s) : launch_one<R, N, false>(p, plan, (unsigned)grid, x, ldx, y, ldy, s);
  VQ_CASE(0, 1, 0) VQ_CASE(0, 2, 1) VQ_CASE(0, 3, 2) VQ_CASE(0, 4, 3) VQ_CASE(0, 6, 4)
  VQ_CASE(8, 1, 0) VQ_CASE(8, 2, 1) VQ_CASE(8, 3, 2) VQ_CASE(8, 4, 3) VQ_CASE(8, 6, 4)
  VQ_CASE(12, 1, 0) VQ_CASE(12, 2, 1) VQ_CASE(12, 3, 2) VQ_CASE(12, 4, 3) VQ_CASE(12, 6, 4)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

// n layers (2 .. 8) of one codebook group each on the same activations in one launch, without a workspace.  VQ_ERR_UNSUPPORTED
// when they do not fit one kernel instantiation (different residual kinds, different in_features); the caller then launches
// them one by one.  The caller has checked gemv_down_mfma_applicable() for each.
int launch_gemv_down_mfma_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys,
                                const long long *ldys, hipStream_t s) {
  if (n < 2 || n > DMULTI_MAX) return VQ_ERR_UNSUPPORTED;
  DownMultiArgs a{};
  a.n = n;
  const int rb = ps[0].k_res ? ps[0].bits_res : 0;
  long long total = 0;
  for (int i = 0; i < n; ++i) {
    if (ps[i].in_features != ps[0].in_features || ps[i].n_groups > 1 || (ps[i].k_res ? ps[i].bits_res : 0) != rb) return VQ_ERR_UNSUPPORTED;
    long long grid = 0;
    const int rc = make_plan(ps[i], ldx, batch, nullptr, nullptr, 1, a.layer[i].plan, &grid);
    if (rc != VQ_OK) return rc;
    a.layer[i].p = ps[i]; a.layer[i].y = ys[i]; a.layer[i].ldy = ldys[i];
    a.first_wg[i] = (int)total;
    total += grid;
    if (total > 0x7FFFFFFFLL) return VQ_ERR_UNSUPPORTED;
  }
  a.first_wg[n] = (int)total;
  const int ntp = (6 * batch + 15) / 16;
#define VQ_CASE(R, N, LO) if (rb == R && ntp > LO && ntp <= N) return launch_multi<R, N>(a, x, ldx, s);
  VQ_CASE(0, 1, 0) VQ_CASE(0, 2, 1) VQ_CASE(0, 3, 2) VQ_CASE(0, 4, 3) VQ_CASE(0, 6, 4)
  VQ_CASE(8, 1, 0) VQ_CASE(8, 2, 1) VQ_CASE(8, 3, 2) VQ_CASE(8, 4, 3) VQ_CASE(8, 6, 4)
  VQ_CASE(12, 1, 0) VQ_CASE(12, 2, 1) VQ_CASE(12, 3, 2) VQ_CASE(12, 4, 3) VQ_CASE(12, 6, 4)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
