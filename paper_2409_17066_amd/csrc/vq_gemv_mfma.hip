// vq_gemv on the matrix cores, for the same layers as the dot-product kernel (v = 6, 12-bit indices,
// optional 12- or 8-bit residual codebook, optional v = 4 outlier columns; App. "Parameter Description")
// and any batch 1..16: the decode-side product of Sec. 2.2's lookup with a handful of activation rows.
//
// One v_mfma_f32_16x16x32_f16 multiplies 16 output rows by 16 tokens over 32 "k" slots.  The k order is
// free as long as both operands agree, so a slot group of 8 halves is one codebook vector: 6 (or 4)
// values plus zero padding.  Lane l of a wave supplies, as operand A, the 16-byte LDS entry of row
// (l & 15) for vector group (l >> 4) -- exactly what one ds_read_b128 gather returns -- and, as operand
// B, the matching 6 activations of token (l & 15).  A gathered centroid therefore feeds one instruction
// instead of 3 * batch dot-product operations, and the sum over a wave's lanes happens inside the MFMA:
// the kernel runs at the LDS gather rate for every batch up to 16.
//
// Work split: a workgroup owns a block of rows (a multiple of 16) and walks them in chunks of up to four
// 16-row blocks; within a chunk it makes passes over the columns: in pass p wave w covers vectors
// [(p * MW + w) * 32, +32), eight per lane, whose 96 index bits are exactly three aligned dwords.  The
// activations of a pass sit in registers (B operands) and are reused by every block of the chunk; index
// words and the next pass's activations are loaded one pass ahead.  Each wave ends a chunk with a
// 16 x 16 partial per block; partials meet in LDS, one wave per block adds them up and applies
// y = scale * sum(d x) + bias * sum(x).  sum(x) comes from one more MFMA per pass against all-ones rows.
//
// Codebook groups (Sec. 3.1: every range of columns has tables of its own): the workgroup walks its rows once per
// group, with that group's tables in LDS and only that group's columns; the per-block sums stay in LDS, in
// binary32, from one group to the next, and the last group applies scale and bias and stores.
#include "vq_common.hpp"
#include "vq_v6.hpp"
#include <cstdlib>

namespace vq {
namespace {

using namespace v6;

constexpr int NBMAX = 4;         // 16-row blocks per chunk
constexpr int VPL = 8;           // vectors per lane per pass: 8 x 12 bits = 3 dwords, 8 x 8 bits = 2 dwords

struct MfmaPlan {
  int rows_per_wg;               // multiple of 16
  int nb;                        // blocks per chunk, 1 .. NBMAX
  int part_bufs;                 // 1: barrier after the reduction as well; 2: chunks alternate buffers
  unsigned lds_out, lds_part, lds_xs;
  unsigned x_bytes;              // bytes from x[0][0] to the end of the last batch row
  int y_wide;                    // y rows allow 8-byte stores
  unsigned lds_sb;               // scale | bias << 16 of the workgroup's rows
  unsigned lds_yacc;             // grouped layers: binary32 sums of the groups so far, 1 KB per 16-row block
  int out_global;                // 1: the outlier table stays in global memory (no room beside two 64 KB tables) and is gathered from there
};

// Which codebook groups a workgroup walks, and where their sums go: the finished fp16 outputs (part == nullptr), or --
// when every workgroup takes one group and the groups meet in a second kernel -- binary32 sums without scale and bias,
// part[token][row] for this range, plus the activation sums of the range's columns, part_xs[group * 16 + token].
struct GroupRange {
  int begin, end;
  float *part, *part_xs;
};

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4v mfma16(uint4v a, uint4v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8v, a), __builtin_bit_cast(half8v, b), c, 0, 0, 0);
}

// Vector-ALU work is what this kernel has least of: a wave-wide VALU instruction occupies its SIMD for four
// cycles, a wave-wide 16-byte LDS gather occupies the LDS for about twelve, so more than ~12 VALU
// instructions per gather (summed over the four SIMDs) and the LDS starves.  Hence: two instructions per
// LDS address, activations loaded straight into MFMA operand registers, load addresses advanced by
// additions, end-of-row masking only in the one column group that needs it.
// `wg` is the workgroup's number within its layer (a launch may hold the workgroups of several layers).
template <int RES_BITS, int MW, int NB, bool GROUPED>
__device__ __forceinline__ void gemv_v6_mfma_body(const Params &p, const MfmaPlan &plan, const __half *__restrict__ x, long long ldx,
                                                  int batch, __half *__restrict__ y, long long ldy, int wg,
                                                  const GroupRange gr = GroupRange{0, 1, nullptr, nullptr}) {
  typedef Layout<RES_BITS> LY;
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  constexpr int PA = NB == 2 ? 4 : 2;                   // passes whose index words are in flight or in registers
  constexpr int XD = 1, XS = XD + 1;                    // activations run XD passes ahead, in XS register sets
  static_assert(PA % XS == 0, "the unrolled pass loop must map passes to activation sets statically");
  constexpr int R = PA * NB;                            // ring of index-word slots: slot (j, b) = j * NB + b
  constexpr int S = RES_BITS ? 2 : 1;                   // loads per slot
  // loads issued after a slot's own by the time the slot is used, while the ring is being refilled: the other
  // R - 1 slots and PA groups of eight activation loads; after a pass's activation loads: XD passes of refills
  // and the activation loads of the passes in between
  constexpr int AFTER_SLOT = (R - 1) * S + 8 * PA, AFTER_X = XD * NB * S + (XD - 1) * 8;
  static_assert(AFTER_SLOT < 64, "vmcnt holds 6 bits");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;       // A: row n of the block, vector group g.  B: token n.  D: token n, rows 4g..4g+3
  const int row0 = wg * plan.rows_per_wg;
  const int rows_here = min(p.out_features - row0, plan.rows_per_wg);
  const int n_blocks = (rows_here + 15) >> 4;
  const int n_chunks = (n_blocks + NB - 1) / NB;
  const unsigned a_out = lds_address(lds) + plan.lds_out;

  const unsigned st_main = (unsigned)p.stride, st_res = (unsigned)p.stride_res, st_out = (unsigned)p.stride_out;
  const uint4v r_main = scalar_rsrc(p.idx + (long long)row0 * p.stride, (unsigned)rows_here * st_main);
  const uint4v r_res = scalar_rsrc(RES_BITS ? p.idx_res + (long long)row0 * p.stride_res : p.idx,
                                   RES_BITS ? (unsigned)rows_here * st_res : 0u);
  const uint4v r_xa = scalar_rsrc(x, plan.x_bytes);
  const __amdgpu_buffer_rsrc_t r_out = make_rsrc(p.Q ? p.idx_out + (long long)row0 * p.stride_out : p.idx,
                                                 p.Q ? (unsigned)rows_here * st_out : 0u);
  const __amdgpu_buffer_rsrc_t r_x = make_rsrc(x, plan.x_bytes);
  const __amdgpu_buffer_rsrc_t r_scale = make_rsrc(p.scale ? p.scale : p.cb, p.scale ? (unsigned)p.out_features * 2u : 0u);
  const __amdgpu_buffer_rsrc_t r_bias = make_rsrc(p.bias ? p.bias : p.cb, p.bias ? (unsigned)p.out_features * 2u : 0u);
  // Lanes of tokens past the batch read out of range, i.e. nothing -- except token 15, which loads the start of the
  // first row so that every activation load keeps a lane in range (rule 2 above; with 16 tokens the rows before the
  // last one do that).  What it feeds into the MFMA only reaches an output column that is never stored.
  const bool token_on = n < batch;
  const unsigned xrow = token_on ? (unsigned)((long long)n * ldx * 2) : n == 15 ? 0u : 0x80000000u;

  uint3v win[R], wres[RES_BITS == 12 ? R : 1];   // index words, PA passes deep
  uint2v wres8[RES_BITS == 8 ? R : 1];
  uint4v bxs[XS][VPL];                           // B operands (activations) of the current and of the next XD passes
#pragma unroll
  for (int i = 0; i < R; ++i) {
    win[i] = uint3v{0u, 0u, 0u};
    if (RES_BITS == 12) wres[i] = uint3v{0u, 0u, 0u};
    if (RES_BITS == 8) wres8[i] = uint2v{0u, 0u};
  }
#pragma unroll
  for (int i = 0; i < XS; ++i)
#pragma unroll
    for (int u = 0; u < VPL; ++u) bxs[i][u] = uint4v{0u, 0u, 0u, 0u};

  const uint4v ones = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0u};
  float4v acc[NB];
  // sum of each token's activations over this wave's columns, kept in LDS (slot [wave][token], touched by this wave only
  // until the first chunk's barrier): a register accumulator would stay allocated through the whole kernel
  float *xs_part = reinterpret_cast<float *>(lds + plan.lds_xs);       // [MW][16]
  if (g == 0) xs_part[wv * 16 + n] = 0.0f;
  int buf = 0;

  const int grp_end = GROUPED ? gr.end : 1;
  const bool partial = GROUPED && gr.part != nullptr;
  for (int grp = GROUPED ? gr.begin : 0; grp < grp_end; ++grp) {
  // ---- this codebook group's vectors [v_lo, v_lo + v_n) and columns [col_lo, col_hi) of every row
  const int v_lo = GROUPED ? grp * p.Pg : 0;                                  // a multiple of 8: a dword boundary in the streams
  const int v_n = GROUPED ? min(p.Pg, p.P - v_lo) : p.P;
  const int col_lo = p.n_out + v_lo * 6;
  const int col_hi = GROUPED ? min(p.in_features, col_lo + v_n * 6) : p.in_features;
  const unsigned gb_main = (unsigned)(v_lo >> 3) * 12u, gb_res = (unsigned)(v_lo >> 3) * (RES_BITS == 8 ? 8u : 12u);
  // passes in which this wave has vectors: a prefix 0 .. my_passes-1 (pass p: group p * MW + wv of 32 vectors)
  const int wave_groups = (v_n + 31) >> 5;
  const int my_passes = wave_groups > wv ? (wave_groups - wv + MW - 1) / MW : 0;
  const int eff_passes = max(my_passes, 1);                                   // a wave without vectors still walks the chunks
  // ... and still fills its prefetch ring at the start, so that the start is one straight line of loads for every wave
  // (a refill inside a branch costs a second set of registers); it loads what wave 0 loads, which is in range, and
  // never looks at it
  const int wl = my_passes > 0 ? wv : 0;
  const int out_groups = grp == 0 ? (p.Q + 31) >> 5 : 0;                      // outlier columns go with the first group
  const int my_out_passes = out_groups > wv ? (out_groups - wv + MW - 1) / MW : 0;
  // a group whose 192 columns (plus the two halves the last 16-byte load overshoots) end before col_hi needs no masking
  const int clean_groups = (col_hi - col_lo - 2) / 192;                       // groups 0 .. clean_groups-1 are clean
  const int last_clean_pass = clean_groups - 1 - wv >= 0 ? (clean_groups - 1 - wv) / MW : -1;

  // The wave's passes form one sequence over all chunks; the loader runs PA passes ahead of the consumer.
  // Loader addresses: byte offset of the loader's pass inside a row, and of each block's row `n` in the streams.
  int lp = 0, lc = 0;
  unsigned l_main = gb_main + (unsigned)(wl * 4 + g) * 12u, l_res = gb_res + (unsigned)(wl * 4 + g) * (RES_BITS == 8 ? 8u : 12u);
  unsigned lrow_main[NB], lrow_res[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) { lrow_main[b] = (unsigned)(b * 16 + n) * st_main; lrow_res[b] = (unsigned)(b * 16 + n) * st_res; }
  auto advance_loader = [&]() {
    if (++lp == eff_passes) {
      lp = 0;
      l_main = gb_main + (unsigned)(wl * 4 + g) * 12u; l_res = gb_res + (unsigned)(wl * 4 + g) * (RES_BITS == 8 ? 8u : 12u);
      // past the last chunk the loader starts over: what it loads then is never used, but stays an ordinary load
      const bool wrap = ++lc == n_chunks;
      if (wrap) lc = 0;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        lrow_main[b] = wrap ? (unsigned)(b * 16 + n) * st_main : lrow_main[b] + (unsigned)(NB * 16) * st_main;
        lrow_res[b] = wrap ? (unsigned)(b * 16 + n) * st_res : lrow_res[b] + (unsigned)(NB * 16) * st_res;
      }
    } else {
      l_main += (MW * 4) * 12u; l_res += (MW * 4) * (RES_BITS == 8 ? 8u : 12u);
    }
  };
  auto load_slot = [&](int slot, int b) {       // rows past the end of a ragged block read zeros
    // a block past the last one (the last chunk may be short) is replaced by the workgroup's first block
    const bool real = lc * NB + b < n_blocks;
    const unsigned o_main = (real ? lrow_main[b] : (unsigned)n * st_main) + l_main;
    const unsigned o_res = (real ? lrow_res[b] : (unsigned)n * st_res) + l_res;
    async_load_b96(win[slot], r_main, o_main);
    if (RES_BITS == 12) async_load_b96(wres[slot], r_res, o_res);
    if (RES_BITS == 8) async_load_b64(wres8[slot], r_res, o_res);
  };
  // activations of one pass: eight overlapping 16-byte loads, one per vector; the fourth dword belongs to the
  // next vector and meets the zero padding of the codebook entries
  auto issue_x = [&](uint4v (&bx)[VPL], int pass) {
    const unsigned off = token_on ? xrow + ((unsigned)col_lo + (unsigned)((pass * MW + wl) * 4 + g) * (VPL * 6u)) * 2u : xrow;
    async_load_b128_at<0>(bx[0], r_xa, off);  async_load_b128_at<12>(bx[1], r_xa, off);
    async_load_b128_at<24>(bx[2], r_xa, off); async_load_b128_at<36>(bx[3], r_xa, off);
    async_load_b128_at<48>(bx[4], r_xa, off); async_load_b128_at<60>(bx[5], r_xa, off);
    async_load_b128_at<72>(bx[6], r_xa, off); async_load_b128_at<84>(bx[7], r_xa, off);
  };

  {
    TableStage<RES_BITS, MW * 64> tables{};
    // (with groups: the thread id is made opaque in every round, or the table addresses derived from it would be kept
    // in registers through the main loop for the next group)
    unsigned tid = threadIdx.x;
    if (GROUPED) asm volatile("" : "+v"(tid));
    tables.issue(p, grp, grp == 0 && !plan.out_global, tid);
#pragma unroll
    for (int j = 0; j < PA; ++j) {
#pragma unroll
      for (int b = 0; b < NB; ++b) load_slot(j * NB + b, b);
      advance_loader();
    }
#pragma unroll
    for (int d = 0; d < XD; ++d) issue_x(bxs[d], d % eff_passes);
    wait_vmem_at_most<R * S + 8 * XD>();         // the tables are in; the index words may still be on their way
    tables.store(p, lds, plan.lds_out, grp == 0 && !plan.out_global, tid);
  }
  // scale and bias of the workgroup's rows, one dword per row, for the reductions at the chunk ends
  for (int r = (int)threadIdx.x; r < (grp == (GROUPED ? gr.begin : 0) && !partial ? plan.rows_per_wg : 0); r += MW * 64) {
    const unsigned short sc = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_scale, (unsigned)(row0 + r) * 2u, 0, 0);
    const unsigned short bi = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r_bias, (unsigned)(row0 + r) * 2u, 0, 0);
    *reinterpret_cast<unsigned *>(lds + plan.lds_sb + (unsigned)r * 4u) = (unsigned)sc | ((unsigned)bi << 16);
  }
  lds_barrier();
  // The counted waits assume the steady pattern of loads that only the loop below issues: everything issued so
  // far has to be in first.
  wait_vmem_at_most<0>();

  int c = 0, pass = 0;
  while (c < n_chunks) {
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      if (c < n_chunks) {
        const int nb_c = min(NB, n_blocks - c * NB);
        const int ep_o = row0 + (c * NB + wv) * 16 + 4 * g;      // wave b finishes block b of the chunk
        if (pass == 0) {
          // ---- chunk start
#pragma unroll
          for (int b = 0; b < NB; ++b) acc[b] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
          // outlier columns (v = 4): same scheme with 8-byte table entries; their loads are not run ahead
          for (int q = 0; q < my_out_passes; ++q) {
            const unsigned lane_group = (unsigned)((q * MW + wv) * 4 + g);
            uint3v wo[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b)
              wo[b] = __builtin_amdgcn_raw_buffer_load_b96(r_out, (unsigned)((c * NB + b) * 16 + n) * st_out + lane_group * 12u, 0, 0);
            const unsigned col = lane_group * (VPL * 4u);
            uint4v xo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) xo[i] = __builtin_amdgcn_raw_buffer_load_b128(r_x, xrow + (col + i * 8u) * 2u, 0, 0);
            const unsigned xd[16] = {xo[0].x, xo[0].y, xo[0].z, xo[0].w, xo[1].x, xo[1].y, xo[1].z, xo[1].w,
                                     xo[2].x, xo[2].y, xo[2].z, xo[2].w, xo[3].x, xo[3].y, xo[3].z, xo[3].w};
            uint4v bx[VPL];
#pragma unroll
            for (int u = 0; u < VPL; ++u) {
              bx[u].x = (int)(col + 4 * u) < p.n_out ? xd[2 * u] : 0u;         // n_out is a multiple of 4
              bx[u].y = (int)(col + 4 * u) < p.n_out ? xd[2 * u + 1] : 0u;
              bx[u].z = 0u; bx[u].w = 0u;
            }
            if (c == 0) {
              float4v xs = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
              for (int u = 0; u < VPL; ++u) xs = mfma16(ones, bx[u], xs);
              if (g == 0) xs_part[wv * 16 + n] += xs.x;
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
              if (b < nb_c) {
                Window<3> cw; cw.w[0] = wo[b].x; cw.w[1] = wo[b].y; cw.w[2] = wo[b].z;
                uint2v e[VPL];
#pragma unroll
                for (int u = 0; u < VPL; ++u) {
                  if (plan.out_global) {       // (an index past a short table is clamped into it)
                    const unsigned off = min(field_addr<12, 3>(cw, u), (unsigned)(p.k_out - 1) * 8u);
                    e[u] = *reinterpret_cast<const uint2v *>(reinterpret_cast<const unsigned char *>(p.cb_out) + off);
                  } else {
                    lds_gather8(e[u], field_addr<12, 3>(cw, u) + a_out);
                  }
                }
                lds_gather_wait();
#pragma unroll
                for (int u = 0; u < VPL; ++u) settle(e[u]);
#pragma unroll
                for (int u = 0; u < VPL; ++u) {
                  uint4v a; a.x = e[u].x; a.y = e[u].y; a.z = 0u; a.w = 0u;
                  acc[b] = mfma16(a, bx[u], acc[b]);
                }
              }
          }
        }

        if (my_passes > 0) {
          // ---- one pass over this wave's 32 vectors of every block of the chunk
          // Every pass issues the same number of loads, also past the end of the sequence (the loader then starts
          // over), so the counted waits hold throughout.
          uint4v (&bx)[VPL] = bxs[j % XS];
          wait_vmem_at_most<AFTER_X>();
#pragma unroll
          for (int u = 0; u < VPL; ++u) settle(bx[u]);
          if (pass > last_clean_pass) {          // the group that holds the end of the row: zero what lies past it
            const int col = col_lo + ((pass * MW + wv) * 4 + g) * (VPL * 6);
#pragma unroll
            for (int u = 0; u < VPL; ++u) {
              bx[u].x = col + 6 * u < col_hi ? bx[u].x : 0u;                  // col_lo and col_hi are even
              bx[u].y = col + 6 * u + 2 < col_hi ? bx[u].y : 0u;
              bx[u].z = col + 6 * u + 4 < col_hi ? bx[u].z : 0u;
              bx[u].w = 0u;
            }
          }
          if (c == 0) {
            float4v xs = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int u = 0; u < VPL; ++u) xs = mfma16(ones, bx[u], xs);
            if (g == 0) xs_part[wv * 16 + n] += xs.x;
          }
          issue_x(bxs[(j + XD) % XS], (pass + XD) % my_passes);
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const int slot = j * NB + b;
            wait_vmem_at_most<AFTER_SLOT>();
            settle(win[slot]);
            if (RES_BITS == 12) settle(wres[slot]);
            if (RES_BITS == 8) settle(wres8[slot]);
            Window<3> cm, cr;
            cm.w[0] = win[slot].x; cm.w[1] = win[slot].y; cm.w[2] = win[slot].z;
            if (RES_BITS == 12) { cr.w[0] = wres[slot].x; cr.w[1] = wres[slot].y; cr.w[2] = wres[slot].z; }
            if (RES_BITS == 8) { cr.w[0] = wres8[slot].x; cr.w[1] = wres8[slot].y; cr.w[2] = 0u; }
            // LDS addresses and the main gathers come before the slot is overwritten by its refill
            unsigned ar[VPL];
            uint4v e[VPL];
#pragma unroll
            for (int u = 0; u < VPL; ++u) {
              if (RES_BITS) { ar[u] = field_addr<RB, LY::RES_SH>(cr, u) + LY::RES_ADD; settle(ar[u]); }
              lds_gather16<LY::MAIN_OFF>(e[u], field_addr<12, LY::MAIN_SH>(cm, u));
            }
            load_slot(slot, b);                                  // refill with the pass PA ahead
            // (waited for on every path, also where a ragged last chunk has no use for the block: no register may be
            // handed back to the compiler with a load into it still on its way)
            lds_gather_wait();
#pragma unroll
            for (int u = 0; u < VPL; ++u) settle(e[u]);
            if (b < nb_c) {
#pragma unroll
              for (int u = 0; u < VPL; ++u) acc[b] = mfma16(e[u], bx[u], acc[b]);
              if (RES_BITS) {
                uint4v f[VPL];
#pragma unroll
                for (int u = 0; u < VPL; ++u) lds_gather16<LY::RES_OFF>(f[u], ar[u]);
                lds_gather_wait();
#pragma unroll
                for (int u = 0; u < VPL; ++u) settle(f[u]);
#pragma unroll
                for (int u = 0; u < VPL; ++u) acc[b] = mfma16(f[u], bx[u], acc[b]);
              }
            }
          }
        }
        advance_loader();

        if (pass == eff_passes - 1) {
          // ---- chunk end: partial sums to LDS; wave b adds up block b, applies scale and bias, stores
          unsigned char *pbase = lds + plan.lds_part + (unsigned)(buf * NB) * (MW * 1024u);
#pragma unroll
          for (int b = 0; b < NB; ++b)
            if (b < nb_c) *reinterpret_cast<float4v *>(pbase + (unsigned)(b * MW + wv) * 1024u + lane * 16u) = acc[b];
          lds_barrier();
          if (wv < nb_c) {
            float4v s = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int w = 0; w < MW; ++w) s += *reinterpret_cast<const float4v *>(pbase + (unsigned)(wv * MW + w) * 1024u + lane * 16u);
            // sums of the groups so far: this lane of this wave is the only one that ever touches its slot
            float4v *ya = reinterpret_cast<float4v *>(lds + plan.lds_yacc + (unsigned)((c * NB + wv) * 64 + lane) * 16u);
            if (GROUPED && grp > gr.begin) s += *ya;
            float xsum = 0.0f;
#pragma unroll
            for (int w = 0; w < MW; ++w) xsum += xs_part[w * 16 + n];
            const float sv[4] = {s.x, s.y, s.z, s.w};
            if (GROUPED && grp + 1 < grp_end) {
              *ya = s;
            } else if (partial) {
              if (n < batch) {
                float *dst = gr.part + (long long)n * p.out_features + ep_o;
                if (ep_o + 3 < p.out_features && (p.out_features & 3) == 0) {
                  *reinterpret_cast<float4v *>(dst) = s;
                } else {
#pragma unroll
                  for (int r = 0; r < 4; ++r)
                    if (ep_o + r < p.out_features) dst[r] = sv[r];
                }
                if (wg == 0 && c == 0 && wv == 0 && g == 0) gr.part_xs[grp * 16 + n] = xsum;
              }
            } else {
            const uint4v sb = *reinterpret_cast<const uint4v *>(lds + plan.lds_sb + (unsigned)((c * NB + wv) * 16 + 4 * g) * 4u);
            const unsigned sbw[4] = {sb.x, sb.y, sb.z, sb.w};             // per row: scale | bias << 16, as staged at the start
            __half out[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float sc = p.scale ? (float)__builtin_bit_cast(_Float16, (unsigned short)sbw[r]) : 1.0f;
              const float bi = p.bias ? (float)__builtin_bit_cast(_Float16, (unsigned short)(sbw[r] >> 16)) : 0.0f;
              out[r] = __float2half_rn(__fmaf_rn(sc, sv[r], bi * xsum));
            }
            if (n < batch) {
              __half *dst = y + (long long)n * ldy + ep_o;
              if (plan.y_wide && ep_o + 3 < p.out_features) {
                uint2v pk;
                pk.x = (unsigned)__half_as_ushort(out[0]) | ((unsigned)__half_as_ushort(out[1]) << 16);
                pk.y = (unsigned)__half_as_ushort(out[2]) | ((unsigned)__half_as_ushort(out[3]) << 16);
                *reinterpret_cast<uint2v *>(dst) = pk;
              } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                  if (ep_o + r < p.out_features) dst[r] = out[r];
              }
            }
            }
          }
          if (plan.part_bufs == 1) lds_barrier(); else buf ^= 1;
          pass = 0; ++c;
        } else {
          ++pass;
        }
      }
    }
  }
  // Loads of the loader's run past the last chunk are still on their way; they must be in before the next group
  // refills the same registers from its own start.
  if (GROUPED) wait_vmem_at_most<0>();
  }
}

template <int RES_BITS, int MW, int NB, bool GROUPED>
__global__ __launch_bounds__(MW * 64) void gemv_v6_mfma_kernel(Params p, MfmaPlan plan, const __half *__restrict__ x, long long ldx,
                                                                int batch, __half *__restrict__ y, long long ldy) {
  warm_kernel_arguments();
  gemv_v6_mfma_body<RES_BITS, MW, NB, GROUPED>(p, plan, x, ldx, batch, y, ldy, (int)blockIdx.x, GroupRange{0, p.n_groups, nullptr, nullptr});
}

// A layer with codebook groups when the caller lends a workspace: every workgroup takes one group (its tables go into
// LDS once) and a share of the rows, the binary32 sums go to the workspace [group][token][row], and the kernel below
// adds the groups up.  Without a workspace the workgroups cannot meet, and each walks all groups (the kernel above).
// (Two waves per SIMD in every instantiation: eight waves in one workgroup, or two workgroups of four.)
template <int RES_BITS, int MW, int NB>
__global__ __launch_bounds__(MW * 64) __attribute__((amdgpu_waves_per_eu(2))) void gemv_v6_mfma_groups_kernel(Params p, MfmaPlan plan, const __half *__restrict__ x, long long ldx,
                                                                       int batch, float *__restrict__ part, float *__restrict__ part_xs,
                                                                       int wgs_per_group) {
  warm_kernel_arguments();
  const int grp = (int)blockIdx.x / wgs_per_group, wg = (int)blockIdx.x - grp * wgs_per_group;
  gemv_v6_mfma_body<RES_BITS, MW, NB, true>(p, plan, x, ldx, batch, nullptr, 0, wg,
                                            GroupRange{grp, grp + 1, part + (long long)grp * batch * p.out_features, part_xs});
}

// y[t][o] = fp16(scale[o] * sum_g part[g][t][o] + bias[o] * sum_g part_xs[g][t]), groups in ascending order.
// The sums were written by other compute units a moment ago and come from beyond this one's caches: the loads of
// FINISH_AHEAD groups are issued together (a group past the last repeats the last and is not added), the additions
// keep their order.
constexpr int FINISH_THREADS = 128;
template <int FINISH_AHEAD>
__global__ __launch_bounds__(FINISH_THREADS) void gemv_groups_finish_kernel(const float *__restrict__ part, const float *__restrict__ part_xs,
                                                                            int n_groups, int batch, int out_features,
                                                                            const __half *__restrict__ scale, const __half *__restrict__ bias,
                                                                            __half *__restrict__ y, long long ldy) {
  const int o = blockIdx.x * FINISH_THREADS + threadIdx.x, t = blockIdx.y;          // one token per grid row
  if (o >= out_features) return;
  const float sc = scale ? __half2float(scale[o]) : 1.0f, bi = bias ? __half2float(bias[o]) : 0.0f;
  float sum = 0.0f, xs = 0.0f;
  for (int g0 = 0; g0 < n_groups; g0 += FINISH_AHEAD) {
    float v[FINISH_AHEAD], w[FINISH_AHEAD];
#pragma unroll
    for (int i = 0; i < FINISH_AHEAD; ++i) {
      const int gi = min(g0 + i, n_groups - 1);
      v[i] = part[((long long)gi * batch + t) * out_features + o];
      w[i] = part_xs[gi * 16 + t];
    }
#pragma unroll
    for (int i = 0; i < FINISH_AHEAD; ++i)
      if (g0 + i < n_groups) { sum += v[i]; xs += w[i]; }
  }
  y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(sc, sum, bi * xs));
}

void launch_finish(const float *part, const float *part_xs, int n_groups, int batch, const Params &p, __half *y, long long ldy, hipStream_t s) {
  const dim3 grid((unsigned)((p.out_features + FINISH_THREADS - 1) / FINISH_THREADS), (unsigned)batch), block(FINISH_THREADS);
  if (n_groups <= 2)
    hipLaunchKernelGGL(gemv_groups_finish_kernel<2>, grid, block, 0, s, part, part_xs, n_groups, batch, p.out_features, p.scale, p.bias, y, ldy);
  else if (n_groups <= 4)
    hipLaunchKernelGGL(gemv_groups_finish_kernel<4>, grid, block, 0, s, part, part_xs, n_groups, batch, p.out_features, p.scale, p.bias, y, ldy);
  else
    hipLaunchKernelGGL(gemv_groups_finish_kernel<8>, grid, block, 0, s, part, part_xs, n_groups, batch, p.out_features, p.scale, p.bias, y, ldy);
}

// Several layers that read the same activations (the query, key and value projections of a decoder layer; its gate
// and up projections) in one launch.  The launch and start-up cost of a decode-sized product (App. "Our
// Dequantization Implementation", second phase) is as large as its streaming time or larger, and one launch pays
// it once.  Every workgroup belongs to one layer and runs the single-layer kernel body on it.
constexpr int MULTI_MAX = 8;
struct MultiLayer {
  Params p;
  MfmaPlan plan;
  __half *y;
  long long ldy;
};
struct MultiArgs {
  int n;
  int first_wg[MULTI_MAX + 1];             // layer i owns workgroups [first_wg[i], first_wg[i + 1])
  MultiLayer layer[MULTI_MAX];
};

template <int RES_BITS, int MW, int NB>
__global__ __launch_bounds__(MW * 64) void gemv_v6_mfma_multi_kernel(MultiArgs a, const __half *__restrict__ x, long long ldx, int batch) {
  warm_kernel_arguments();
  int i = 0;
  while (i + 1 < a.n && (int)blockIdx.x >= a.first_wg[i + 1]) ++i;
  const MultiLayer &l = a.layer[i];
  gemv_v6_mfma_body<RES_BITS, MW, NB, false>(l.p, l.plan, x, ldx, batch, l.y, l.ldy, (int)blockIdx.x - a.first_wg[i]);
}


template <int RES_BITS, int MW, int NB, bool GROUPED>
int launch_one(const Params &p, const MfmaPlan &plan, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx, int batch,
               __half *y, long long ldy, hipStream_t s) {
  auto kernel = gemv_v6_mfma_kernel<RES_BITS, MW, NB, GROUPED>;
  VQ_ALLOW_FULL_LDS(kernel);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(MW * 64), lds_bytes, s, p, plan, x, ldx, batch, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

#ifndef VQ_MFMA_WAVES
#define VQ_MFMA_WAVES 8
#endif
constexpr int MW = VQ_MFMA_WAVES;
constexpr int NARROW_WAVES = 4;            // workgroup size for layers whose codebook groups are narrow (see narrow_groups)

}  // namespace


namespace {

struct Planned {
  MfmaPlan plan;
  unsigned lds_bytes, grid;
  int rb;
  bool grouped;
};

// Work split and LDS layout of one layer when every workgroup takes `blocks_per_wg` 16-row blocks.  nb_force > 0
// fixes the blocks per chunk (several layers in one launch share one kernel instantiation).
// `waves` and `lds_cap`: the workgroup's size and its share of the compute unit's LDS (the defaults: one workgroup of
// MW waves per compute unit).
int make_plan(const Params &p, int batch, long long ldx, const __half *y, long long ldy, int blocks_per_wg, int nb_force, Planned *out,
              bool partial = false, int waves = MW, unsigned lds_cap = 160u * 1024u) {
  MfmaPlan plan{};
  if (p.in_features < 64) return VQ_ERR_UNSUPPORTED;      // idle lanes load the first 100 bytes of the first activation row
  const int rb = p.k_res ? p.bits_res : 0;
  unsigned off = rb == 0 ? Layout<0>::BYTES : rb == 8 ? Layout<8>::BYTES : Layout<12>::BYTES;
  // the 32 KB outlier table goes into LDS too, unless two 64 KB tables are already there
  plan.out_global = p.Q && rb == 12 ? 1 : 0;
  plan.lds_out = off; off += p.Q && !plan.out_global ? 4096u * 8u : 0u;
  plan.lds_xs = off; off += (unsigned)waves * 16u * 4u;
  const int blocks_total = (p.out_features + 15) / 16;
  plan.rows_per_wg = blocks_per_wg * 16;
  out->grid = (unsigned)((blocks_total + blocks_per_wg - 1) / blocks_per_wg);
  plan.lds_sb = off; off += partial ? 0u : (unsigned)plan.rows_per_wg * 4u;
  const bool grouped = p.n_groups > 1;
  if (grouped && (p.Pg & 7)) return VQ_ERR_UNSUPPORTED;   // a group must start on a dword of the 12- and 8-bit streams
  plan.lds_yacc = off; off += grouped && !partial ? (unsigned)blocks_per_wg * 1024u : 0u;
  plan.lds_part = off;
  if (off + (unsigned)waves * 1024u > lds_cap) return VQ_ERR_UNSUPPORTED;
  const int fit = (int)((lds_cap - off) / ((unsigned)waves * 1024u));    // 16-row partial blocks that fit
  // Blocks per chunk: as many as the kernel's 256 registers allow -- four, or three with a residual index stream in the
  // prefetch ring.  More would spill, which these kernels must not (see the build script).
  // (with codebook groups one fewer: the group loop costs registers of its own)
  const int nb_regs = grouped ? (rb == 12 ? 2 : 3) : (rb ? 3 : NBMAX);
  plan.nb = min(min(nb_regs, blocks_per_wg), fit);
  if (nb_force > 0) { if (nb_force > plan.nb) return VQ_ERR_UNSUPPORTED; plan.nb = nb_force; }
  if (plan.nb < 1) return VQ_ERR_UNSUPPORTED;
  plan.part_bufs = (fit >= 2 * plan.nb && blocks_per_wg > plan.nb) ? 2 : 1;
  off += (unsigned)(plan.part_bufs * plan.nb) * ((unsigned)waves * 1024u);
  const long long max_stride = max(p.stride, max(p.stride_res, p.stride_out));
  if ((long long)(plan.rows_per_wg + 16 * NBMAX * 8) * max_stride >= (1LL << 31)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  const long long x_bytes = ((long long)(batch - 1) * ldx + p.in_features) * 2;
  if (ldx < 0 || x_bytes >= (1LL << 31) - (1 << 20)) return VQ_ERR_UNSUPPORTED;
  plan.x_bytes = (unsigned)x_bytes;
  plan.y_wide = ((reinterpret_cast<uintptr_t>(y) & 7) == 0 && (ldy & 3) == 0) ? 1 : 0;
  out->plan = plan; out->lds_bytes = off; out->rb = rb; out->grouped = grouped;
  return VQ_OK;
}

// A codebook group of at most 128 vectors gives work to four waves at most (a wave takes 32 vectors of a row at a
// time): such layers run in workgroups of four waves, two to a compute unit, each with its own copy of its group's
// tables -- when two copies fit the LDS, i.e. without a 12-bit residual table and without the outlier table.  Only
// with a workspace, where a workgroup loads one group's tables: when every workgroup walks all groups the table
// loads dominate, and twice as many workgroups doing them was measured slower (15 groups of 48 vectors on an
// 11008 x 4096 layer, batch 4: 66 us against 55 us).
bool narrow_groups(const Params &p) {
  return p.n_groups > 1 && (p.Pg + 31) / 32 <= NARROW_WAVES && !(p.k_res && p.bits_res == 12) && p.Q == 0;
}

template <int RES_BITS, int NB>
int launch_multi(const MultiArgs &a, unsigned lds_bytes, unsigned grid, const __half *x, long long ldx, int batch, hipStream_t s) {
  auto kernel = gemv_v6_mfma_multi_kernel<RES_BITS, MW, NB>;
  VQ_ALLOW_FULL_LDS(kernel);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(MW * 64), lds_bytes, s, a, x, ldx, batch);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Launch for batch 1..16.  The caller has checked gemv_fast_applicable().
int launch_gemv_mfma(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  const int blocks_total = (p.out_features + 15) / 16;
  const int cus = cu_count();
  Planned pl;
  const int rc = make_plan(p, batch, ldx, y, ldy, (blocks_total + cus - 1) / cus, 0, &pl);
  if (rc != VQ_OK) return rc;
  const MfmaPlan &plan = pl.plan;
  const int rb = pl.rb;
  const bool grouped = pl.grouped;
  const unsigned off = pl.lds_bytes, grid = pl.grid;
#define VQ_CASE(RBITS, NBLK) \
  if (rb == RBITS && plan.nb == NBLK && !grouped) return launch_one<RBITS, MW, NBLK, false>(p, plan, off, grid, x, ldx, batch, y, ldy, s); \
  if (rb == RBITS && plan.nb == NBLK && grouped && NBLK <= (RBITS == 12 ? 2 : 3)) \
    return launch_one<RBITS, MW, (NBLK <= (RBITS == 12 ? 2 : 3) ? NBLK : 1), true>(p, plan, off, grid, x, ldx, batch, y, ldy, s);
  VQ_CASE(0, 1) VQ_CASE(0, 2) VQ_CASE(0, 3) VQ_CASE(0, 4)
  VQ_CASE(8, 1) VQ_CASE(8, 2) VQ_CASE(8, 3)
  VQ_CASE(12, 1) VQ_CASE(12, 2) VQ_CASE(12, 3)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

// Bytes of the workspace with which a layer with codebook groups runs as "one group per workgroup, then add up"; 0 when
// that route does not apply (one group, group size not a multiple of 8 vectors, more groups than compute units).
size_t gemv_mfma_groups_workspace_bytes(const Params &p, int batch) {
  if (p.n_groups < 2 || (p.Pg & 7) || p.n_groups > cu_count()) return 0;
  return ((size_t)p.n_groups * ((size_t)batch * (size_t)p.out_features + 16) * sizeof(float) + 255) / 256 * 256;
}

// The caller has checked gemv_fast_applicable() and that the workspace holds gemv_mfma_groups_workspace_bytes().
int launch_gemv_mfma_groups(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, void *workspace,
                            hipStream_t s) {
  const int blocks_total = (p.out_features + 15) / 16;
  bool narrow = narrow_groups(p) && 2 * cu_count() / p.n_groups >= 1;
  Planned pl;
  int rc = VQ_ERR_UNSUPPORTED;
  if (narrow) {
    const int wgs_per_group = 2 * cu_count() / p.n_groups;
    rc = make_plan(p, batch, ldx, y, ldy, (blocks_total + wgs_per_group - 1) / wgs_per_group, 0, &pl, true, NARROW_WAVES, 80u * 1024u);
    if (rc != VQ_OK) narrow = false;
  }
  if (!narrow) {
    const int wgs_per_group = cu_count() / p.n_groups;
    if (wgs_per_group < 1) return VQ_ERR_UNSUPPORTED;
    rc = make_plan(p, batch, ldx, y, ldy, (blocks_total + wgs_per_group - 1) / wgs_per_group, 0, &pl, true);
    if (rc != VQ_OK) return rc;
  }
  float *part = static_cast<float *>(workspace);
  float *part_xs = part + (size_t)p.n_groups * (size_t)batch * (size_t)p.out_features;
  const unsigned grid = pl.grid * (unsigned)p.n_groups;            // pl.grid workgroups per group
  const void *kernel = nullptr;
#define VQ_CASE(RBITS, NBLK) \
  if (!narrow && pl.rb == RBITS && pl.plan.nb == NBLK && NBLK <= (RBITS == 12 ? 2 : 3)) \
    kernel = reinterpret_cast<const void *>(gemv_v6_mfma_groups_kernel<RBITS, MW, (NBLK <= (RBITS == 12 ? 2 : 3) ? NBLK : 1)>);
  VQ_CASE(0, 1) VQ_CASE(0, 2) VQ_CASE(0, 3) VQ_CASE(8, 1) VQ_CASE(8, 2) VQ_CASE(8, 3) VQ_CASE(12, 1) VQ_CASE(12, 2)
#undef VQ_CASE
#define VQ_CASE(RBITS, NBLK) \
  if (narrow && pl.rb == RBITS && pl.plan.nb == NBLK) kernel = reinterpret_cast<const void *>(gemv_v6_mfma_groups_kernel<RBITS, NARROW_WAVES, NBLK>);
  VQ_CASE(0, 1) VQ_CASE(0, 2) VQ_CASE(0, 3) VQ_CASE(8, 1) VQ_CASE(8, 2)
#undef VQ_CASE
  if (!kernel) return VQ_ERR_UNSUPPORTED;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return VQ_ERR_HIP;
  Params pc = p;
  MfmaPlan plan = pl.plan;
  int wpg = (int)pl.grid;
  void *args[] = {&pc, &plan, &x, &ldx, &batch, &part, &part_xs, &wpg};
  if (hipLaunchKernel(kernel, dim3(grid), dim3((narrow ? NARROW_WAVES : MW) * 64), args, pl.lds_bytes, s) != hipSuccess) return VQ_ERR_HIP;
  launch_finish(part, part_xs, p.n_groups, batch, p, y, ldy, s);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// y = scale * (sum over the groups) + bias * (sum of their activation sums), for any kernel that left per-group sums in a workspace.
int launch_groups_finish(const float *part, const float *part_xs, int n_groups, int batch, const Params &p, __half *y, long long ldy,
                         hipStream_t s) {
  launch_finish(part, part_xs, n_groups, batch, p, y, ldy, s);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// n layers (2 .. MULTI_MAX) on the same activations in one launch.  VQ_ERR_UNSUPPORTED when the layers do not fit
// one kernel instantiation (different residual kinds, codebook groups, different in_features) or one launch; the
// caller then launches them one by one.  The caller has checked gemv_fast_applicable() for each.
int launch_gemv_mfma_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys,
                           const long long *ldys, hipStream_t s) {
  if (n < 2 || n > MULTI_MAX) return VQ_ERR_UNSUPPORTED;
  const int cus = cu_count();
  long long blocks_all = 0;
  for (int i = 0; i < n; ++i) {
    if (ps[i].in_features != ps[0].in_features || ps[i].n_groups > 1) return VQ_ERR_UNSUPPORTED;
    if ((ps[i].k_res ? ps[i].bits_res : 0) != (ps[0].k_res ? ps[0].bits_res : 0)) return VQ_ERR_UNSUPPORTED;
    blocks_all += (ps[i].out_features + 15) / 16;
  }
  // every workgroup takes the same number of 16-row blocks of one layer: the smallest number with which all the
  // workgroups run at once, one per compute unit
  int b = (int)((blocks_all + cus - 1) / cus);
  for (;; ++b) {
    long long wgs = 0;
    for (int i = 0; i < n; ++i) wgs += ((ps[i].out_features + 15) / 16 + b - 1) / b;
    if (wgs <= cus) break;
  }
  MultiArgs a{};
  Planned pl[MULTI_MAX];
  int nb = NBMAX;
  for (int pass = 0; pass < 2; ++pass) {                  // first the blocks per chunk every layer admits, then the plans with it
    for (int i = 0; i < n; ++i) {
      const int rc = make_plan(ps[i], batch, ldx, ys[i], ldys[i], b, pass ? nb : 0, &pl[i]);
      if (rc != VQ_OK) return rc;
      if (!pass) nb = min(nb, pl[i].plan.nb);
    }
  }
  unsigned lds_bytes = 0;
  a.n = n;
  for (int i = 0; i < n; ++i) {
    a.first_wg[i + 1] = a.first_wg[i] + (int)pl[i].grid;
    a.layer[i].p = ps[i]; a.layer[i].plan = pl[i].plan; a.layer[i].y = ys[i]; a.layer[i].ldy = ldys[i];
    lds_bytes = max(lds_bytes, pl[i].lds_bytes);
  }
  const unsigned grid = (unsigned)a.first_wg[n];
  const int rb = pl[0].rb;
#define VQ_CASE(RBITS, NBLK) if (rb == RBITS && nb == NBLK) return launch_multi<RBITS, NBLK>(a, lds_bytes, grid, x, ldx, batch, s);
  VQ_CASE(0, 1) VQ_CASE(0, 2) VQ_CASE(0, 3) VQ_CASE(0, 4)
  VQ_CASE(8, 1) VQ_CASE(8, 2) VQ_CASE(8, 3)
  VQ_CASE(12, 1) VQ_CASE(12, 2) VQ_CASE(12, 3)
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
