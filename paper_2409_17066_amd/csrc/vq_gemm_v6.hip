// vq_gemm without a workspace for v = 6 layers with 12-bit indices (the 2-bit settings of the paper's main tables): Y = X * W^T
// with W restored on the fly from codebooks that sit in LDS, W never in memory (App. "Our Dequantization Implementation",
// prompt phase; Sec. 3.2.2 for the residual sum).
//
// The tile machinery is that of the v = 8 kernel (vq_gemm_fused.hip): a workgroup owns BM tokens x 128 output channels, BM / 64
// consumer waves issue v_mfma_f32_32x32x16_f16 from swizzled 64-byte LDS rows, four producer waves write the FP16 W tile of
// every 32-column step (double buffered), one LDS-only barrier per step.  What differs is where the centroids come from:
// the main table (and a residual table of up to 4096 entries) is staged once per workgroup in LDS as 16-byte entries, so a
// lookup is one ds_read_b128 instead of a 128-byte line out of L2 -- which is what bounds the v = 8 kernel.  A 32-column
// step does not hold whole 6-column vectors: a producer thread makes 16 consecutive columns of one channel, which lie in the
// four vectors from floor(c0 / 6) on; c0 is a multiple of 16, so they start 0, 1 or 2 dwords into the twelve dwords of those
// four entries.  Its 48 index bits (and 32 or 48 residual index bits) are three dwords of the channel's stream, loaded GD
// steps ahead from inline assembly and waited for by count.  Outlier columns (Sec. 3.2.3: the first n_outlier_cols stored
// columns, here in whole runs of 16) are the few steps at the start of every row; a producer thread looks those up one
// column at a time through the caches, with ordinary loads.
// LDS: tables 64 KB (+ 64 KB or 4 KB), W tiles 16 KB, activation stages BM x 64 bytes each -- with a 12-bit residual table
// that leaves room for two stages of 128 tokens, which is the tile such layers get.
#include "vq_gemm_tiles.hpp"

namespace vq {

namespace {

using namespace gemm_tiles;

typedef unsigned uint3v __attribute__((ext_vector_type(3)));

__device__ __forceinline__ void async_load12(uint3v &dst, __amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
  asm volatile("buffer_load_dwordx3 %0, %1, %2, 0 offen" : "=&v"(dst) : "v"(byte_offset), "s"(r) : "memory");
}
__device__ __forceinline__ void lds_read16(uint4v &dst, unsigned lds_addr) { asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(lds_addr)); }

// main + residual (binary32 sum, Sec. 3.2.2), scale and bias, two weights at a time
template <bool RES>
__device__ __forceinline__ unsigned restore_pair(unsigned main, unsigned res, float s, float b) {
  float lo = __half2float(__ushort_as_half((unsigned short)(main & 0xFFFFu)));
  float hi = __half2float(__ushort_as_half((unsigned short)(main >> 16)));
  if (RES) {
    lo = __fadd_rn(lo, __half2float(__ushort_as_half((unsigned short)(res & 0xFFFFu))));
    hi = __fadd_rn(hi, __half2float(__ushort_as_half((unsigned short)(res >> 16))));
  }
  return (unsigned)__half_as_ushort(restore(lo, s, b)) | ((unsigned)__half_as_ushort(restore(hi, s, b)) << 16);
}

// XD: activation copies run this many steps ahead, in XD + 1 stages.
template <int BM, int RES_BITS, int XD>
__global__ __launch_bounds__((BM / 64 + 4) * 64) void gemm_v6_kernel(Params p, const __half *__restrict__ X, long long ldx, int tokens,
                                                                     __half *__restrict__ Y, long long ldy) {
  constexpr int NC = BM / 64;                   // consumer waves: each owns 64 token rows x 128 channels
  constexpr int NT = (NC + 4) * 64;             // threads
  constexpr int MB = 2;                         // 32-row MFMA blocks per consumer wave along the tokens
  constexpr int NSX6 = XD + 1;
  constexpr unsigned XSTAGE = BM * 64u;         // bytes per activation stage
  constexpr unsigned W_OFF = NSX6 * XSTAGE, TAB_OFF = W_OFF + 2u * BN * LDT * 2u, RES_OFF = TAB_OFF + 65536u;
  constexpr int RES_ENTRIES = RES_BITS == 12 ? 4096 : RES_BITS == 8 ? 256 : 0;
  constexpr int LOADS = RES_BITS ? 2 : 1;       // index loads per producer thread and step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *Xs = smem;                                                        // [NSX6][BM][64 bytes]
  __half *Ws = reinterpret_cast<__half *>(smem + W_OFF);                           // [2][BN][LDT]

  const int lane = threadIdx.x & 63;
  const int wave8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool producer = wave8 >= NC;
  const int wave = producer ? wave8 - NC : wave8;             // index within the role
  const int tid = producer ? (int)threadIdx.x - NC * 64 : (int)threadIdx.x;   // thread index within the role
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int ksteps = p.in_features / BK;

  // ---- tables into LDS, entries padded 12 -> 16 bytes, zero past the table's k entries (what an index >= k then reads)
  for (int e = threadIdx.x; e < 4096 + RES_ENTRIES; e += NT) {
    const bool res = e >= 4096;
    const int i = res ? e - 4096 : e;
    uint4v v = {0u, 0u, 0u, 0u};
    if (i < (res ? p.k_res : p.k)) {
      const unsigned *src = reinterpret_cast<const unsigned *>(res ? p.cb_res : p.cb) + (long long)i * 3;
      v.x = src[0]; v.y = src[1]; v.z = src[2];
    }
    *reinterpret_cast<uint4v *>(smem + (res ? RES_OFF : TAB_OFF) + (unsigned)i * 16u) = v;
  }
  __syncthreads();
  const unsigned lds0 = (unsigned)reinterpret_cast<size_t>((const __attribute__((address_space(3))) void *)smem);

  // activations: range-checked against the end of the last token row, so rows >= tokens read zeros
  const __amdgpu_buffer_rsrc_t r_x = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<__half *>(X), 0, (unsigned)(((long long)(tokens - 1) * ldx + p.in_features) * 2), 0x00020000);

  if (producer) {
    // this thread's share of the W tile: channel w_row, columns 16 w_half .. + 15 of every step (w_half is the same for a whole wave)
    const int w_row = tid & 127, w_half = __builtin_amdgcn_readfirstlane(tid >> 7);
    const bool w_on = n0 + w_row < p.out_features;
    const int o_w = min(n0 + w_row, p.out_features - 1);
    const float s_w = p.scale ? __half2float(p.scale[o_w]) : 1.0f;
    const float b_w = p.bias ? __half2float(p.bias[o_w]) : 0.0f;
    // index streams, range-checked over the whole arrays (the four vectors of a step may reach past the end of a row: such
    // indices meet columns past in_features, which no step holds)
    const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.out_features * p.stride), 0x00020000);
    const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(RES_BITS ? p.idx_res : p.idx), 0,
                                                                         RES_BITS ? (unsigned)((long long)p.out_features * p.stride_res) : 0u, 0x00020000);
    const unsigned row_i = (unsigned)o_w * (unsigned)p.stride, row_r = (unsigned)o_w * (unsigned)p.stride_res;
    constexpr int RB = RES_BITS == 8 ? 8 : 12;
    uint3v ireg[GD], rreg[GD];                  // index dwords of the steps in flight; step kt uses slot kt % GD
    // first vector and dword offset into the twelve dwords of step kt (wave-uniform: scalar arithmetic)
    // (stored columns [0, n_out) are the outlier columns, n_out a multiple of 16: a thread's 16 columns of a step are either all
    // outlier columns, made by make_outlier_tile below while the ring loads main-stream words that nobody looks at, or none)
    auto main_col = [&](int kt) { return (unsigned)max(kt * BK + w_half * 16 - p.n_out, 0); };
    auto first_vector = [&](int kt) { return main_col(kt) / 6u; };
    auto issue = [&](int slot, int kt) {
      const unsigned p0 = first_vector(kt);
      async_load12(ireg[slot], r_i, row_i + ((p0 * 12u) >> 5) * 4u);
      if (RES_BITS) async_load12(rreg[slot], r_r, row_r + ((p0 * (unsigned)RB) >> 5) * 4u);
    };
    // four consecutive BITS-bit fields that start `sh` bits into three dwords
    auto fields = [&](const uint3v &w, unsigned sh, int bits, unsigned (&out)[4]) {
      const unsigned lo = __builtin_amdgcn_alignbit(w.y, w.x, sh), hi = __builtin_amdgcn_alignbit(w.z, w.y, sh);   // bits [sh, sh + 32), [sh + 32, sh + 64)
      const unsigned mask = (1u << bits) - 1u;
      out[0] = lo & mask;
      out[1] = (lo >> bits) & mask;
      out[2] = bits == 12 ? __builtin_amdgcn_alignbit(hi, lo, 24) & mask : (lo >> 16) & mask;
      out[3] = bits == 12 ? (hi >> 4) & mask : lo >> 24;
    };
    // 16 outlier columns (Sec. 3.2.3) from stored column col0 on: their own stream and table, no residual; the few steps that
    // hold them (288 of 28672 columns on the 70B layer) look every column up through the caches with ordinary loads
    auto make_outlier_tile = [&](int buf, int col0) {
      const uint8_t *ro = p.idx_out + (long long)o_w * p.stride_out;
      unsigned h[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = col0 + j, q = c / p.v_out, el = c - q * p.v_out;
        const unsigned i = min(load_index(ro, q, p.bits_out), (unsigned)p.k_out - 1u);
        h[j] = (unsigned)__half_as_ushort(p.cb_out[(long long)i * p.v_out + el]);
      }
      uint4v a, b;
      a.x = restore_pair<false>(h[0] | (h[1] << 16), 0u, s_w, b_w);   a.y = restore_pair<false>(h[2] | (h[3] << 16), 0u, s_w, b_w);
      a.z = restore_pair<false>(h[4] | (h[5] << 16), 0u, s_w, b_w);   a.w = restore_pair<false>(h[6] | (h[7] << 16), 0u, s_w, b_w);
      b.x = restore_pair<false>(h[8] | (h[9] << 16), 0u, s_w, b_w);   b.y = restore_pair<false>(h[10] | (h[11] << 16), 0u, s_w, b_w);
      b.z = restore_pair<false>(h[12] | (h[13] << 16), 0u, s_w, b_w); b.w = restore_pair<false>(h[14] | (h[15] << 16), 0u, s_w, b_w);
      if (!w_on) { a = uint4v{0u, 0u, 0u, 0u}; b = uint4v{0u, 0u, 0u, 0u}; }
      unsigned char *wt = reinterpret_cast<unsigned char *>(Ws + buf * BN * LDT);
      *reinterpret_cast<uint4v *>(wt + x_slot((unsigned)w_row, (unsigned)(w_half * 2))) = a;
      *reinterpret_cast<uint4v *>(wt + x_slot((unsigned)w_row, (unsigned)(w_half * 2 + 1))) = b;
    };
    auto make_tile = [&](int buf, int slot, int kt) {
      settle(ireg[slot]);
      if (RES_BITS) settle(rreg[slot]);
      if (kt * BK + w_half * 16 < p.n_out) { make_outlier_tile(buf, kt * BK + w_half * 16); return; }   // (the same for the whole wave)
      const unsigned p0 = first_vector(kt);
      const unsigned skip = (main_col(kt) - p0 * 6u) >> 1;        // 0, 1 or 2 dwords of the first entry lie before the run
      unsigned im[4], ir[4];
      fields(ireg[slot], (p0 * 12u) & 31u, 12, im);
      if (RES_BITS) fields(rreg[slot], (p0 * (unsigned)RB) & 31u, RB, ir);
      uint4v e[4], f[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) lds_read16(e[q], lds0 + TAB_OFF + im[q] * 16u);
      if (RES_BITS) {
#pragma unroll
        for (int q = 0; q < 4; ++q) lds_read16(f[q], lds0 + RES_OFF + min(ir[q], (unsigned)RES_ENTRIES - 1u) * 16u);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int q = 0; q < 4; ++q) { settle(e[q]); if (RES_BITS) settle(f[q]); }
      // the run starts `skip` dwords into the twelve dwords of the four entries: three straight-line versions, chosen by a
      // wave-uniform branch (one version that picks its dwords at run time keeps them in an array in scratch memory)
      unsigned char *wt = reinterpret_cast<unsigned char *>(Ws + buf * BN * LDT);
      auto emit = [&](unsigned m0, unsigned m1, unsigned m2, unsigned m3, unsigned m4, unsigned m5, unsigned m6, unsigned m7,
                      unsigned r0, unsigned r1, unsigned r2, unsigned r3, unsigned r4, unsigned r5, unsigned r6, unsigned r7) {
        uint4v a, b;
        a.x = restore_pair<RES_BITS != 0>(m0, r0, s_w, b_w); a.y = restore_pair<RES_BITS != 0>(m1, r1, s_w, b_w);
        a.z = restore_pair<RES_BITS != 0>(m2, r2, s_w, b_w); a.w = restore_pair<RES_BITS != 0>(m3, r3, s_w, b_w);
        b.x = restore_pair<RES_BITS != 0>(m4, r4, s_w, b_w); b.y = restore_pair<RES_BITS != 0>(m5, r5, s_w, b_w);
        b.z = restore_pair<RES_BITS != 0>(m6, r6, s_w, b_w); b.w = restore_pair<RES_BITS != 0>(m7, r7, s_w, b_w);
        if (!w_on) { a = uint4v{0u, 0u, 0u, 0u}; b = uint4v{0u, 0u, 0u, 0u}; }
        *reinterpret_cast<uint4v *>(wt + x_slot((unsigned)w_row, (unsigned)(w_half * 2))) = a;
        *reinterpret_cast<uint4v *>(wt + x_slot((unsigned)w_row, (unsigned)(w_half * 2 + 1))) = b;
      };
      if (!RES_BITS) {
#pragma unroll
        for (int q = 0; q < 4; ++q) f[q] = uint4v{0u, 0u, 0u, 0u};
      }
      if (skip == 0) emit(e[0].x, e[0].y, e[0].z, e[1].x, e[1].y, e[1].z, e[2].x, e[2].y, f[0].x, f[0].y, f[0].z, f[1].x, f[1].y, f[1].z, f[2].x, f[2].y);
      else if (skip == 1) emit(e[0].y, e[0].z, e[1].x, e[1].y, e[1].z, e[2].x, e[2].y, e[2].z, f[0].y, f[0].z, f[1].x, f[1].y, f[1].z, f[2].x, f[2].y, f[2].z);
      else emit(e[0].z, e[1].x, e[1].y, e[1].z, e[2].x, e[2].y, e[2].z, e[3].x, f[0].z, f[1].x, f[1].y, f[1].z, f[2].x, f[2].y, f[2].z, f[3].x);
    };
    // Memory operations of a producer wave, in issue order: LOADS index loads per step (for step kt + 1 + GD), every step, also
    // where that step lies past the last one (the last step's words are loaded again and never looked at): the same
    // number of loads separates every load from its use, so one counted wait serves all steps, on every path.
#pragma unroll
    for (int j = 0; j < GD; ++j) issue(j, j);                                   // steps 0 .. GD-1 (ksteps % GD == 0)
    wait_vmem_at_most<0>();
    make_tile(0, 0, 0);
    issue(0, min(GD, ksteps - 1));                                              // slot 0 now carries step GD
    step_barrier();
    for (int k0 = 0; k0 < ksteps; k0 += GD) {
#pragma unroll
      for (int j = 0; j < GD; ++j) {
        const int kt = k0 + j;
        // the loads of step kt+1 (slot (j+1) % GD) went out at the end of step kt-GD, followed by LOADS in each of the GD-1 steps since
        wait_vmem_at_most<LOADS * (GD - 1)>();
        const int sl = (j + 1) % GD;
        make_tile((kt & 1) ^ 1, sl, min(kt + 1, ksteps - 1));                   // (after the last step: a tile nobody reads)
        issue(sl, min(kt + 1 + GD, ksteps - 1));
        step_barrier();
      }
    }
    wait_vmem_at_most<0>();
    return;
  }

  // ---- consumers: each wave streams its own 64 token rows through its slice of the activation stages (no other wave
  // touches them, so only the wave's own counted wait stands between a copy and its use) and multiplies
  auto copy_x = [&](int kt) {
    const unsigned stage = (unsigned)(kt % NSX6) * XSTAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned piece = (unsigned)(wave * 4 + i);                  // 16 rows per 1 KB piece
      const unsigned r = piece * 16u + ((unsigned)lane >> 2), cs = (unsigned)lane & 3u;   // LDS slot (r, cs) holds chunk cs ^ swz(r)
      const unsigned c = cs ^ swz(r);
      const unsigned goff = (unsigned)(((long long)(m0 + (int)r) * ldx + (long long)kt * BK + c * 8) * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(Xs + stage + piece * 1024u), 16, goff, 0, 0, 0);
    }
  };
  float16v acc[MB][4];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
  const int wm = wave * 64;
#pragma unroll
  for (int j = 0; j < XD; ++j)
    if (j < ksteps) copy_x(j);
  wait_vmem_at_most<0>();
  step_barrier();                                               // the W tile of step 0 is in LDS
  for (int kt = 0; kt < ksteps; ++kt) {
    const int cur = kt & 1;
    if (kt + XD < ksteps) copy_x(kt + XD);
    const unsigned char *xs = Xs + (unsigned)(kt % NSX6) * XSTAGE;
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      half8 af[MB], bf[4];
#pragma unroll
      for (int a = 0; a < MB; ++a)
        af[a] = *reinterpret_cast<const half8 *>(xs + x_slot((unsigned)(wm + a * 32 + (lane & 31)), (unsigned)(ks / 8 + (lane >> 5))));
#pragma unroll
      for (int c = 0; c < 4; ++c)
        bf[c] = *reinterpret_cast<const half8 *>(reinterpret_cast<const unsigned char *>(Ws + cur * BN * LDT) + x_slot((unsigned)(c * 32 + (lane & 31)), (unsigned)(ks / 8 + (lane >> 5))));
#pragma unroll
      for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[c], acc[a][c], 0, 0, 0);
    }
    // this wave's rows of step kt+1 went out at step kt+1-XD; four copies per step since
    if (kt + XD < ksteps) wait_vmem_at_most<4 * (XD - 1)>(); else wait_vmem_at_most<0>();
    step_barrier();
  }

  // ---- store: lane holds channel (lane & 31) of block c and 16 token rows of block a
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int o = n0 + c * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = m0 + wm + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (t < tokens && o < p.out_features) Y[(long long)t * ldy + o] = __float2half_rn(acc[a][c][r]);
      }
    }
}

template <int BM, int RES_BITS, int XD>
int launch_v6(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, hipStream_t s) {
  auto kernel = gemm_v6_kernel<BM, RES_BITS, XD>;
  const unsigned lds = (XD + 1) * BM * 64u + 2u * BN * LDT * 2u + 65536u + (RES_BITS == 12 ? 65536u : RES_BITS == 8 ? 4096u : 0u);
  static_assert((XD + 1) * BM * 64u + 2u * BN * LDT * 2u + 65536u + (RES_BITS == 12 ? 65536u : RES_BITS == 8 ? 4096u : 0u) <= 160u * 1024u, "LDS");
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned gx = (unsigned)((p.out_features + BN - 1) / BN), gy = (unsigned)((tokens + BM - 1) / BM);
  if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3(gx, gy), dim3((BM / 64 + 4) * 64), lds, s, p, X, ldx, tokens, Y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// v = 6 with 12-bit indices along the rows, outlier columns in whole runs of 16, one codebook group, no residual or one of 8 or
// 12 index bits; whole groups of GD steps; stream offsets that fit 32 bits.
bool gemm_v6_applicable(const Params &p) {
  return p.orientation == 0 && p.v == 6 && p.bits == 12 && p.n_out % 16 == 0 && p.n_groups == 1 && !p.perm &&
         (p.k_res == 0 || p.bits_res == 8 || p.bits_res == 12) && p.in_features % (GD * BK) == 0 &&
         (long long)p.out_features * p.stride < (1LL << 32) && (long long)p.out_features * p.stride_res < (1LL << 32);
}

int launch_gemm_v6(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, hipStream_t s) {
  if (((long long)(tokens - 1) * ldx + p.in_features) * 2 >= (1LL << 32)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  const long long col_blocks = (p.out_features + BN - 1) / BN;
  if (p.k_res && p.bits_res == 12) return launch_v6<128, 12, 1>(p, X, ldx, tokens, Y, ldy, s);      // what fits beside two 64 KB tables
  // lookups out of LDS are cheap, so the token tile only has to fill the chip: the tallest that still gives 200 workgroups
  const int bm = col_blocks * ((tokens + 255) / 256) >= 200 ? 256 : 128;
  if (p.k_res) return bm == 256 ? launch_v6<256, 8, 3>(p, X, ldx, tokens, Y, ldy, s) : launch_v6<128, 8, 3>(p, X, ldx, tokens, Y, ldy, s);
  return bm == 256 ? launch_v6<256, 0, 3>(p, X, ldx, tokens, Y, ldy, s) : launch_v6<128, 0, 3>(p, X, ldx, tokens, Y, ldy, s);
}

}  // namespace vq
