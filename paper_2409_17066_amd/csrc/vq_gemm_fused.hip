// vq_gemm fast path for v = 8 with 16-bit indices (k up to 65536: the codebook is 1 MiB and lives in
// L2 / Infinity Cache, not in LDS), no residual, no outlier columns -- the paper's v=8 / k=65536 setting
// (App. "Impact of Vector Length").  Y = X * W^T with W restored on the fly; W never touches memory.
// The same kernel also runs "dense": its producers then copy tiles of an FP16 W that vq_dequant has written
// to a caller-supplied workspace (the paper's own prompt-phase scheme, Sec. on inference throughput), which
// on this hardware is the faster route once a workspace is there: see launch_gemm in vq_gemm.hip.
//
// A workgroup owns BM tokens x 128 output channels and splits its waves in two roles that share the SIMDs:
//  * BM/64 "consumer" waves only issue MFMA: wave w owns token rows [64 w, 64 w + 64) and all 128 channels as
//    2 x 4 blocks of v_mfma_f32_32x32x16_f16, reading both operands from LDS;
//  * four "producer" waves keep the tiles coming: per 32-column step they gather 128 x 4 centroids
//    (16 bytes each, two per thread, issued GD steps ahead), apply scale and bias, write the FP16 W tile
//    to LDS (double buffered), and start the asynchronous global->LDS copies of the activation tile
//    XD steps ahead (XOR-swizzled 64-byte rows).
// One barrier per step.  The taller the token tile, the fewer times a centroid is gathered: each gather
// pulls a whole 128-byte line out of L2 for 16 useful bytes, which is what finally bounds this kernel.
#include "vq_gemm_tiles.hpp"
#include <cstdlib>

namespace vq {

namespace {

using namespace gemm_tiles;

// in_features % 32 == 0 here.  Wave w owns token rows [w*BM/4, (w+1)*BM/4) and all 128 channels.
template <int BM, bool DENSE>
__global__ __launch_bounds__((BM / 64 + 4) * 64) void gemm_v8_kernel(Params p, const __half *__restrict__ X, long long ldx, int tokens,
                                                      __half *__restrict__ Y, long long ldy, const __half *__restrict__ Wd, long long ldw) {
  constexpr int NC = BM / 64;                   // consumer waves: each owns 64 token rows x 128 channels
  constexpr int MB = 2;                         // 32-row MFMA blocks per consumer wave along the tokens
  constexpr unsigned XSTAGE = BM * 64u;         // bytes per activation stage
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *Xs = smem;                                                        // [NSX][BM][64 bytes]
  __half *Ws = reinterpret_cast<__half *>(smem + NSX * XSTAGE);                    // [2][BN][LDT]

  const int lane = threadIdx.x & 63;
  const int wave8 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool producer = wave8 >= NC;
  const int wave = producer ? wave8 - NC : wave8;             // index within the role
  const int tid = producer ? (int)threadIdx.x - NC * 64 : (int)threadIdx.x;   // thread index within the role
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int ksteps = p.in_features / BK;

  // ---- this thread's share of the W tile: row w_row, vectors 2*w_half and 2*w_half + 1 of every step
  const int w_row = tid >> 1, w_half = tid & 1;
  const bool w_on = n0 + w_row < p.out_features;
  const int o_w = min(n0 + w_row, p.out_features - 1);
  const float s_w = p.scale ? __half2float(p.scale[o_w]) : 1.0f;
  const float b_w = p.bias ? __half2float(p.bias[o_w]) : 0.0f;
  // activations: range-checked against the end of the last token row, so rows >= tokens read zeros
  const __amdgpu_buffer_rsrc_t r_x = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<__half *>(X), 0, (unsigned)(((long long)(tokens - 1) * ldx + p.in_features) * 2), 0x00020000);

  // The two roles run separate loops with the same number of barriers (one after the prologue, one per step),
  // so that the accumulators of the consumers and the gather registers of the producers never live together.
  if (producer && DENSE) {
    // W comes from memory as FP16 rows (ldw halfs apart, 16-byte aligned): this thread copies 32 bytes of row
    // w_row per step, GD steps ahead, through registers into the same LDS tile the gather path fills.
    uint4v greg[GD][2];
    const unsigned char *wrow = reinterpret_cast<const unsigned char *>(Wd + (long long)o_w * ldw) + w_half * 32;
    auto issue_copy = [&](uint4v (&g)[2], int kt) {
      async_load16(g[0], wrow + (long long)kt * (BK * 2));
      async_load16(g[1], wrow + (long long)kt * (BK * 2) + 16);
    };
    auto store_w = [&](int buf, uint4v (&g)[2]) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        settle(g[j]);
        *reinterpret_cast<uint4v *>(reinterpret_cast<unsigned char *>(Ws + buf * BN * LDT) + x_slot((unsigned)w_row, (unsigned)(w_half * 2 + j))) = w_on ? g[j] : uint4v{0u, 0u, 0u, 0u};
      }
    };
#pragma unroll
    for (int j = 0; j < GD; ++j) issue_copy(greg[j], j);                      // steps 0 .. GD-1 (ksteps % GD == 0)
    wait_vmem_at_most<0>();
    store_w(0, greg[0]);
    // Every step issues its two loads, also where step kt + 1 + GD lies past the last one (the last step's words are loaded
    // again and never looked at): the same number of loads separates every load from its use, so one counted wait serves
    // all steps on every path.
    issue_copy(greg[0], min(GD, ksteps - 1));
    step_barrier();
    for (int k0 = 0; k0 < ksteps; k0 += GD) {
#pragma unroll
      for (int j = 0; j < GD; ++j) {
        const int kt = k0 + j;
        // the loads of step kt+1 went out at the end of step kt-GD, followed by two loads in each of the GD-1 steps since
        wait_vmem_at_most<2 * (GD - 1)>();
        const int sl = (j + 1) % GD;
        store_w((kt & 1) ^ 1, greg[sl]);                      // (after the last step: a tile nobody reads)
        issue_copy(greg[sl], min(kt + 1 + GD, ksteps - 1));
        step_barrier();
      }
    }
    wait_vmem_at_most<0>();
    return;
  }
  if (producer) {
    uint4v greg[GD][2];       // centroids of the steps in flight; step kt uses slot kt % GD
    struct IdxGroup { uint4v q[GD / 2]; };   // raw indices of GD consecutive steps of this row: 8 bytes per step
    const unsigned char *irow = p.idx + (long long)o_w * p.stride;     // ksteps % GD == 0: every read stays in the row
    auto load_indices = [&](int k0, IdxGroup &g) {
#pragma unroll
      for (int i = 0; i < GD / 2; ++i) async_load16(g.q[i], irow + (long long)k0 * 8 + i * 16);
    };
    auto settle_group = [&](IdxGroup &g) {
#pragma unroll
      for (int i = 0; i < GD / 2; ++i) settle(g.q[i]);
    };
    auto pick = [&](const IdxGroup &g, int j) -> unsigned {     // this thread's index pair of step k0 + j
      const uint4v &v = g.q[j >> 1];
      return (j & 1) ? (w_half ? v.w : v.z) : (w_half ? v.y : v.x);
    };
    auto issue_gather = [&](uint4v (&g)[2], unsigned pair) {
      const unsigned i0 = min(pair & 0xFFFFu, (unsigned)p.k - 1u), i1 = min(pair >> 16, (unsigned)p.k - 1u);
      async_load16(g[0], p.cb, i0 * 16u);
      async_load16(g[1], p.cb, i1 * 16u);
    };
    auto store_w = [&](int buf, uint4v (&g)[2]) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        settle(g[j]);
        *reinterpret_cast<uint4v *>(reinterpret_cast<unsigned char *>(Ws + buf * BN * LDT) + x_slot((unsigned)w_row, (unsigned)(w_half * 2 + j))) = restore8(g[j], s_w, b_w, w_on);
      }
    };
    // Memory operations of a producer wave, in issue order: per step two centroid gathers (for step kt+1+GD), plus
    // GD/2 index loads at the start of every group of GD steps.  They complete in order.
    // Every step and every group issues its loads, also past the end of the row (the last group and the last step are
    // loaded again and never looked at), so the counted wait below is the same on every path.
    IdxGroup nxt, far;        // raw indices of the next group and of the group after it
    load_indices(0, far);
    load_indices(min(GD, ksteps - GD), nxt);
    wait_vmem_at_most<0>();
    settle_group(far); settle_group(nxt);
#pragma unroll
    for (int j = 0; j < GD; ++j) issue_gather(greg[j], pick(far, j));        // steps 0 .. GD-1
    wait_vmem_at_most<0>();
    store_w(0, greg[0]);
    issue_gather(greg[0], pick(nxt, 0));                                     // slot 0 now carries step GD
    step_barrier();
    for (int k0 = 0; k0 < ksteps; k0 += GD) {
      load_indices(min(k0 + 2 * GD, ksteps - GD), far);                      // first used at the last step of this group
#pragma unroll
      for (int j = 0; j < GD; ++j) {
        const int kt = k0 + j;                                    // ksteps % GD == 0: kt < ksteps
        // The centroids of step kt+1 (slot (j+1) % GD) went out at the end of step kt-GD, followed by two
        // gathers in each of the GD-1 steps since (index loads not counted: with them the bound only gets safer).
        wait_vmem_at_most<2 * (GD - 1)>();
        const int sl = (j + 1) % GD;
        store_w((kt & 1) ^ 1, greg[sl]);                          // (after the last step: a tile nobody reads)
        // the wait above also covers the index loads this gather needs (they are older than those centroids)
        if (j + 1 < GD) { settle_group(nxt); issue_gather(greg[sl], pick(nxt, j + 1)); }
        else { settle_group(far); issue_gather(greg[sl], pick(far, 0)); }
        step_barrier();
      }
      nxt = far;      // the group after next becomes the next group (its loads completed before the last wait above)
    }
    wait_vmem_at_most<0>();
    return;
  }

  // ---- consumers: each wave streams its own 64 token rows through its slice of the activation stages (no other
  // wave touches them, so only the wave's own counted wait stands between a copy and its use) and multiplies
  auto copy_x = [&](int kt) {
    const unsigned stage = (unsigned)(kt % NSX) * XSTAGE;
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
    const unsigned char *xs = Xs + (unsigned)(kt % NSX) * XSTAGE;
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

// Dense product for many tokens: Y = X * Wd^T with both operands FP16 in memory (Wd is what vq_dequant wrote).  The tiling
// above spends as many LDS cycles on operand reads as matrix-core cycles on the products (a wave's 64 x 128 block reads
// 0.75 KB per MFMA).  Here a workgroup of four waves owns 256 tokens x 256 channels, a wave 128 x 128: 16 operand reads
// feed 32 MFMAs (0.5 KB each), and the 256 accumulator registers that takes are there because a wave has its SIMD to
// itself (512 registers).  No producer waves: every wave starts the asynchronous global->LDS copies of its share of both
// tiles three steps ahead (same swizzled 64-byte rows as above).  With one wave per SIMD nothing else hides LDS latency,
// so the loop is pipelined by half steps: the operands of the next half step are read before the products of the current
// one are issued, and the barrier of a step sits between its two halves.
constexpr int DT = 256;       // tokens and channels per workgroup
constexpr int DNS = 4;        // stages of both tiles in LDS

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_dense256_kernel(const __half *__restrict__ X, long long ldx, int tokens,
                                                            const __half *__restrict__ Wd, long long ldw, int out_features, int in_features,
                                                            __half *__restrict__ Y, long long ldy) {
  constexpr unsigned TILE = DT * 64u;           // bytes of one tile of one stage: 256 rows x 32 halfs
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [DNS][X tile | W tile]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  const int n0 = blockIdx.x * DT, m0 = blockIdx.y * DT;
  const int ksteps = in_features / BK;
  __builtin_assume(ksteps > 0);        // (the launcher's layers have whole groups of eight steps: no path around the loop, whose last step collects the reads in flight)
  // range-checked against the end of the last row: rows past the matrix read zeros
  const __amdgpu_buffer_rsrc_t r_x = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<__half *>(X), 0, (unsigned)(((long long)(tokens - 1) * ldx + in_features) * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_w = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<__half *>(Wd), 0, (unsigned)(((long long)(out_features - 1) * ldw + in_features) * 2), 0x00020000);

  // this wave's share of a step's copies: pieces 4 wave .. 4 wave + 3 (16 rows x 64 bytes each) of both tiles
  // (byte offsets of the lane's four pieces at step 0, worked out once; a step adds 64 bytes)
  unsigned gx0[4], gw0[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned piece = (unsigned)(wave * 4 + i);
    const unsigned r = piece * 16u + ((unsigned)lane >> 2), cs = (unsigned)lane & 3u;   // LDS slot (r, cs) holds chunk cs ^ swz(r)
    const unsigned c = cs ^ swz(r);
    gx0[i] = (unsigned)(((long long)(m0 + (int)r) * ldx + c * 8) * 2);
    gw0[i] = (unsigned)(((long long)(n0 + (int)r) * ldw + c * 8) * 2);
  }
  auto copy_tiles = [&](int kt) {
    unsigned char *stage = smem + (unsigned)(kt % DNS) * (2u * TILE);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned piece = (unsigned)(wave * 4 + i);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(stage + piece * 1024u), 16, gx0[i] + (unsigned)kt * (BK * 2u), 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_w, (__attribute__((address_space(3))) void *)(stage + TILE + piece * 1024u), 16, gw0[i] + (unsigned)kt * (BK * 2u), 0, 0, 0);
    }
  };
  // operand addresses: row (block base + lane & 31), whose swizzle depends on the lane only, chunk ks / 8 + (lane >> 5):
  // one base per tile and half step, blocks 2 KB apart
  const unsigned sw = ((unsigned)(lane & 31) >> 2) & 3u;
  const unsigned xo[2] = {(unsigned)(wm + (lane & 31)) * 64u + ((((unsigned)lane >> 5) ^ sw) << 4),
                          (unsigned)(wm + (lane & 31)) * 64u + (((2u + ((unsigned)lane >> 5)) ^ sw) << 4)};
  const unsigned wo[2] = {TILE + (unsigned)(wn + (lane & 31)) * 64u + ((((unsigned)lane >> 5) ^ sw) << 4),
                          TILE + (unsigned)(wn + (lane & 31)) * 64u + (((2u + ((unsigned)lane >> 5)) ^ sw) << 4)};
  // The reads are issued from inline assembly, in program order, and waited for by count: left to itself the compiler
  // gives both sets of operands the same registers and so has to issue a set's reads after the other set's products.
  const unsigned lds0 = (unsigned)reinterpret_cast<size_t>((const __attribute__((address_space(3))) void *)smem);
  auto read_operands = [&](int kt, int ks, half8 (&af)[4], half8 (&bf)[4]) {
    const unsigned stage = lds0 + (unsigned)(kt % DNS) * (2u * TILE);
    unsigned xa = stage + xo[ks >> 4], wa = stage + wo[ks >> 4];
    asm volatile("" : "+v"(xa), "+v"(wa));      // both addresses in registers of their own before the first read goes out
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:2048\n\tds_read_b128 %2, %4 offset:4096\n\tds_read_b128 %3, %4 offset:6144"
                 : "=&v"(af[0]), "=&v"(af[1]), "=&v"(af[2]), "=&v"(af[3]) : "v"(xa) : "memory");
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:2048\n\tds_read_b128 %2, %4 offset:4096\n\tds_read_b128 %3, %4 offset:6144"
                 : "=&v"(bf[0]), "=&v"(bf[1]), "=&v"(bf[2]), "=&v"(bf[3]) : "v"(wa) : "memory");
  };
  auto operands_in = [&](half8 (&af)[4], half8 (&bf)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { settle(af[i]); settle(bf[i]); }
  };
  float16v acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
  auto multiply = [&](const half8 (&af)[4], const half8 (&bf)[4]) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[c], acc[a][c], 0, 0, 0);
  };

  // copies run DNS - 1 steps ahead; a wave waits for its own by count (eight per step), the barrier covers the others'
#pragma unroll
  for (int j = 0; j < DNS - 1; ++j)
    if (j < ksteps) copy_tiles(j);
  if (ksteps >= 3) wait_vmem_at_most<16>(); else wait_vmem_at_most<0>();
  step_barrier();
  half8 a0[4], b0[4], a1[4], b1[4];
  read_operands(0, 0, a0, b0);
  for (int kt = 0; kt < ksteps; ++kt) {
    if (kt + DNS - 1 < ksteps) copy_tiles(kt + DNS - 1);     // into the stage of step kt - 1: everyone has passed that step's barrier
    read_operands(kt, 16, a1, b1);
    asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");        // LDS reads return in order: all but the eight just issued are in
    operands_in(a0, b0);
    multiply(a0, b0);
    // this wave's copies of step kt + 1 went out at step kt - 2; the steps since have issued eight each
    if (kt + DNS - 1 < ksteps) wait_vmem_at_most<16>(); else wait_vmem_at_most<0>();
    step_barrier();                                           // (waits for the operand reads above as well: they are LDS traffic)
    // (statements from inline assembly keep their order: the reads of the next half step go out first, then the products
    // of this one, which the compiler may not move ahead of the statement that hands it their operands)
    read_operands(kt + 1 < ksteps ? kt + 1 : kt, 0, a0, b0);  // (past the end: any stage, never used; keeps the loop one straight line)
    operands_in(a1, b1);
    multiply(a1, b1);
    // the reads issued past the last step come in before the loop is left, while their registers are still the loop's
    // (the empty statements that follow the wait name the registers, so they stay the operands' until the wait is over)
    if (kt + 1 == ksteps) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      operands_in(a0, b0);
    }
  }

  // ---- store: lane holds channel (lane & 31) of block c and 16 token rows of block a.  Range-checked 2-byte buffer stores
  // with 32-bit offsets (256 64-bit addresses would not fit the registers): rows past the last token fall off the end of
  // the buffer, channels past the last one are sent there on purpose.
  const __amdgpu_buffer_rsrc_t r_y = __builtin_amdgcn_make_buffer_rsrc(Y, 0, (unsigned)(((long long)(tokens - 1) * ldy + out_features) * 2), 0x00020000);
  const unsigned ldy2 = (unsigned)ldy * 2u;
  const unsigned y_lane = (unsigned)(m0 + wm + 4 * (lane >> 5)) * ldy2 + (unsigned)(n0 + wn + (lane & 31)) * 2u;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool o_on = n0 + wn + c * 32 + (lane & 31) < out_features;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const unsigned off = y_lane + (unsigned)(a * 32 + 8 * (r >> 2) + (r & 3)) * ldy2 + (unsigned)(c * 64);
        const __half h = __float2half_rn(acc[a][c][r]);
        __builtin_amdgcn_raw_buffer_store_b16((short)__half_as_ushort(h), r_y, o_on ? off : 0xFFFFFFF0u, 0, 0);
      }
    }
    asm volatile("" ::: "memory");
  }
}

int launch_dense256(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, const __half *Wd, long long ldw,
                    hipStream_t s) {
  const unsigned lds = DNS * 2u * DT * 64u;
  VQ_ALLOW_FULL_LDS(gemm_dense256_kernel);
  if (((long long)(p.out_features - 1) * ldw + p.in_features) * 2 >= (1LL << 32)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  if (((long long)(tokens + DT) * ldy + p.out_features + DT) * 2 >= 0xFFFFFFF0LL) return VQ_ERR_UNSUPPORTED;
  const unsigned gx = (unsigned)((p.out_features + DT - 1) / DT), gy = (unsigned)((tokens + DT - 1) / DT);
  if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(gemm_dense256_kernel, dim3(gx, gy), dim3(256), lds, s, X, ldx, tokens, Wd, ldw, p.out_features, p.in_features, Y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int BM, bool DENSE>
int launch_fused(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, const __half *Wd, long long ldw,
                 hipStream_t s) {
  auto kernel = gemm_v8_kernel<BM, DENSE>;
  const unsigned lds = NSX * BM * 64u + 2u * BN * LDT * 2u;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned gx = (unsigned)((p.out_features + BN - 1) / BN), gy = (unsigned)((tokens + BM - 1) / BM);
  if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3(gx, gy), dim3((BM / 64 + 4) * 64), lds, s, p, X, ldx, tokens, Y, ldy, Wd, ldw);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

bool gemm_fused_applicable(const Params &p) {
  return p.orientation == 0 && p.v == 8 && p.bits == 16 && p.k_res == 0 && p.n_out == 0 && p.n_groups == 1 && p.in_features % (GD * BK) == 0;
}

// Wd == nullptr: W is restored on the fly.  Otherwise Wd is the FP16 matrix [out][ldw] that vq_dequant wrote
// (16-byte aligned rows) and the producers copy its tiles.
int launch_gemm_fused(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, const __half *Wd,
                      long long ldw, hipStream_t s) {
  if (((long long)(tokens - 1) * ldx + p.in_features) * 2 >= (1LL << 32)) return VQ_ERR_UNSUPPORTED;   // 32-bit buffer offsets
  if (Wd) {
    // The four-wave kernel with 256 x 256 tiles or the producer/consumer kernel with BM x 128 tiles (no gathers to amortise:
    // its tile height only has to fill the chip, out/128 x tokens/BM workgroups): whichever needs less time for its rounds of
    // one workgroup per compute unit.  A round of the other kernel costs about 1.5 / 0.8 / 0.55 of a 256 x 256 round at BM =
    // 512 / 256 / 128 (11008 x 4096: 86 tiles 127 against 143 us, 172 tiles 140 against 169 us; 4096 x 4096: 128 tiles 133
    // against 112 us; 8192 x 28672: 128 tiles 1001 against 696 us, 160 tiles 997 against 1223 us).  Switch dense=1 / =0:
    // always / never the four-wave kernel, for measurement and tests.
    const int force_dense = switches().dense;
    const long long tiles256 = (long long)((p.out_features + DT - 1) / DT) * ((tokens + DT - 1) / DT);
    const long long col_blocks = (p.out_features + BN - 1) / BN;
    const int bm = (col_blocks * ((tokens + 511) / 512) >= 200 ? 512 : col_blocks * ((tokens + 255) / 256) >= 200 ? 256 : 128);
    const long long cus = cu_count();
    const long long rounds256 = (tiles256 + cus - 1) / cus, rounds_bm = (col_blocks * ((tokens + bm - 1) / bm) + cus - 1) / cus;
    const long long cost_bm = rounds_bm * (bm == 512 ? 150 : bm == 256 ? 80 : 55);
    if (force_dense == 1 || (force_dense != 0 && rounds256 * 100 <= cost_bm)) {
      const int rc = launch_dense256(p, X, ldx, tokens, Y, ldy, Wd, ldw, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    if (bm == 512) return launch_fused<512, true>(p, X, ldx, tokens, Y, ldy, Wd, ldw, s);
    if (bm == 128) return launch_fused<128, true>(p, X, ldx, tokens, Y, ldy, Wd, ldw, s);
    return launch_fused<256, true>(p, X, ldx, tokens, Y, ldy, Wd, ldw, s);
  }
  const int bm = (tokens > 512 ? 512 : 256);
  if (bm == 512) return launch_fused<512, false>(p, X, ldx, tokens, Y, ldy, nullptr, 0, s);
  if (bm == 128) return launch_fused<128, false>(p, X, ldx, tokens, Y, ldy, nullptr, 0, s);
  return launch_fused<256, false>(p, X, ldx, tokens, Y, ldy, nullptr, 0, s);
}

}  // namespace vq
