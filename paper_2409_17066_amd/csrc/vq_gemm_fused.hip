// vq_gemm fast path for v = 8 with 16-bit indices (k up to 65536: the codebook is 1 MiB and lives in
// L2 / Infinity Cache, not in LDS), no residual, no outlier columns -- the paper's v=8 / k=65536 setting
// (App. "Impact of Vector Length").  Y = X * W^T with W restored on the fly; W never touches memory.
//
// A workgroup of 4 waves owns BM tokens x 128 output channels; wave w owns token rows [w*BM/4, ...) and
// all 128 channels, as (BM/128) x 4 MFMA 32x32x16 blocks.  Per 32-column step the workgroup gathers
// 128 x 4 centroids (16 bytes each, one per thread-vector) from the codebook, applies scale and bias,
// and writes the FP16 tile to LDS; the activation tile goes through LDS too.  Both tiles are double
// buffered, and the centroid gathers run GD steps ahead of their use, fed by an index tile that is
// staged in LDS every 16 steps.  The taller the token tile, the fewer times a centroid is gathered:
// each gather pulls a whole 128-byte line out of L2 for 16 useful bytes, which is what bounds this kernel.
#include "vq_common.hpp"
#include <cstdlib>

namespace vq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

constexpr int BN = 128;       // output channels per workgroup
constexpr int BK = 32;        // columns per step (4 vectors of 8)
constexpr int LDT = BK + 8;   // LDS row pitch in halfs (80 bytes: 8 consecutive rows fall in 8 different 16-byte bank groups)
constexpr int SS = 16;        // steps per index tile (16 * 4 = 64 indices = 128 bytes per row)
constexpr int GD = 3;         // gather distance in steps

__device__ __forceinline__ unsigned restore2(unsigned packed, float s, float b, bool lo_on, bool hi_on) {
  const unsigned short l = (unsigned short)(packed & 0xFFFFu), h = (unsigned short)(packed >> 16);
  const __half rl = lo_on ? restore(__half2float(__ushort_as_half(l)), s, b) : __ushort_as_half(0);
  const __half rh = hi_on ? restore(__half2float(__ushort_as_half(h)), s, b) : __ushort_as_half(0);
  return (unsigned)__half_as_ushort(rl) | ((unsigned)__half_as_ushort(rh) << 16);
}

// eight halfs -> scale * d + bias in binary32 -> eight halfs; elements >= valid become zero
__device__ __forceinline__ uint4v restore8(uint4v d, float s, float b, int valid) {
  uint4v out;
  out.x = restore2(d.x, s, b, 0 < valid, 1 < valid);
  out.y = restore2(d.y, s, b, 2 < valid, 3 < valid);
  out.z = restore2(d.z, s, b, 4 < valid, 5 < valid);
  out.w = restore2(d.w, s, b, 6 < valid, 7 < valid);
  return out;
}

template <int BM>
__global__ __launch_bounds__(256) void gemm_v8_kernel(Params p, const __half *__restrict__ X, long long ldx, int tokens,
                                                      __half *__restrict__ Y, long long ldy) {
  constexpr int MB = BM / 128;                 // 32-row MFMA blocks per wave along the tokens
  constexpr int XCH = BM * BK * 2 / 16 / 256;  // 16-byte activation chunks per thread per step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __half *Xs = reinterpret_cast<__half *>(smem);                                   // [2][BM][LDT]
  __half *Ws = Xs + 2 * BM * LDT;                                                  // [2][BN][LDT]
  unsigned short *Is = reinterpret_cast<unsigned short *>(Ws + 2 * BN * LDT);      // [2][BN][SS*4]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int ksteps = (p.in_features + BK - 1) / BK;

  // ---- this thread's share of the W tile: row w_row, vectors w_vec and w_vec + 1 of every step
  const int w_row = tid >> 1, w_vec = (tid & 1) * 2;
  const int o_w = min(n0 + w_row, p.out_features - 1);
  const float s_w = p.scale ? __half2float(p.scale[o_w]) : 1.0f;
  const float b_w = p.bias ? __half2float(p.bias[o_w]) : 0.0f;
  const uint4v *cb = reinterpret_cast<const uint4v *>(p.cb);

  // index tile loader: 128 rows x 128 bytes per 16 steps = 1024 chunks of 16 bytes, 4 per thread
  uint4v ireg[4];
  auto load_index_tile = [&](int ss) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * 256, row = c >> 3, part = c & 7;
      const int o = min(n0 + row, p.out_features - 1);
      const long long off = (long long)ss * (SS * 8) + part * 16;
      ireg[i] = (off + 16 <= p.stride) ? *reinterpret_cast<const uint4v *>(p.idx + (long long)o * p.stride + off)
                                       : uint4v{0u, 0u, 0u, 0u};
    }
  };
  auto store_index_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * 256, row = c >> 3, part = c & 7;
      *reinterpret_cast<uint4v *>(Is + (buf * BN + row) * (SS * 4) + part * 8) = ireg[i];
    }
  };

  // gather ring: centroids of steps kt+1 .. kt+GD in flight
  uint4v greg[GD][2];
  auto issue_gather = [&](int slot, int kt) {      // kt: step whose centroids to fetch; its index tile is in LDS
    const int buf = (kt / SS) & 1, col = (kt % SS) * 4 + w_vec;
    const unsigned pair = *reinterpret_cast<const unsigned *>(Is + (buf * BN + w_row) * (SS * 4) + col);
    const unsigned i0 = min(pair & 0xFFFFu, (unsigned)p.k - 1u), i1 = min(pair >> 16, (unsigned)p.k - 1u);
    greg[slot][0] = cb[i0];
    greg[slot][1] = cb[i1];
  };

  // activation tile loader
  uint4v xreg[XCH];
  auto load_x = [&](int kt) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int c = tid + i * 256, row = c >> 2, col = (c & 3) * 8;
      const int t = m0 + row, cc = kt * BK + col;
      uint4v v = {0u, 0u, 0u, 0u};
      if (t < tokens && cc < p.in_features) {
        const __half *src = X + (long long)t * ldx + cc;
        if (cc + 8 <= p.in_features) {
          v = *reinterpret_cast<const uint4v *>(src);
        } else {
          __half tmp[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) tmp[j] = (cc + j < p.in_features) ? src[j] : __ushort_as_half(0);
          v = *reinterpret_cast<uint4v *>(tmp);
        }
      }
      xreg[i] = v;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int c = tid + i * 256, row = c >> 2, col = (c & 3) * 8;
      *reinterpret_cast<uint4v *>(Xs + (buf * BM + row) * LDT + col) = xreg[i];
    }
  };
  auto store_w = [&](int buf, int slot, int kt) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c0 = (kt * 4 + w_vec + j) * 8;                       // first column of this vector
      const int valid = (n0 + w_row < p.out_features) ? max(0, min(8, p.in_features - c0)) : 0;
      const uint4v w = restore8(greg[slot][j], s_w, b_w, valid);
      *reinterpret_cast<uint4v *>(Ws + (buf * BN + w_row) * LDT + (w_vec + j) * 8) = w;
    }
  };

  float16v acc[MB][4];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;

  // ---- prologue: index tile 0 (and 1), activations of step 0, centroids of steps 0 .. GD-1
  load_index_tile(0);
  load_x(0);
  store_index_tile(0);
  __syncthreads();
  if (SS < ksteps) load_index_tile(1);
  {
    // step 0's centroids are needed at once: fetch them through slot 0, then refill the ring for steps 1 .. GD
    issue_gather(0, 0);
    store_x(0);
    store_w(0, 0, 0);
  }
#pragma unroll
  for (int g = 0; g < GD; ++g)
    if (1 + g < ksteps) issue_gather(g, 1 + g);      // slot g holds step 1 + g  (step kt lives in slot (kt - 1) % GD)
  __syncthreads();

  const int wm = wave * (BM / 4);
  for (int kt = 0; kt < ksteps; ++kt) {
    const int cur = kt & 1, nxt = cur ^ 1;
    const bool more = kt + 1 < ksteps;
    if (more) load_x(kt + 1);
    // a new index tile becomes current every SS steps: tile (kt+1+GD)/SS must be in LDS before its gathers go out
    // ---- MFMA on the current buffers
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      half8 af[MB], bf[4];
#pragma unroll
      for (int a = 0; a < MB; ++a)
        af[a] = *reinterpret_cast<const half8 *>(Xs + (cur * BM + wm + a * 32 + (lane & 31)) * LDT + ks + (lane >> 5) * 8);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        bf[c] = *reinterpret_cast<const half8 *>(Ws + (cur * BN + c * 32 + (lane & 31)) * LDT + ks + (lane >> 5) * 8);
#pragma unroll
      for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[c], acc[a][c], 0, 0, 0);
    }
    if (more) {
      store_x(nxt);
      store_w(nxt, kt % GD, kt + 1);                 // step kt+1 lives in slot kt % GD
    }
    // index tile hand-over: when step kt+1+GD starts a new tile, that tile must already sit in LDS
    const int g_next = kt + 1 + GD;                  // step whose gather is issued after this barrier
    if (g_next % SS == 0 && g_next < ksteps) store_index_tile((g_next / SS) & 1);
    __syncthreads();
    if (g_next % SS == 0 && g_next + SS < ksteps) load_index_tile(g_next / SS + 1);
    if (g_next < ksteps) issue_gather(kt % GD, g_next);
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

template <int BM>
int launch_fused(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, hipStream_t s) {
  static bool configured = false;
  auto kernel = gemm_v8_kernel<BM>;
  const unsigned lds = (2 * BM * LDT + 2 * BN * LDT) * 2 + 2 * BN * SS * 4 * 2;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return VQ_ERR_HIP;
    configured = true;
  }
  const unsigned gx = (unsigned)((p.out_features + BN - 1) / BN), gy = (unsigned)((tokens + BM - 1) / BM);
  if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3(gx, gy), dim3(256), lds, s, p, X, ldx, tokens, Y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

bool gemm_fused_applicable(const Params &p) {
  return p.v == 8 && p.bits == 16 && p.k_res == 0 && p.n_out == 0;
}

int launch_gemm_fused(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, hipStream_t s) {
  static const int force_bm = [] { const char *e = getenv("VQ_GEMM_BM"); return e ? atoi(e) : 0; }();
  const int bm = force_bm ? force_bm : (tokens > 512 ? 512 : 256);
  if (bm == 512) return launch_fused<512>(p, X, ldx, tokens, Y, ldy, s);
  if (bm == 128) return launch_fused<128>(p, X, ldx, tokens, Y, ldy, s);
  return launch_fused<256>(p, X, ldx, tokens, Y, ldy, s);
}

}  // namespace vq
