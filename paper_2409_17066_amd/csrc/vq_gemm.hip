// vq_gemm: prompt-phase product Y = X * W^T with W restored on the fly into LDS tiles that feed the
// FP16 matrix cores (paper App. "Our Dequantization Implementation", first phase, but without ever
// writing W to memory).  Accumulation in binary32, FP16 result.
#include "vq_common.hpp"
#include <cstdlib>

namespace vq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 128;        // tokens per workgroup tile
constexpr int BN = 128;        // output channels per workgroup tile
constexpr int BK = 32;         // input columns per step
constexpr int LDT = BK + 8;    // LDS row pitch in halfs: 80 bytes, so 8 consecutive rows hit 8 different 16-byte bank groups

// Restore columns [c0, c0+n) of row o into dst (LDS), zero past in_features.  Any layer shape.
__device__ __forceinline__ void restore_run_generic(const Params &p, int o, int c0, int n, float s, float b, __half *dst) {
  if (p.orientation == 1) {               // vectors down the output dimension: every column of the run is a vector of its own
    for (int t = 0; t < n; ++t) {
      const int c = c0 + t;
      if (o >= p.out_features || c >= p.in_features) { dst[t] = __float2half_rn(0.0f); continue; }
      float d;
      if (c < p.n_out) {
        const int sq = o / p.v_out;
        unsigned i = min(load_index(p.idx_out + (long long)sq * p.stride_out, c, p.bits_out), (unsigned)p.k_out - 1u);
        d = __half2float(p.cb_out[(long long)i * p.v_out + (o - sq * p.v_out)]);
      } else {
        const int pos = c - p.n_out, sp = o / p.v, j = o - sp * p.v;
        const long long group = pos / p.Pg;
        unsigned i = min(load_index(p.idx + (long long)sp * p.stride, pos, p.bits), (unsigned)p.k - 1u);
        d = __half2float(p.cb[(group * p.k + i) * p.v + j]);
        if (p.k_res) {
          unsigned r = min(load_index(p.idx_res + (long long)sp * p.stride_res, pos, p.bits_res), (unsigned)p.k_res - 1u);
          d = __fadd_rn(d, __half2float(p.cb_res[(group * p.k_res + r) * p.v + j]));
        }
      }
      dst[t] = restore(d, s, b);
    }
    return;
  }
  int c = c0;
  int j = 0, len = 0;                     // position inside / length of the current vector
  const __half *e = nullptr, *er = nullptr;
  for (int t = 0; t < n; ++t, ++c) {
    if (o >= p.out_features || c >= p.in_features) { dst[t] = __float2half_rn(0.0f); continue; }
    if (j >= len) {                       // fetch the vector that holds column c
      er = nullptr;
      if (c < p.n_out) {
        const int q = c / p.v_out;
        j = c - q * p.v_out; len = p.v_out;
        unsigned i = min(load_index(p.idx_out + (long long)o * p.stride_out, q, p.bits_out), (unsigned)p.k_out - 1u);
        e = p.cb_out + (long long)i * p.v_out;
      } else {
        const int cc = c - p.n_out;
        const int pp = cc / p.v;
        j = cc - pp * p.v; len = p.v;
        unsigned i = min(load_index(p.idx + (long long)o * p.stride, pp, p.bits), (unsigned)p.k - 1u);
        const long long group = pp / p.Pg;
        e = p.cb + (group * p.k + i) * p.v;
        if (p.k_res) {
          unsigned r = min(load_index(p.idx_res + (long long)o * p.stride_res, pp, p.bits_res), (unsigned)p.k_res - 1u);
          er = p.cb_res + (group * p.k_res + r) * p.v;
        }
      }
    }
    float d = __half2float(e[j]);
    if (er) d = __fadd_rn(d, __half2float(er[j]));
    dst[t] = restore(d, s, b);
    ++j;
    if (c + 1 == p.n_out) j = len;        // the outlier region ends: force a fetch from the main stream
  }
}

// 256 threads = 4 waves in a 2x2 arrangement; each wave owns a 64x64 block of the 128x128 tile as
// 2x2 MFMA 32x32x16 blocks.  Operand layout of v_mfma_f32_32x32x16_f16: lane l supplies row/column
// (l & 31) and the 8 consecutive k values starting at 8*(l >> 5); it receives column (l & 31) and,
// in result register r, row 8*(r >> 2) + 4*(l >> 5) + (r & 3).
__global__ __launch_bounds__(256) void gemm_tile_kernel(Params p, const __half *__restrict__ X, long long ldx, int tokens,
                                                        __half *__restrict__ Y, long long ldy) {
  __shared__ __attribute__((aligned(16))) __half Xs[BM * LDT];
  __shared__ __attribute__((aligned(16))) __half Ws[BN * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;

  float16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;

  // W restore assignment: thread -> (row tid/2, 16 columns)
  const int w_row = tid >> 1, w_col = (tid & 1) * 16;
  const int o_w = n0 + w_row;
  const float s_w = (p.scale && o_w < p.out_features) ? __half2float(p.scale[o_w]) : 1.0f;
  const float b_w = (p.bias && o_w < p.out_features) ? __half2float(p.bias[o_w]) : 0.0f;

  for (int k0 = 0; k0 < p.in_features; k0 += BK) {
    // X tile: 128 rows x 4 chunks of 8 halfs; thread takes chunks tid and tid+256
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int chunk = tid + h * 256;
      const int row = chunk >> 2, col = (chunk & 3) * 8;
      const int t = m0 + row, c = k0 + col;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (t < tokens && p.perm) {                       // permuted column order: stored column c + i meets X[t][perm[c + i]]
        __half tmp[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int u = c + i < p.in_features ? p.perm[c + i] : -1;
          tmp[i] = (unsigned)u < (unsigned)p.in_features ? X[(long long)t * ldx + u] : __float2half_rn(0.0f);
        }
        val = *reinterpret_cast<uint4 *>(tmp);
      } else if (t < tokens) {
        const __half *src = X + (long long)t * ldx + c;
        if (c + 8 <= p.in_features) {
          val = *reinterpret_cast<const uint4 *>(src);
        } else if (c < p.in_features) {
          __half tmp[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) tmp[i] = (c + i < p.in_features) ? src[i] : __float2half_rn(0.0f);
          val = *reinterpret_cast<uint4 *>(tmp);
        }
      }
      *reinterpret_cast<uint4 *>(&Xs[row * LDT + col]) = val;
    }
    restore_run_generic(p, o_w, k0 + w_col, 16, s_w, b_w, &Ws[w_row * LDT + w_col]);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      half8 af[2], bf[2];
#pragma unroll
      for (int a = 0; a < 2; ++a)
        af[a] = *reinterpret_cast<const half8 *>(&Xs[(wm + a * 32 + (lane & 31)) * LDT + ks + (lane >> 5) * 8]);
#pragma unroll
      for (int c = 0; c < 2; ++c)
        bf[c] = *reinterpret_cast<const half8 *>(&Ws[(wn + c * 32 + (lane & 31)) * LDT + ks + (lane >> 5) * 8]);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
          acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[c], acc[a][c], 0, 0, 0);
    }
    __syncthreads();
  }

#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int o = n0 + wn + c * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = m0 + wm + a * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (t < tokens && o < p.out_features) Y[(long long)t * ldy + o] = __float2half_rn(acc[a][c][r]);
      }
    }
}

size_t gemm_workspace_bytes(const Params &, int) { return 0; }

// Bytes of the FP16 weight matrix [out][in] that the two-step route below writes; 0 when that route does not apply.
// For a layer with a permuted column order (Sec. 3.2.3) the activations, gathered into stored order, come first: tokens
// rows of in_features rounded up to 8 halfs, the whole rounded up to 256 bytes; every kernel then works in stored order.
static size_t permuted_x_bytes(const Params &p, int tokens) { return ((size_t)tokens * (size_t)((p.in_features + 7) & ~7) * sizeof(__half) + 255) / 256 * 256; }

size_t gemm_fast_workspace_bytes(const Params &p, int tokens) {
  const size_t head = p.perm ? permuted_x_bytes(p, tokens) : 0;
  if (p.in_features % 256 != 0) return head;                 // the dense kernel walks the columns in groups of 8 x 32
  return head + (size_t)p.out_features * (size_t)p.in_features * sizeof(__half);
}

bool gemm_fused_applicable(const Params &p);
bool gemv_has_lds_kernel(const Params &p, const __half *x, long long ldx);
bool gemm_v6_applicable(const Params &p);
int launch_gemm_v6(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, hipStream_t s);
int launch_gemm_fused(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy, const __half *Wd,
                      long long ldw, hipStream_t s);

// Routes, in this order:
//  1. a workspace of gemm_fast_workspace_bytes() is there: vq_dequant into it, then the MFMA kernel with plain
//     tile copies as its producers.  This is the paper's prompt-phase scheme (restore to FP16, then a dense
//     product); on gfx950 it beats restoring on the fly because every 16-byte centroid gather drags a 128-byte
//     line out of L2 and a tile is gathered again for every token tile, while the restored matrix is read in
//     full lines.  Any layer the library can dequantize qualifies (in_features a multiple of 256).
//  2. v = 8 / 16-bit indices: restore on the fly inside the MFMA kernel (no workspace, W never in memory).
//  3. v = 6 / 12-bit indices without outlier columns or groups: restore on the fly from tables in LDS (vq_gemm_v6.hip), when
//     there is no workspace and more than 64 tokens (fewer go through vq_gemv's kernels, sixteen rows at a time).
//  4. the generic tile kernel.
// Switch gemm=g forces 4, =f skips 1, =w takes 1 whenever a workspace is there, =6 takes 3 for every token count
// (measurement and tests).
int launch_gemm(const Params &p, const __half *X, long long ldx, int tokens, __half *Y, long long ldy,
                void *workspace, size_t workspace_bytes, hipStream_t s) {
  if (p.perm && tokens <= 65535 && workspace && workspace_bytes >= permuted_x_bytes(p, tokens) && (reinterpret_cast<uintptr_t>(workspace) & 15) == 0 &&
      switches().gemm != 'g') {
    // room for the gathered activations: from here on the layer is an unpermuted one (the rest of the workspace is its own)
    Params q = p;
    q.perm = nullptr;
    __half *Xp = static_cast<__half *>(workspace);
    const long long ldxp = (p.in_features + 7) & ~7;
    const int rc = launch_gather_cols(X, ldx, tokens, p.in_features, p.perm, Xp, ldxp, s);
    if (rc != VQ_OK) return rc;
    const size_t head = permuted_x_bytes(p, tokens);
    return launch_gemm(q, Xp, ldxp, tokens, Y, ldy, static_cast<unsigned char *>(workspace) + head, workspace_bytes - head, s);
  }
  if (p.perm) {                                            // no room: the generic tile kernel looks every activation up
    const unsigned gx = (unsigned)((p.out_features + BN - 1) / BN), gy = (unsigned)((tokens + BM - 1) / BM);
    if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(gemm_tile_kernel, dim3(gx, gy), dim3(256), 0, s, p, X, ldx, tokens, Y, ldy);
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  const char forced = switches().gemm;
  const size_t fast = gemm_fast_workspace_bytes(p, tokens);
  // measured on the 8192 x 8192 v=8 layer: up to 512 tokens restoring on the fly is still ahead (167 vs 184 us), from
  // 1024 tokens on the restored matrix wins (215 vs 267 us, 365 vs 407 us at 2048); gemm=w takes it always
  const bool worth_it = forced == 'w' || !gemm_fused_applicable(p) || tokens > 512;
  const bool have_ws = fast && workspace && workspace_bytes >= fast && (reinterpret_cast<uintptr_t>(workspace) & 15) == 0;
  // Layers that only the generic tile kernel would take (no workspace and not the v = 8 layout of the fused kernel), and
  // token counts too small for the restored-matrix route to fill the chip with tiles, go through vq_gemv's kernels sixteen
  // rows at a time where that was measured faster.  Row-wise v = 6 layers (the matrix-core GEMV, whose sixteen rows cost
  // little more than one): always without a workspace, up to 96 tokens with one -- 4096 x 4096, 64 tokens 42 us against
  // 83 us with a workspace and 667 us without; 512 tokens without a workspace 322 against 700 us.  The other layers with
  // a specialised GEMV kernel (v = 8; orientation 1), whose cost grows faster with the rows: only without a workspace and
  // up to 128 tokens (v = 8, k = 65536 with a residual, 64 tokens: 191 against 848 us; 512 tokens would be 1480 against 880).
  // gemm=r: always.
  // (the on-the-fly kernel for v = 6 from 65 tokens on; up to 128 tokens only where its 128 x 128 tiles give 80 workgroups --
  // 8192 x 28672 at 128 tokens: 64 workgroups, 612 us against 515 us for eight passes of the GEMV)
  const bool v6_tiles_fill = tokens > 128 || (long long)((p.out_features + 127) / 128) * ((tokens + 127) / 128) >= 80;
  if (gemm_v6_applicable(p) && (forced == '6' || (forced == '\0' && !have_ws && tokens > 64 && v6_tiles_fill))) {
    const int rc = launch_gemm_v6(p, X, ldx, tokens, Y, ldy, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  const bool rows_cheap = p.orientation == 0 && p.v == 6;
  // (layers of the LDS-table decode kernels, whose only tile kernel is the generic one -- about 1 ms for any token count up to
  // 128 on 11008 x 4096 -- and whose decode kernels take four rows a launch: up to 32 tokens, 4 with a workspace; v = 12 with two
  // tables, 16 tokens: 239 against 987 us, with a workspace 164 us)
  const bool lds_rows = forced == '\0' && !gemm_fused_applicable(p) && !gemm_v6_applicable(p) && gemv_has_lds_kernel(p, X, ldx) &&
                        tokens <= (have_ws ? 4 : 32);
  if (forced == 'r' || lds_rows ||
      (forced == '\0' && !gemm_fused_applicable(p) && gemv_has_fast_kernel(p, X, ldx) &&
       (rows_cheap ? (!have_ws || tokens <= 96) : (!have_ws && tokens <= 128)))) {
    for (int t0 = 0; t0 < tokens; t0 += 16) {
      const int rc = launch_gemv(p, X + (long long)t0 * ldx, ldx, tokens - t0 < 16 ? tokens - t0 : 16, Y + (long long)t0 * ldy, ldy, s);
      if (rc != VQ_OK) return rc;
    }
    return VQ_OK;
  }
  if (forced != 'g' && forced != 'f' && worth_it && fast && workspace && workspace_bytes >= fast &&
      (reinterpret_cast<uintptr_t>(workspace) & 15) == 0) {
    __half *Wd = static_cast<__half *>(workspace);
    int rc = launch_dequant(p, Wd, p.in_features, s);
    if (rc == VQ_OK) rc = launch_gemm_fused(p, X, ldx, tokens, Y, ldy, Wd, p.in_features, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  if (forced != 'g' && gemm_fused_applicable(p)) {
    const int rc = launch_gemm_fused(p, X, ldx, tokens, Y, ldy, nullptr, 0, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  const unsigned gx = (unsigned)((p.out_features + BN - 1) / BN), gy = (unsigned)((tokens + BM - 1) / BM);
  if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(gemm_tile_kernel, dim3(gx, gy), dim3(256), 0, s, p, X, ldx, tokens, Y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace vq
