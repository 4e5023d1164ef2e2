// vq_gemv for layers with vectors of eight components (Sec. 3.1; the v = 8, k = 65536 setting of the tables of 2-bit
// parameters in App. "Parameter Description"), one to eight activation rows per launch: the decode-phase product of
// App. "Our Dequantization Implementation".
//
// A table of 65536 x 8 binary16 values is 1 MB: it does not fit LDS, so the entries are gathered from global memory
// (the table stays in L2).  What makes that fast is that an entry is exactly 16 bytes and 16-byte aligned -- one
// load per vector -- and that the 8- or 16-bit indices need no bit extraction.  One wave per output row; in a step
// its 64 lanes take 4 x 64 consecutive vectors of the row: four independent chains of index load -> gather ->
// multiply-add per lane, all addresses clamped into the row instead of branched around (a lane past the row's end
// repeats the last vector and adds nothing), so that the loads of a step are issued together.
//   y[t][o] = fp16(scale[o] * sum_c d[o][c] * x[t][c] + bias[o] * sum_c x[t][c]),  d = C[idx] (+ C_res[idx_res]),
// products and sums in binary32 (v_dot2_f32_f16).
#include "vq_common.hpp"

namespace vq {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));

// (The operands stay vectors of halves from the load to the instruction: this compiler turned bit casts of the dwords of
// a four-dword load into four uses of the first dword.)
__device__ __forceinline__ float dot8(const half8v a, const half8v b, float c) {
  c = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), c, false);
  c = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), c, false);
  c = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), c, false);
  c = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), c, false);
  return c;
}

template <int BYTES> __device__ __forceinline__ unsigned load_idx(const uint8_t *row, int pv) {
  return BYTES == 2 ? (unsigned)reinterpret_cast<const unsigned short *>(row)[pv] : (unsigned)row[pv];
}

constexpr int WAVES = 4, CHAINS = 4;

// B rows of x; IB / RB: bytes per main / residual index (RB = 0: no residual table); R output rows per wave.  With
// R = 2 a wave walks two rows at once, CHAINS / 2 chains each: as many gathers in flight, but every activation it
// loads serves both rows -- x is otherwise re-read once per output row, which is what four and more tokens pay for.
template <int B, int IB, int RB, int R>
__global__ __launch_bounds__(WAVES * 64) void gemv_v8_kernel(Params p, const __half *__restrict__ x, long long ldx, __half *__restrict__ y,
                                                             long long ldy) {
  constexpr int NC = CHAINS / R;
  const int lane = threadIdx.x & 63;
  const int o0 = (blockIdx.x * WAVES + (threadIdx.x >> 6)) * R;
  if (o0 >= p.out_features) return;
  const uint8_t *irow[R], *rrow[R];
#pragma unroll
  for (int q = 0; q < R; ++q) {                   // a row past the last one repeats the last and is not stored
    const int o = min(o0 + q, p.out_features - 1);
    irow[q] = p.idx + (long long)o * p.stride;
    rrow[q] = RB ? p.idx_res + (long long)o * p.stride_res : nullptr;
  }
  const half8v ones = {1, 1, 1, 1, 1, 1, 1, 1}, zeros = {0, 0, 0, 0, 0, 0, 0, 0};
  const bool with_bias = p.bias != nullptr;
  float acc[R][B], xs[B];
#pragma unroll
  for (int t = 0; t < B; ++t) {
    xs[t] = 0.0f;
#pragma unroll
    for (int q = 0; q < R; ++q) acc[q][t] = 0.0f;
  }
  for (int base = 0; base < p.P; base += NC * 64) {
    half8v e[NC][R], f[NC][R];
    int pvc[NC];
    bool on[NC];
    unsigned i[NC][R], r[NC][R];
#pragma unroll
    for (int u = 0; u < NC; ++u) {                // the step's index loads first, all of them ...
      const int pv = base + u * 64 + lane;
      on[u] = pv < p.P;
      pvc[u] = on[u] ? pv : p.P - 1;
#pragma unroll
      for (int q = 0; q < R; ++q) {
        i[u][q] = load_idx<IB>(irow[q], pvc[u]);
        if (RB) r[u][q] = load_idx<RB ? RB : 1>(rrow[q], pvc[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < NC; ++u) {                // ... then its gathers (indices past a short table are clamped into it)
      const long long group = p.n_groups > 1 ? pvc[u] / p.Pg : 0;
#pragma unroll
      for (int q = 0; q < R; ++q) {
        e[u][q] = *reinterpret_cast<const half8v *>(p.cb + (group * p.k + min(i[u][q], (unsigned)p.k - 1u)) * 8);
        if (RB) f[u][q] = *reinterpret_cast<const half8v *>(p.cb_res + (group * p.k_res + min(r[u][q], (unsigned)p.k_res - 1u)) * 8);
      }
    }
#pragma unroll
    for (int u = 0; u < NC; ++u) {
#pragma unroll
      for (int t = 0; t < B; ++t) {
        half8v xv = *reinterpret_cast<const half8v *>(x + (long long)t * ldx + (long long)pvc[u] * 8);
        if (!on[u]) xv = zeros;
#pragma unroll
        for (int q = 0; q < R; ++q) {
          acc[q][t] = dot8(e[u][q], xv, acc[q][t]);
          if (RB) acc[q][t] = dot8(f[u][q], xv, acc[q][t]);
        }
        if (with_bias) xs[t] = dot8(ones, xv, xs[t]);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < B; ++t) {
    const float xsum = with_bias ? wave_sum(xs[t]) : 0.0f;
#pragma unroll
    for (int q = 0; q < R; ++q) {
      const float sum = wave_sum(acc[q][t]);
      const int o = o0 + q;
      if (lane == 0 && o < p.out_features) {
        const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = with_bias ? __half2float(p.bias[o]) : 0.0f;
        y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(sc, sum, bi * xsum));
      }
    }
  }
}

template <int B, int IB, int RB, int R>
int launch_rows(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  hipLaunchKernelGGL((gemv_v8_kernel<B, IB, RB, R>), dim3((unsigned)((p.out_features + WAVES * R - 1) / (WAVES * R))), dim3(WAVES * 64), 0, s, p, x, ldx,
                     y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// Two rows per wave from four tokens and 8192 columns on, where the re-reading of x weighs more than the halved number of
// waves (batch 8: 8192 x 8192 74 -> 66 us, 8192 x 28672 242 -> 203 us; 4096 x 4096 would go from 22.3 to 23.5 us).
template <int B, int IB, int RB>
int launch_one(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  if (B >= 4 && p.in_features >= 8192) return launch_rows<B, IB, RB, (B >= 4 ? 2 : 1)>(p, x, ldx, y, ldy, s);
  return launch_rows<B, IB, RB, 1>(p, x, ldx, y, ldy, s);
}

// The same for layers stored with vectors down the output dimension (Sec. 3.1, Algorithm 1: W[8s + j][c] =
// C[idx[s][c]][j]): one workgroup per index stream, i.e. per 8 output rows; its DWAVES waves take contiguous quarters of
// the columns, a lane keeps 8 sums per token (the entry's components as binary32, times the lane's activation), the
// waves' sums meet in LDS.
constexpr int DWAVES = 4;

template <int B, int IB, int RB>
__global__ __launch_bounds__(DWAVES * 64) void gemv_v8_down_kernel(Params p, const __half *__restrict__ x, long long ldx, __half *__restrict__ y,
                                                                   long long ldy) {
  __shared__ float red[DWAVES][B][9];            // per wave and token: 8 row sums and the activation sum
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int stream = blockIdx.x;                 // the grid has p.S workgroups
  const uint8_t *irow = p.idx + (long long)stream * p.stride;
  const uint8_t *rrow = RB ? p.idx_res + (long long)stream * p.stride_res : nullptr;
  const bool with_bias = p.bias != nullptr;
  const int per = (p.P + DWAVES * CHAINS * 64 - 1) / (DWAVES * CHAINS * 64) * (CHAINS * 64);   // columns per wave, whole steps
  const int c0 = min(p.P, wv * per), c1 = min(p.P, c0 + per);
  float acc[B][8], xs[B];
#pragma unroll
  for (int t = 0; t < B; ++t) {
    xs[t] = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[t][j] = 0.0f;
  }
  for (int base = c0; base < c1; base += CHAINS * 64) {
    half8v e[CHAINS], f[CHAINS];
    int cc[CHAINS];
    bool on[CHAINS];
    unsigned i[CHAINS], r[CHAINS];
#pragma unroll
    for (int u = 0; u < CHAINS; ++u) {
      const int c = base + u * 64 + lane;
      on[u] = c < c1;
      cc[u] = on[u] ? c : c1 - 1;                // c1 > c0 inside the loop: a column of this wave
      i[u] = load_idx<IB>(irow, cc[u]);
      if (RB) r[u] = load_idx<RB ? RB : 1>(rrow, cc[u]);
    }
#pragma unroll
    for (int u = 0; u < CHAINS; ++u) {
      const long long group = p.n_groups > 1 ? cc[u] / p.Pg : 0;
      e[u] = *reinterpret_cast<const half8v *>(p.cb + (group * p.k + min(i[u], (unsigned)p.k - 1u)) * 8);
      if (RB) f[u] = *reinterpret_cast<const half8v *>(p.cb_res + (group * p.k_res + min(r[u], (unsigned)p.k_res - 1u)) * 8);
    }
#pragma unroll
    for (int u = 0; u < CHAINS; ++u) {
      float d[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) d[j] = RB ? (float)e[u][j] + (float)f[u][j] : (float)e[u][j];
#pragma unroll
      for (int t = 0; t < B; ++t) {
        const float xv = on[u] ? __half2float(x[(long long)t * ldx + cc[u]]) : 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[t][j] = __fmaf_rn(d[j], xv, acc[t][j]);
        xs[t] += xv;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < B; ++t) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float sum = wave_sum(acc[t][j]);
      if (lane == 0) red[wv][t][j] = sum;
    }
    const float xsum = wave_sum(xs[t]);
    if (lane == 0) red[wv][t][8] = xsum;
  }
  __syncthreads();
  if ((int)threadIdx.x < B * 8) {
    const int t = (int)threadIdx.x >> 3, j = (int)threadIdx.x & 7, o = stream * 8 + j;
    float sum = 0.0f, xsum = 0.0f;
#pragma unroll
    for (int w = 0; w < DWAVES; ++w) { sum += red[w][t][j]; xsum += red[w][t][8]; }
    if (o < p.out_features) {
      const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = with_bias ? __half2float(p.bias[o]) : 0.0f;
      y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(sc, sum, bi * xsum));
    }
  }
}

template <int B, int IB, int RB>
int launch_one_down(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  hipLaunchKernelGGL((gemv_v8_down_kernel<B, IB, RB>), dim3((unsigned)p.S), dim3(DWAVES * 64), 0, s, p, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

int index_bytes(int bits) { return bits == 8 ? 1 : bits == 16 ? 2 : 0; }

}  // namespace

// Row-wise layers of 8-component vectors with byte-aligned indices, no outlier columns, whole vectors only; x rows
// 16-byte aligned.  (The tables are 16-byte aligned by the descriptor's rules; an index row by its 16-byte stride.)
bool gemv_v8_applicable(const Params &p, const __half *x, long long ldx) {
  if (p.orientation != 0 || p.v != 8 || p.Q != 0 || p.n_out != 0 || (p.in_features & 7)) return false;
  if (!index_bytes(p.bits) || (p.k_res && !index_bytes(p.bits_res))) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (ldx & 7)) return false;
  if ((reinterpret_cast<uintptr_t>(p.cb) & 15) || (p.k_res && (reinterpret_cast<uintptr_t>(p.cb_res) & 15))) return false;
  return (p.stride & 1) == 0 && (!p.k_res || (p.stride_res & 1) == 0);
}

// batch = 1, 2, 4 or 8 rows of x.  The caller has checked gemv_v8_applicable().
int launch_gemv_v8(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  const int ib = index_bytes(p.bits), rb = p.k_res ? index_bytes(p.bits_res) : 0;
#define VQ_CASE(BB, IB, RB) if (batch == BB && ib == IB && rb == RB) return launch_one<BB, IB, RB>(p, x, ldx, y, ldy, s);
#define VQ_CASES(BB) VQ_CASE(BB, 2, 0) VQ_CASE(BB, 2, 2) VQ_CASE(BB, 2, 1) VQ_CASE(BB, 1, 0) VQ_CASE(BB, 1, 1) VQ_CASE(BB, 1, 2)
  VQ_CASES(1) VQ_CASES(2) VQ_CASES(4) VQ_CASES(8)
#undef VQ_CASES
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

// Layers of 8-component vectors down the output dimension, byte-aligned indices, no outlier columns.
bool gemv_v8_down_applicable(const Params &p) {
  if (p.orientation != 1 || p.v != 8 || p.Q != 0 || p.n_out != 0 || p.S < 1 || p.P < 1) return false;
  if (!index_bytes(p.bits) || (p.k_res && !index_bytes(p.bits_res))) return false;
  if ((reinterpret_cast<uintptr_t>(p.cb) & 15) || (p.k_res && (reinterpret_cast<uintptr_t>(p.cb_res) & 15))) return false;
  return (p.stride & 1) == 0 && (!p.k_res || (p.stride_res & 1) == 0);
}

// batch = 1, 2 or 4 rows of x.  The caller has checked gemv_v8_down_applicable().
int launch_gemv_v8_down(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  const int ib = index_bytes(p.bits), rb = p.k_res ? index_bytes(p.bits_res) : 0;
#define VQ_CASE(BB, IB, RB) if (batch == BB && ib == IB && rb == RB) return launch_one_down<BB, IB, RB>(p, x, ldx, y, ldy, s);
#define VQ_CASES(BB) VQ_CASE(BB, 2, 0) VQ_CASE(BB, 2, 2) VQ_CASE(BB, 2, 1) VQ_CASE(BB, 1, 0) VQ_CASE(BB, 1, 1) VQ_CASE(BB, 1, 2)
  VQ_CASES(1) VQ_CASES(2) VQ_CASES(4)
#undef VQ_CASES
#undef VQ_CASE
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
