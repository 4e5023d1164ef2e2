// vq_quantize_columns: the column loop of the quantizer (Algorithm 1, Sec. 3.1 "VPTQ Algorithm"; error update: the
// Delta W equation of that section).  Columns are quantized one at a time -- every column a stack of length-v vectors
// that each take their nearest centroid (Eq. 2; with a residual codebook a second one for what the first leaves, Sec.
// 3.2.2) -- and the column's error, divided by the diagonal entry of the matrix the algorithm calls H^-1, is spread over
// the later columns: inside a block of B columns at once, over the rest of the matrix at the end of the block.
//
// The rows of the matrix never meet in this loop: a vector's v rows only ever read their own weights and rows of H^-1.
// So one wave owns one stack position (v rows) for a whole block of columns and keeps its v x B tile of running weights
// in registers (lane l holds columns l and l + 64 of the block).  The columns of a position are a dependent chain, so what
// counts is the time of one column, most of which is the nearest-centroid search (2 v + 3 vector-ALU instructions per
// centroid, as in vq_assign, whose distance arithmetic this follows): four waves share it, each a quarter of the
// centroids over its 64 lanes, and meet through LDS.  The end-of-block update W[:, rest] -= E * Hinv[block, rest] is a
// dense binary32 product and runs on the matrix cores (v_mfma_f32_32x32x2_f32) from LDS tiles.
#include "vq_common.hpp"

namespace vq {
namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int QS = 3;            // stack positions per workgroup of the column kernel
constexpr int SW = 4;            // waves that share the search of one position
constexpr int QB = 128;          // most columns per block: two per lane
constexpr int CPL = QB / 64;

constexpr int entry_halfs(int v) { return v <= 4 ? 4 : v <= 8 ? 8 : 16; }     // table entries padded to 8, 16 or 32 bytes

struct QArgs {
  float *W; long long ldw; int rows, cols;
  const float *Hinv; long long ldh;
  const __half *cb; int k; const __half *cb_res; int k_res;
  int s, s_end;
  unsigned *idx; long long idx_dwords; int bits;             // streams as dwords: stride in dwords
  unsigned *idx_res; long long idx_res_dwords; int bits_res;
  float *T; long long ldt;
  float *E;                                                   // [rows][QB]: the block's scaled errors
};

// Minimum of an unsigned value over the wave, in every lane: shifts within rows of 16 lanes, then the row broadcasts
// (lanes without a source keep the identity), then the last lane's value read back.
__device__ __forceinline__ unsigned wave_min_u32(unsigned v) {
#define VQ_DPP_MIN(CTRL, ROWS) v = min(v, (unsigned)__builtin_amdgcn_update_dpp((int)0xFFFFFFFFu, (int)v, CTRL, ROWS, 0xF, false))
  VQ_DPP_MIN(0x111, 0xF);      // row_shr:1
  VQ_DPP_MIN(0x112, 0xF);      // row_shr:2
  VQ_DPP_MIN(0x114, 0xF);      // row_shr:4
  VQ_DPP_MIN(0x118, 0xF);      // row_shr:8  -> lane 15 of every row holds the row's minimum
  VQ_DPP_MIN(0x142, 0xA);      // row_bcast:15 into rows 1 and 3
  VQ_DPP_MIN(0x143, 0xC);      // row_bcast:31 into rows 2 and 3 -> lane 63 holds the wave's minimum
#undef VQ_DPP_MIN
  return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

// smaller distance, else smaller index: the rule by which the lanes' candidates meet.  Distances are sums of squares, so
// their bit patterns order like the numbers: the smallest pattern first, then the smallest index among its holders.
__device__ __forceinline__ void wave_arg_min(float &d, unsigned &i) {
  const unsigned bits = __float_as_uint(d);
  const unsigned lowest = wave_min_u32(bits);
  i = wave_min_u32(bits == lowest ? i : 0xFFFFFFFFu);
  d = __uint_as_float(lowest);
}

typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));

// One padded table entry (EH halfs) as EH / 2 dwords.  From LDS the read is issued from inline assembly as one or two whole
// 16-byte reads (8 bytes for the smallest entries): left to the compiler, a read whose tail is unused is narrowed and
// split into 2- and 8-byte reads at odd offsets, which the LDS serves many times slower.  The caller waits
// (lds_reads_done) before it looks at the registers.
template <int EH>
__device__ __forceinline__ void read_entry_lds(unsigned (&dst)[EH / 2], unsigned lds_addr) {
  if constexpr (EH == 4) {
    uint2v r;
    asm volatile("ds_read_b64 %0, %1" : "=v"(r) : "v"(lds_addr));
    dst[0] = r.x; dst[1] = r.y;
  } else {
#pragma unroll
    for (int q = 0; q < EH / 8; ++q) {
      uint4v r;
      if (q == 0) asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(lds_addr));
      else asm volatile("ds_read_b128 %0, %1 offset:16" : "=v"(r) : "v"(lds_addr));
      dst[4 * q] = r.x; dst[4 * q + 1] = r.y; dst[4 * q + 2] = r.z; dst[4 * q + 3] = r.w;
    }
  }
}
template <int N>
__device__ __forceinline__ void lds_reads_done(unsigned (&regs)[N]) {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(regs[i]));      // nothing reads them ahead of the wait
}
template <int EH>
__device__ __forceinline__ void read_entry_global(unsigned (&dst)[EH / 2], const __half *entry) {
#pragma unroll
  for (int q = 0; q < EH / 2; ++q) dst[q] = reinterpret_cast<const unsigned *>(entry)[q];
}
__device__ __forceinline__ float half_of(unsigned dword, int hi) { return __half2float(__ushort_as_half((unsigned short)(hi ? dword >> 16 : dword & 0xFFFFu))); }

// Candidate of one wave for the nearest of `count` centroids to t[0 .. len): the wave is search wave `sw` of SW, its lane
// l takes centroids 64 sw + l, + 64 SW, ... in ascending order (strict "less" keeps the lowest index of equal distances
// among its own), then the lanes meet by (distance, index).  Distance: binary32, one subtraction and one fused
// multiply-add per element into a sum that starts at +0, elements ascending.  The table is `lds_table` (an LDS byte
// address) when IN_LDS, else `table`; entries are EH halfs apart.
template <int V, int EH, int SW, bool IN_LDS>
__device__ __forceinline__ void nearest(unsigned lds_table, const __half *table, int count, const float (&t)[V], int len, int lane, int sw,
                                        float &best, unsigned &arg) {
  best = __builtin_inff();
  arg = 0xFFFFFFFFu;                                          // a lane without centroids never wins
  constexpr int UN = EH == 16 ? (IN_LDS ? 2 : 1) : 4;                        // centroids in flight per lane: their sums do not depend on each other
  for (int i0 = sw * 64 + lane; i0 < count; i0 += 64 * SW * UN) {
    unsigned c[UN][EH / 2];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int i = min(i0 + 64 * SW * u, count - 1);         // (past the end: the last entry again, never taken below)
      if constexpr (IN_LDS) read_entry_lds<EH>(c[u], lds_table + (unsigned)i * (EH * 2u));
      else read_entry_global<EH>(c[u], table + (long long)i * EH);
    }
    if constexpr (IN_LDS) {
#pragma unroll
      for (int u = 0; u < UN; ++u) lds_reads_done(c[u]);
    }
    float d[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      d[u] = 0.0f;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        if (j < len) {
          // t - c as one fused operation on the binary16 value (the same single rounding as a subtraction of the widened
          // value: the product c * -1 is exact), which the mixed-precision multiply-add takes without a conversion
          const float diff = __fmaf_rn(half_of(c[u][j >> 1], j & 1), -1.0f, t[j]);
          d[u] = __fmaf_rn(diff, diff, d[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u)
      if (i0 + 64 * SW * u < count && d[u] < best) { best = d[u]; arg = (unsigned)(i0 + 64 * SW * u); }
  }
  wave_arg_min(best, arg);
}

// workgroup barrier that waits for LDS traffic only (the owner waves keep a row of H^-1 on its way across it)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One workgroup: QS stack positions (v rows each), SW waves per position.  Wave 0 of a position owns its v x B tile of
// running weights in registers (lane l holds columns l and l + 64 of the block) and does everything but the search, which
// all SW waves share: per column the owner posts the vector in LDS, every wave searches its share of the centroids and
// posts its candidate, the owner takes the best of them (smaller distance, else smaller index).  All positions of a
// workgroup walk the block's columns in step (two barriers a column, four with a residual codebook).
template <int V, bool IN_LDS>
__global__ __launch_bounds__(QS * SW * 64) void qcol_block_kernel(QArgs a, unsigned table_bytes) {
  constexpr int EH = entry_halfs(V);
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // smem: [k][EH] then [k_res][EH] halfs when IN_LDS, then the exchange area
  float *post = reinterpret_cast<float *>(smem + (IN_LDS ? table_bytes : 0u));   // [QS][2][16]: the vector, then what the first stage leaves
  float *cand_d = post + QS * 32;                                             // [QS][SW]
  unsigned *cand_i = reinterpret_cast<unsigned *>(cand_d + QS * SW);          // [QS][SW]
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int st = wave / SW, sw = wave % SW;
  const bool owner = sw == 0;
  if constexpr (IN_LDS) {
    const int n16 = ((a.k + a.k_res) * EH + 7) / 8;                        // both tables are one contiguous padded array (its end rounded up)
    for (int e = threadIdx.x; e < n16; e += QS * SW * 64) reinterpret_cast<uint4 *>(smem)[e] = reinterpret_cast<const uint4 *>(a.cb)[e];
    __syncthreads();
  }
  // (table pointers are formed from the LDS array itself where the tables are in LDS: a pointer that could be either kind
  // of memory would be read with flat loads)
  const unsigned lds0 = (unsigned)reinterpret_cast<size_t>((const __attribute__((address_space(3))) void *)smem);
  auto find = [&](bool residual, int count, const float (&vec)[V], int len_, float &d, unsigned &i) {
    nearest<V, EH, SW, IN_LDS>(lds0 + (residual ? (unsigned)a.k * (EH * 2u) : 0u), residual ? a.cb_res : a.cb, count, vec, len_, lane, sw, d, i);
  };
  auto entry = [&](bool residual, unsigned index, int j) -> float {
    if constexpr (IN_LDS) return __half2float((reinterpret_cast<const __half *>(smem) + (residual ? (long long)a.k * EH : 0LL))[(long long)index * EH + j]);
    else return __half2float((residual ? a.cb_res : a.cb)[(long long)index * EH + j]);
  };
  const int p = blockIdx.x * QS + st;
  const int m0 = p * V;
  const bool active = m0 < a.rows;                      // (a position past the last one still walks the barriers)
  const int len = active ? min(V, a.rows - m0) : 0;
  const int nb = a.s_end - a.s;
  float *my_post = post + st * 32;

  // the owner's tiles, lane l holding columns l and l + 64 of the block: running weights, and -- filled in column by column,
  // written out in whole rows at the end of the block -- the scaled errors and the columns as they stood when quantized
  // (vectors longer than 8 would need more registers than a wave of a 16-wave workgroup has: their errors and columns
  // are stored column by column instead)
  constexpr bool TILES = V <= 8;
  constexpr int TV = TILES ? V : 1;
  float w[CPL][V], et[CPL][TV], tt[CPL][TV];
  unsigned code[CPL] = {0u, 0u}, code_res[CPL] = {0u, 0u};
  float h[CPL] = {0.0f, 0.0f}, h1[CPL] = {0.0f, 0.0f};      // rows n and n + 1 of H^-1 (the row after them is on its way)
  auto hinv_row = [&](int nn_, int i) -> float {
    const int c = a.s + lane + 64 * i;
    return (nn_ < nb && c < a.s_end) ? a.Hinv[(long long)(a.s + nn_) * a.ldh + c] : 0.0f;
  };
  if (owner) {
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = a.s + lane + 64 * i;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        w[i][j] = (c < a.s_end && j < len) ? a.W[(long long)(m0 + j) * a.ldw + c] : 0.0f;
        if (j < TV) { et[i][j] = 0.0f; tt[i][j] = 0.0f; }
      }
      h[i] = hinv_row(0, i);
      h1[i] = hinv_row(1, i);
    }
  }

  for (int nn = 0; nn < nb; ++nn) {
    const int src = nn & 63, slot = nn >> 6;                                // the lane and register that hold column n
    float h_next[CPL] = {0.0f, 0.0f};
    float hd = 1.0f;
    float t[V], q[V];
    if (owner) {
      // the row of H^-1 two columns on goes out before the search
#pragma unroll
      for (int i = 0; i < CPL; ++i) h_next[i] = hinv_row(nn + 2, i);
      hd = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(slot ? h[1] : h[0]), src));     // Hinv[n][n]
#pragma unroll
      for (int j = 0; j < V; ++j) t[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(slot ? w[1][j] : w[0][j]), src));
      if (lane == 0) {
#pragma unroll
        for (int j = 0; j < V; ++j) my_post[j] = t[j];
      }
    }
    lds_barrier();
#pragma unroll
    for (int j = 0; j < V; ++j) t[j] = my_post[j];
    {
      float d; unsigned i;
      find(false, active ? a.k : 0, t, len, d, i);
      if (lane == 0) { cand_d[st * SW + sw] = d; cand_i[st * SW + sw] = i; }
    }
    lds_barrier();
    unsigned best = 0u, best_res = 0u;
    if (owner && active) {
      float bd = cand_d[st * SW]; best = cand_i[st * SW];
#pragma unroll
      for (int x = 1; x < SW; ++x) {
        const float d2 = cand_d[st * SW + x]; const unsigned i2 = cand_i[st * SW + x];
        if (d2 < bd || (d2 == bd && i2 < best)) { bd = d2; best = i2; }
      }
#pragma unroll
      for (int j = 0; j < V; ++j) q[j] = entry(false, best, j);
    }
    if (a.k_res) {
      if (owner && active && lane == 0) {
#pragma unroll
        for (int j = 0; j < V; ++j) my_post[16 + j] = __fsub_rn(t[j], q[j]);
      }
      lds_barrier();
      {
        float r[V];
#pragma unroll
        for (int j = 0; j < V; ++j) r[j] = my_post[16 + j];
        float d; unsigned i;
        find(true, active ? a.k_res : 0, r, len, d, i);
        if (lane == 0) { cand_d[st * SW + sw] = d; cand_i[st * SW + sw] = i; }
      }
      lds_barrier();
      if (owner && active) {
        float bd = cand_d[st * SW]; best_res = cand_i[st * SW];
#pragma unroll
        for (int x = 1; x < SW; ++x) {
          const float d2 = cand_d[st * SW + x]; const unsigned i2 = cand_i[st * SW + x];
          if (d2 < bd || (d2 == bd && i2 < best_res)) { bd = d2; best_res = i2; }
        }
#pragma unroll
        for (int j = 0; j < V; ++j) {
          // what inference restores: the binary32 sum of the two centroids, rounded to binary16 (Sec. 3.2.2)
          float sum = __fadd_rn(q[j], entry(true, best_res, j));
          asm volatile("" : "+v"(sum));
          q[j] = __half2float(__float2half_rn(sum));
        }
      }
    }
    if (owner && active) {
      float e[V];
#pragma unroll
      for (int j = 0; j < V; ++j) e[j] = j < len ? __fdiv_rn(__fsub_rn(t[j], q[j]), hd) : 0.0f;
      // spread over the block's later columns; column n itself becomes its quantized value
#pragma unroll
      for (int i = 0; i < CPL; ++i) {
        const int col = lane + 64 * i;
#pragma unroll
        for (int j = 0; j < V; ++j) {
          if (col > nn) w[i][j] = __fmaf_rn(-e[j], h[i], w[i][j]);
          else if (col == nn) w[i][j] = q[j];
        }
        if (col == nn) {
          code[i] = best; code_res[i] = best_res;
          if constexpr (TILES) {
#pragma unroll
            for (int j = 0; j < V; ++j) { et[i][j] = e[j]; tt[i][j] = t[j]; }
          }
        }
      }
      if constexpr (!TILES) {
        if (lane == 0) {
#pragma unroll
          for (int j = 0; j < V; ++j)
            if (j < len) {
              if (a.T) a.T[(long long)(m0 + j) * a.ldt + a.s + nn] = t[j];
              a.E[(long long)(m0 + j) * QB + nn] = e[j];
            }
        }
      }
#pragma unroll
      for (int i = 0; i < CPL; ++i) { h[i] = h1[i]; h1[i] = h_next[i]; }
    }
  }
  if (!(owner && active)) return;

  // the block's quantized columns, and their indices into the packed streams (one per column: stream p, position n;
  // the streams were cleared beforehand and no other wave touches stream p)
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = a.s + lane + 64 * i;
    if (c < a.s_end) {
#pragma unroll
      for (int j = 0; j < V; ++j)
        if (j < len) {
          a.W[(long long)(m0 + j) * a.ldw + c] = w[i][j];
          if constexpr (TILES) {
            a.E[(long long)(m0 + j) * QB + lane + 64 * i] = et[i][j];
            if (a.T) a.T[(long long)(m0 + j) * a.ldt + c] = tt[i][j];
          }
        }
      {
        const unsigned long long bit = (unsigned long long)c * (unsigned)a.bits;
        unsigned *row = a.idx + (long long)p * a.idx_dwords + (bit >> 5);
        const unsigned sh = (unsigned)(bit & 31u);
        atomicOr(row, code[i] << sh);
        if (sh + a.bits > 32) atomicOr(row + 1, code[i] >> (32u - sh));
      }
      if (a.k_res) {
        const unsigned long long bit = (unsigned long long)c * (unsigned)a.bits_res;
        unsigned *row = a.idx_res + (long long)p * a.idx_res_dwords + (bit >> 5);
        const unsigned sh = (unsigned)(bit & 31u);
        atomicOr(row, code_res[i] << sh);
        if (sh + a.bits_res > 32) atomicOr(row + 1, code_res[i] >> (32u - sh));
      }
    }
  }
}

// Tables as padded entries, main then residual, one array (what the column kernel copies into LDS or reads in place).
__global__ __launch_bounds__(256) void pad_tables_kernel(const __half *__restrict__ cb, int k, const __half *__restrict__ cb_res, int k_res, int v, int eh,
                                                         __half *__restrict__ out) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= (k + k_res) * eh) return;
  const int entry = e / eh, j = e - entry * eh;
  __half val = __float2half_rn(0.0f);
  if (j < v) val = entry < k ? cb[(long long)entry * v + j] : cb_res[(long long)(entry - k) * v + j];
  out[e] = val;
}

__global__ __launch_bounds__(256) void clear_dwords_kernel(unsigned *p, long long stride_dwords, int dwords_per_row, int rows) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)rows * dwords_per_row) return;
  const long long r = e / dwords_per_row;
  p[r * stride_dwords + (e - r * dwords_per_row)] = 0u;
}

// W[:, c0 ...] -= E[:, 0 .. nb) * Hinv[s .. s + nb, c0 ...]: one workgroup per 64 x 64 tile of W, a wave per 32 x 32 quarter,
// both operands through LDS, v_mfma_f32_32x32x2_f32 (lane l gives A[l & 31][l >> 5] and B[l >> 5][l & 31]; it gets back
// column l & 31 and, in register r, row 8 (r >> 2) + 4 (l >> 5) + (r & 3)).
__global__ __launch_bounds__(256) void qcol_trailing_kernel(float *__restrict__ W, long long ldw, int rows, int cols, const float *__restrict__ E,
                                                            const float *__restrict__ Hinv, long long ldh, int s, int nb, int c_first) {
  extern __shared__ __attribute__((aligned(16))) float tiles[];
  float (*As)[QB + 1] = reinterpret_cast<float (*)[QB + 1]>(tiles);                  // [64][QB + 1]
  float (*Bs)[64] = reinterpret_cast<float (*)[64]>(tiles + 64 * (QB + 1));         // [QB][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = blockIdx.y * 64, c0 = c_first + blockIdx.x * 64;
  for (int e = threadIdx.x; e < 64 * QB; e += 256) {
    const int r = e / QB, kk = e - r * QB;
    As[r][kk] = (r0 + r < rows && kk < nb) ? E[(long long)(r0 + r) * QB + kk] : 0.0f;
  }
  for (int e = threadIdx.x; e < QB * 64; e += 256) {
    const int kk = e >> 6, c = e & 63;
    Bs[kk][c] = (kk < nb && c0 + c < cols) ? Hinv[(long long)(s + kk) * ldh + c0 + c] : 0.0f;
  }
  __syncthreads();
  const int wr = (wave >> 1) * 32, wc = (wave & 1) * 32;
  float16v acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const int kmax = (nb + 1) & ~1;
  for (int kk = 0; kk < kmax; kk += 2)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[wr + (lane & 31)][kk + (lane >> 5)], Bs[kk + (lane >> 5)][wc + (lane & 31)], acc, 0, 0, 0);
  const int c = c0 + wc + (lane & 31);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = r0 + wr + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (row < rows && c < cols) W[(long long)row * ldw + c] -= acc[r];
  }
}

template <int V>
int launch_block(const QArgs &a, bool in_lds, unsigned lds_bytes, hipStream_t st) {
  const unsigned grid = (unsigned)(((a.rows + V - 1) / V + QS - 1) / QS);
  const unsigned exchange = (QS * 32 + 2 * QS * SW) * 4u;            // posted vectors and candidates
  if (in_lds) {
    VQ_ALLOW_FULL_LDS((qcol_block_kernel<V, true>));
    hipLaunchKernelGGL((qcol_block_kernel<V, true>), dim3(grid), dim3(QS * SW * 64), lds_bytes + exchange, st, a, lds_bytes);
  } else {
    hipLaunchKernelGGL((qcol_block_kernel<V, false>), dim3(grid), dim3(QS * SW * 64), exchange, st, a, 0u);
  }
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Workspace: the block's errors E [rows][128] binary32, then both tables as padded entries.
size_t quantize_columns_workspace_bytes(int rows, int v, int k, int k_res) {
  const size_t e = ((size_t)rows * QB * sizeof(float) + 255) / 256 * 256;
  return e + ((size_t)(k + k_res) * entry_halfs(v) * sizeof(__half) + 255) / 256 * 256;
}

int launch_quantize_columns(float *W, long long ldw, int rows, int cols, const float *Hinv, long long ldh, const __half *cb, int v, int k,
                            const __half *cb_res, int k_res, int block, unsigned char *idx, long long idx_stride, unsigned char *idx_res,
                            long long idx_res_stride, float *T, long long ldt, void *workspace, hipStream_t st) {
  const int eh = entry_halfs(v);
  const int bits = index_bits(k), bits_res = k_res ? index_bits(k_res) : 0;
  const int S = (rows + v - 1) / v;
  float *E = static_cast<float *>(workspace);
  __half *padded = reinterpret_cast<__half *>(static_cast<unsigned char *>(workspace) + ((size_t)rows * QB * sizeof(float) + 255) / 256 * 256);
  const int n_pad = (k + k_res) * eh;
  hipLaunchKernelGGL(pad_tables_kernel, dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st, cb, k, cb_res, k_res, v, eh, padded);
  // every dword that holds one of a stream's cols * bits bits starts at zero (the column kernel ORs its indices in)
  const int dw = (int)(((long long)cols * bits + 31) / 32), dw_res = (int)(((long long)cols * bits_res + 31) / 32);
  hipLaunchKernelGGL(clear_dwords_kernel, dim3((unsigned)(((long long)S * dw + 255) / 256)), dim3(256), 0, st, reinterpret_cast<unsigned *>(idx),
                     idx_stride / 4, dw, S);
  if (k_res)
    hipLaunchKernelGGL(clear_dwords_kernel, dim3((unsigned)(((long long)S * dw_res + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<unsigned *>(idx_res), idx_res_stride / 4, dw_res, S);
  if (hipGetLastError() != hipSuccess) return VQ_ERR_HIP;
  const size_t table_bytes = (size_t)n_pad * sizeof(__half);
  const bool in_lds = table_bytes <= 150 * 1024;
  QArgs a{};
  a.W = W; a.ldw = ldw; a.rows = rows; a.cols = cols; a.Hinv = Hinv; a.ldh = ldh;
  a.cb = padded; a.k = k; a.cb_res = padded + (size_t)k * eh; a.k_res = k_res;
  a.idx = reinterpret_cast<unsigned *>(idx); a.idx_dwords = idx_stride / 4; a.bits = bits;
  a.idx_res = reinterpret_cast<unsigned *>(idx_res); a.idx_res_dwords = idx_res_stride / 4; a.bits_res = bits_res;
  a.T = T; a.ldt = ldt; a.E = E;
  for (int s = 0; s < cols; s += block) {
    a.s = s; a.s_end = s + block < cols ? s + block : cols;
    int rc = VQ_ERR_UNSUPPORTED;
    switch (v) {
#define VQ_CASE(V) case V: rc = launch_block<V>(a, in_lds, (unsigned)table_bytes, st); break;
      VQ_CASE(1) VQ_CASE(2) VQ_CASE(3) VQ_CASE(4) VQ_CASE(5) VQ_CASE(6) VQ_CASE(7) VQ_CASE(8)
      VQ_CASE(9) VQ_CASE(10) VQ_CASE(11) VQ_CASE(12) VQ_CASE(13) VQ_CASE(14) VQ_CASE(15) VQ_CASE(16)
#undef VQ_CASE
    }
    if (rc != VQ_OK) return rc;
    if (a.s_end < cols) {
      const unsigned gx = (unsigned)((cols - a.s_end + 63) / 64), gy = (unsigned)((rows + 63) / 64);
      if (gy > 65535u) return VQ_ERR_UNSUPPORTED;
      VQ_ALLOW_FULL_LDS(qcol_trailing_kernel);
      hipLaunchKernelGGL(qcol_trailing_kernel, dim3(gx, gy), dim3(256), (64 * (QB + 1) + QB * 64) * sizeof(float), st, W, ldw, rows, cols, E, Hinv,
                         ldh, s, a.s_end - s, a.s_end);
      if (hipGetLastError() != hipSuccess) return VQ_ERR_HIP;
    }
  }
  return VQ_OK;
}

}  // namespace vq
