// vq_dequant fast paths (paper Sec. 2.2: restore by index and centroid; App. "Our Dequantization
// Implementation", first phase).  Output-write bound: 2 bytes out per weight against 0.25-0.5 bytes in.
//
//  * v = 6, 12-bit indices, optional residual (12- or 8-bit indices), optional outlier columns (v = 4,
//    12-bit indices): codebooks in LDS, one wave restores 64 consecutive vectors (768 bytes of a row)
//    at a time, passes them through a private LDS strip and writes them out as aligned 16-byte stores.
//  * v = 8, 16-bit indices (k up to 65536, codebook in L2): one lane per vector, one 16-byte gather and
//    one 16-byte store.
// The arithmetic is the bit-exact definition: binary32 add of main and residual centroid, one binary32
// fma with scale and bias, one round-to-nearest-even conversion.
#include "vq_common.hpp"
#include <cstdlib>

namespace vq {

namespace {

typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint3v __attribute__((ext_vector_type(3)));

constexpr int NW = 16;   // waves per workgroup (v = 6 kernel)

__device__ __forceinline__ unsigned restore_pair(unsigned main, unsigned res, bool has_res, float s, float b) {
  float lo = __half2float(__ushort_as_half((unsigned short)(main & 0xFFFFu)));
  float hi = __half2float(__ushort_as_half((unsigned short)(main >> 16)));
  if (has_res) {
    lo = __fadd_rn(lo, __half2float(__ushort_as_half((unsigned short)(res & 0xFFFFu))));
    hi = __fadd_rn(hi, __half2float(__ushort_as_half((unsigned short)(res >> 16))));
  }
  return (unsigned)__half_as_ushort(restore(lo, s, b)) | ((unsigned)__half_as_ushort(restore(hi, s, b)) << 16);
}

struct DqPlan {
  unsigned lds_res, lds_out, lds_strip;   // byte offsets in dynamic LDS (main table at 0)
  int main_chunks, out_chunks;            // 64-vector chunks per row
  long long total_chunks;
  long long step;                         // chunks between consecutive chunks of one wave = workgroups x waves
  int step_rows, step_chunks;             // step = step_rows * chunks per row + step_chunks
  int wide;                               // 1: every row start is 16-byte aligned and ldw % 8 == 0
};

// wgs_per_group > 0: a layer with codebook groups (Sec. 3.1).  A group is a layer of its own over a range of columns --
// its tables, its part of the index streams (a group of 8 n vectors starts on a dword of a 12- or 8-bit stream), its
// columns of W -- so workgroups [g * wgs_per_group, (g + 1) * wgs_per_group) take group g and see only that layer; the
// outlier columns go with group 0.
template <int RES_BITS>
__global__ __launch_bounds__(NW * 64) void dequant_v6_kernel(Params p, DqPlan plan, __half *__restrict__ W, long long ldw, int wgs_per_group) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int wg = (int)blockIdx.x;
  if (wgs_per_group > 0) {
    const int grp = wg / wgs_per_group;
    wg -= grp * wgs_per_group;
    const int v_lo = grp * p.Pg;
    p.P = min(p.Pg, p.P - v_lo);
    p.cb += (long long)grp * p.k * 6;
    if (RES_BITS) p.cb_res += (long long)grp * p.k_res * 6;
    p.idx += (long long)(v_lo >> 3) * 12;
    if (RES_BITS) p.idx_res += (long long)(v_lo >> 3) * RES_BITS;
    const int col_lo = grp ? p.n_out + v_lo * 6 : 0;
    p.in_features = min(p.in_features, p.n_out + (v_lo + p.P) * 6) - col_lo;
    W += col_lo;
    if (grp) { p.n_out = 0; p.Q = 0; plan.out_chunks = 0; }
    plan.main_chunks = (p.P + 63) / 64;
    const int cpr = plan.main_chunks + plan.out_chunks;
    plan.total_chunks = (long long)cpr * p.out_features;
    plan.step = (long long)wgs_per_group * NW;
    plan.step_rows = (int)(plan.step / cpr);
    plan.step_chunks = (int)(plan.step % cpr);
  }
  // ---- codebooks into LDS: entries padded to 16 bytes (v = 6) or kept at 8 bytes (v = 4)
  {
    const unsigned *s = reinterpret_cast<const unsigned *>(p.cb);
    for (int e = threadIdx.x; e < 4096; e += NW * 64) {
      uint4v val = {0u, 0u, 0u, 0u};
      if (e < p.k) { val.x = s[e * 3]; val.y = s[e * 3 + 1]; val.z = s[e * 3 + 2]; }
      *reinterpret_cast<uint4v *>(lds + e * 16) = val;
    }
    if (RES_BITS) {
      const unsigned *r = reinterpret_cast<const unsigned *>(p.cb_res);
      for (int e = threadIdx.x; e < (1 << RES_BITS); e += NW * 64) {
        uint4v val = {0u, 0u, 0u, 0u};
        if (e < p.k_res) { val.x = r[e * 3]; val.y = r[e * 3 + 1]; val.z = r[e * 3 + 2]; }
        *reinterpret_cast<uint4v *>(lds + plan.lds_res + e * 16) = val;
      }
    }
    if (plan.out_chunks) {
      const unsigned *q = reinterpret_cast<const unsigned *>(p.cb_out);
      for (int e = threadIdx.x; e < 4096; e += NW * 64) {
        uint2v val = {0u, 0u};
        if (e < p.k_out) { val.x = q[e * 2]; val.y = q[e * 2 + 1]; }
        *reinterpret_cast<uint2v *>(lds + plan.lds_out + e * 8) = val;
      }
    }
  }
  __syncthreads();

  unsigned char *strip = lds + plan.lds_strip + wv * 768;     // this wave's 64 x 12 bytes
  const int chunks_per_row = plan.main_chunks + plan.out_chunks;

  // One chunk = 64 vectors of one row.  What a chunk needs from memory (its index words, the row's scale and bias)
  // is loaded one chunk ahead: with one round trip per chunk exposed, the kernel ran at the memory latency.
  struct Fetch { unsigned m0, m1, r0, r1, sc, bi; };
  auto fetch = [&](int o, int ch, Fetch &f) {
    f.sc = p.scale ? (unsigned)__half_as_ushort(p.scale[o]) : 0x3C00u;
    f.bi = p.bias ? (unsigned)__half_as_ushort(p.bias[o]) : 0u;
    f.m0 = f.m1 = f.r0 = f.r1 = 0u;
    if (ch < plan.out_chunks) {
      const int q = ch * 64 + lane;
      if (q < p.Q) {
        const unsigned *w = reinterpret_cast<const unsigned *>(p.idx_out + (long long)o * p.stride_out) + ((q * 12) >> 5);
        f.m0 = w[0]; f.m1 = ((q * 12) & 31) > 20 ? w[1] : 0u;
      }
    } else {
      const int pp = (ch - plan.out_chunks) * 64 + lane;
      if (pp < p.P) {
        const unsigned *w = reinterpret_cast<const unsigned *>(p.idx + (long long)o * p.stride) + ((pp * 12) >> 5);
        f.m0 = w[0]; f.m1 = ((pp * 12) & 31) > 20 ? w[1] : 0u;
        if (RES_BITS) {
          constexpr int RB = RES_BITS ? RES_BITS : 8;
          const unsigned *r = reinterpret_cast<const unsigned *>(p.idx_res + (long long)o * p.stride_res) + ((pp * RB) >> 5);
          f.r0 = r[0]; f.r1 = ((pp * RB) & 31) > 32 - RB ? r[1] : 0u;
        }
      }
    }
  };
  auto field12 = [](unsigned w0, unsigned w1, int bit) { return __builtin_amdgcn_alignbit(w1, w0, (unsigned)bit & 31u) & 0xFFFu; };

  // chunk ids of this wave: first, first + step, ...; (row, chunk in row) advance without a division
  const long long first = (long long)wg * NW + wv;
  int o = (int)(first / chunks_per_row), ch = (int)(first - (long long)o * chunks_per_row);
  Fetch cur, nxt;
  if (first < plan.total_chunks) fetch(o, ch, cur);
  for (long long id = first; id < plan.total_chunks; id += plan.step) {
    int o2 = o + plan.step_rows, ch2 = ch + plan.step_chunks;
    if (ch2 >= chunks_per_row) { ch2 -= chunks_per_row; ++o2; }
    if (id + plan.step < plan.total_chunks) fetch(o2, ch2, nxt);
    const float s = __half2float(__ushort_as_half((unsigned short)cur.sc));
    const float b = __half2float(__ushort_as_half((unsigned short)cur.bi));
    __half *wrow = W + (long long)o * ldw;
    int c_first, n_cols;                   // first column of the chunk, its valid columns
    if (ch < plan.out_chunks) {
      const int q = ch * 64 + lane;
      c_first = ch * 256; n_cols = min(256, p.n_out - c_first);
      uint2v w = {0u, 0u};
      if (q < p.Q) {
        const unsigned i = field12(cur.m0, cur.m1, q * 12);
        const uint2v e = *reinterpret_cast<const uint2v *>(lds + plan.lds_out + i * 8);
        w.x = restore_pair(e.x, 0u, false, s, b);
        w.y = restore_pair(e.y, 0u, false, s, b);
      }
      *reinterpret_cast<uint2v *>(strip + lane * 8) = w;
    } else {
      const int pp = (ch - plan.out_chunks) * 64 + lane;
      c_first = p.n_out + (ch - plan.out_chunks) * 384; n_cols = min(384, p.in_features - c_first);
      unsigned w0 = 0u, w1 = 0u, w2 = 0u;
      if (pp < p.P) {
        const unsigned i = field12(cur.m0, cur.m1, pp * 12);
        const uint4v e = *reinterpret_cast<const uint4v *>(lds + i * 16);
        uint4v f = {0u, 0u, 0u, 0u};
        if (RES_BITS) {
          constexpr int RB = RES_BITS ? RES_BITS : 8;
          const unsigned r = __builtin_amdgcn_alignbit(cur.r1, cur.r0, (unsigned)(pp * RB) & 31u) & ((1u << RB) - 1u);
          f = *reinterpret_cast<const uint4v *>(lds + plan.lds_res + r * 16);
        }
        w0 = restore_pair(e.x, f.x, RES_BITS != 0, s, b);
        w1 = restore_pair(e.y, f.y, RES_BITS != 0, s, b);
        w2 = restore_pair(e.z, f.z, RES_BITS != 0, s, b);
      }
      unsigned *dst = reinterpret_cast<unsigned *>(strip + lane * 12);
      dst[0] = w0; dst[1] = w1; dst[2] = w2;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- strip -> memory: n_cols halfs starting at column c_first
    if (plan.wide && (c_first & 7) == 0) {
      const int c = lane * 8;                                   // 48 lanes x 8 halfs cover 384 columns
      if (c + 8 <= n_cols) {
        *reinterpret_cast<uint4v *>(wrow + c_first + c) = *reinterpret_cast<const uint4v *>(strip + c * 2);
      } else {
        for (int j = c; j < n_cols; ++j) wrow[c_first + j] = *reinterpret_cast<const __half *>(strip + j * 2);
      }
    } else {
      for (int j = lane; j < n_cols; j += 64) wrow[c_first + j] = *reinterpret_cast<const __half *>(strip + j * 2);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    o = o2; ch = ch2; cur = nxt;
  }
}

__device__ __forceinline__ unsigned restore_pair_v8(unsigned main, unsigned res, bool has_res, float s, float b, bool lo_on, bool hi_on) {
  float lo = __half2float(__ushort_as_half((unsigned short)(main & 0xFFFFu)));
  float hi = __half2float(__ushort_as_half((unsigned short)(main >> 16)));
  if (has_res) {
    lo = __fadd_rn(lo, __half2float(__ushort_as_half((unsigned short)(res & 0xFFFFu))));
    hi = __fadd_rn(hi, __half2float(__ushort_as_half((unsigned short)(res >> 16))));
  }
  const unsigned rl = lo_on ? (unsigned)__half_as_ushort(restore(lo, s, b)) : 0u;
  const unsigned rh = hi_on ? (unsigned)__half_as_ushort(restore(hi, s, b)) : 0u;
  return rl | (rh << 16);
}

// v = 8, indices of IB bytes, a residual table with indices of RB bytes (0: none), no outlier columns.  One lane per
// vector; the 16-byte table entries come through L2.
template <int IB, int RB>
__global__ __launch_bounds__(256) void dequant_v8_kernel(Params p, __half *__restrict__ W, long long ldw, int wide, int blocks_per_row) {
  const int o = blockIdx.x / blocks_per_row;
  const int pp = (blockIdx.x % blocks_per_row) * 256 + threadIdx.x;
  if (pp >= p.P) return;
  const uint8_t *irow = p.idx + (long long)o * p.stride;
  const unsigned raw = IB == 2 ? (unsigned)reinterpret_cast<const unsigned short *>(irow)[pp] : (unsigned)irow[pp];
  const unsigned i = min(raw, (unsigned)p.k - 1u);
  const size_t group = (size_t)(pp / p.Pg);                                                          // its group's tables
  const uint4v e = reinterpret_cast<const uint4v *>(p.cb)[group * (size_t)p.k + i];
  uint4v f = {0u, 0u, 0u, 0u};
  if (RB) {
    const uint8_t *rrow = p.idx_res + (long long)o * p.stride_res;
    const unsigned rraw = RB == 2 ? (unsigned)reinterpret_cast<const unsigned short *>(rrow)[pp] : (unsigned)rrow[pp];
    f = reinterpret_cast<const uint4v *>(p.cb_res)[group * (size_t)p.k_res + min(rraw, (unsigned)p.k_res - 1u)];
  }
  const float s = p.scale ? __half2float(p.scale[o]) : 1.0f;
  const float b = p.bias ? __half2float(p.bias[o]) : 0.0f;
  const int c0 = pp * 8, valid = min(8, p.in_features - c0);
  uint4v w;
  w.x = restore_pair_v8(e.x, f.x, RB != 0, s, b, 0 < valid, 1 < valid);
  w.y = restore_pair_v8(e.y, f.y, RB != 0, s, b, 2 < valid, 3 < valid);
  w.z = restore_pair_v8(e.z, f.z, RB != 0, s, b, 4 < valid, 5 < valid);
  w.w = restore_pair_v8(e.w, f.w, RB != 0, s, b, 6 < valid, 7 < valid);
  __half *dst = W + (long long)o * ldw + c0;
  if (wide && valid == 8) {
    *reinterpret_cast<uint4v *>(dst) = w;
  } else {
    const unsigned d[4] = {w.x, w.y, w.z, w.w};
    for (int j = 0; j < valid; ++j) dst[j] = __ushort_as_half((unsigned short)(d[j >> 1] >> ((j & 1) * 16)));
  }
}

// The same layers when W allows aligned 16-byte stores everywhere (W 16-byte aligned, ldw and the outlier column count
// multiples of 8), main columns only, one codebook group: a wave takes 256 consecutive vectors of a row at a time, four per
// lane (48 index bits: two dwords and a funnel shift), so that the trip through the LDS strip -- each lane leaves its 48
// bytes, then reads three 16-byte pieces in store order -- ends in three stores of 1 KB per wave instead of one of 768
// bytes, and a row has a third as many units.  blockDim.x / 64 waves, a 3 KB strip each.
template <int RES_BITS>
__global__ __launch_bounds__(1024) void dequant_v6_wide_kernel(Params p, unsigned lds_res, unsigned lds_strip, __half *__restrict__ W, long long ldw) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  const int lane = threadIdx.x & 63, n_waves = (int)blockDim.x >> 6;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  {
    const unsigned *src = reinterpret_cast<const unsigned *>(p.cb);
    for (int e = threadIdx.x; e < 4096; e += (int)blockDim.x) {
      uint4v val = {0u, 0u, 0u, 0u};
      if (e < p.k) { val.x = src[e * 3]; val.y = src[e * 3 + 1]; val.z = src[e * 3 + 2]; }
      *reinterpret_cast<uint4v *>(lds + e * 16) = val;
    }
    if (RES_BITS) {
      const unsigned *r = reinterpret_cast<const unsigned *>(p.cb_res);
      for (int e = threadIdx.x; e < (1 << RB); e += (int)blockDim.x) {
        uint4v val = {0u, 0u, 0u, 0u};
        if (e < p.k_res) { val.x = r[e * 3]; val.y = r[e * 3 + 1]; val.z = r[e * 3 + 2]; }
        *reinterpret_cast<uint4v *>(lds + lds_res + e * 16) = val;
      }
    }
  }
  __syncthreads();
  const __amdgpu_buffer_rsrc_t r_main = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(p.idx), 0, (unsigned)p.out_features * (unsigned)p.stride, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_res = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(RES_BITS ? p.idx_res : p.idx), 0,
                                                                         RES_BITS ? (unsigned)p.out_features * (unsigned)p.stride_res : 0u, 0x00020000);
  unsigned char *strip = lds + lds_strip + wv * 3072;
  const int cpr = (p.P + 255) / 256;                       // units per row
  const long long units = (long long)p.out_features * cpr, step = (long long)gridDim.x * n_waves;
  // what a unit needs from memory is asked for one unit ahead
  struct Fetch { unsigned m0, m1, r0, r1; };
  const unsigned lane_off = ((unsigned)lane * 6u) & ~3u, lane_sh = ((unsigned)lane & 1u) * 16u;
  auto fetch = [&](long long unit, Fetch &f) {
    const int o = (int)(unit / cpr), q = (int)(unit - (long long)o * cpr);
    const uint2v m = __builtin_amdgcn_raw_buffer_load_b64(r_main, (unsigned)o * (unsigned)p.stride + (unsigned)q * 384u + lane_off, 0, 0);
    f.m0 = m.x; f.m1 = m.y; f.r0 = f.r1 = 0u;
    if (RES_BITS == 12) {
      const uint2v r = __builtin_amdgcn_raw_buffer_load_b64(r_res, (unsigned)o * (unsigned)p.stride_res + (unsigned)q * 384u + lane_off, 0, 0);
      f.r0 = r.x; f.r1 = r.y;
    }
    if (RES_BITS == 8) f.r0 = __builtin_amdgcn_raw_buffer_load_b32(r_res, (unsigned)o * (unsigned)p.stride_res + (unsigned)q * 256u + (unsigned)lane * 4u, 0, 0);
  };
  const long long first = (long long)blockIdx.x * n_waves + wv;
  Fetch cur, nxt;
  if (first < units) fetch(first, cur);
  for (long long unit = first; unit < units; unit += step) {
    if (unit + step < units) fetch(unit + step, nxt);
    const int o = (int)(unit / cpr), q = (int)(unit - (long long)o * cpr);
    const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
    // the lane's 48 index bits, first index at bit 0
    const unsigned w0 = __builtin_amdgcn_alignbit(cur.m1, cur.m0, lane_sh), w1 = cur.m1 >> lane_sh;
    const unsigned idx[4] = {w0 & 0xFFFu, (w0 >> 12) & 0xFFFu, ((w0 >> 24) | (w1 << 8)) & 0xFFFu, (w1 >> 4) & 0xFFFu};
    unsigned ridx[4] = {0u, 0u, 0u, 0u};
    if (RES_BITS == 12) {
      const unsigned v0 = __builtin_amdgcn_alignbit(cur.r1, cur.r0, lane_sh), v1 = cur.r1 >> lane_sh;
      ridx[0] = v0 & 0xFFFu; ridx[1] = (v0 >> 12) & 0xFFFu; ridx[2] = ((v0 >> 24) | (v1 << 8)) & 0xFFFu; ridx[3] = (v1 >> 4) & 0xFFFu;
    }
    if (RES_BITS == 8) { ridx[0] = cur.r0 & 0xFFu; ridx[1] = (cur.r0 >> 8) & 0xFFu; ridx[2] = (cur.r0 >> 16) & 0xFFu; ridx[3] = cur.r0 >> 24; }
    unsigned out[12];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint4v e = *reinterpret_cast<const uint4v *>(lds + idx[u] * 16);
      uint4v f = {0u, 0u, 0u, 0u};
      if (RES_BITS) f = *reinterpret_cast<const uint4v *>(lds + lds_res + ridx[u] * 16);
      out[3 * u] = restore_pair(e.x, f.x, RES_BITS != 0, sc, bi);
      out[3 * u + 1] = restore_pair(e.y, f.y, RES_BITS != 0, sc, bi);
      out[3 * u + 2] = restore_pair(e.z, f.z, RES_BITS != 0, sc, bi);
    }
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      uint4v pk; pk.x = out[4 * h]; pk.y = out[4 * h + 1]; pk.z = out[4 * h + 2]; pk.w = out[4 * h + 3];
      *reinterpret_cast<uint4v *>(strip + lane * 48 + h * 16) = pk;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int c_first = p.n_out + q * 1536, n_cols = min(1536, p.in_features - c_first);
    __half *wrow = W + (long long)o * ldw + c_first;
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      const int c = (h * 64 + lane) * 8;
      if (c + 8 <= n_cols) {
        *reinterpret_cast<uint4v *>(wrow + c) = *reinterpret_cast<const uint4v *>(strip + c * 2);
      } else {
        for (int j = c; j < n_cols; ++j) wrow[j] = *reinterpret_cast<const __half *>(strip + j * 2);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    cur = nxt;
  }
}

// Orientation 1 (vectors down the output dimension; Sec. 3.1, Algorithm 1), v = 6, 12-bit indices, optional residual:
// a wave takes 512 consecutive columns of one index stream at a time, eight per lane (three aligned index dwords), and
// restores the six rows the stream serves: a lane's eight centroids give, row by row, eight consecutive halves -- one
// 16-byte store each, a wave writes 1 KB of a row at a time.  Tables in LDS, units (stream, 512 columns) dealt round-robin to
// the waves of all workgroups.  The outlier columns are left to the generic kernel.
template <int RES_BITS>
__global__ __launch_bounds__(NW * 64) void dequant_down_v6_kernel(Params p, unsigned lds_res, __half *__restrict__ W, long long ldw, int wide) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int RB = RES_BITS ? RES_BITS : 8;
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  {
    const unsigned *src = reinterpret_cast<const unsigned *>(p.cb);
    for (int e = threadIdx.x; e < 4096; e += NW * 64) {
      uint4v val = {0u, 0u, 0u, 0u};
      if (e < p.k) { val.x = src[e * 3]; val.y = src[e * 3 + 1]; val.z = src[e * 3 + 2]; }
      *reinterpret_cast<uint4v *>(lds + e * 16) = val;
    }
    if (RES_BITS) {
      const unsigned *r = reinterpret_cast<const unsigned *>(p.cb_res);
      for (int e = threadIdx.x; e < (1 << RB); e += NW * 64) {
        uint4v val = {0u, 0u, 0u, 0u};
        if (e < p.k_res) { val.x = r[e * 3]; val.y = r[e * 3 + 1]; val.z = r[e * 3 + 2]; }
        *reinterpret_cast<uint4v *>(lds + lds_res + e * 16) = val;
      }
    }
  }
  __syncthreads();
  const int passes = (p.P + 511) / 512;
  const __amdgpu_buffer_rsrc_t r_main = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(p.idx), 0, (unsigned)p.S * (unsigned)p.stride, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_res = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(RES_BITS ? p.idx_res : p.idx), 0,
                                                                         RES_BITS ? (unsigned)p.S * (unsigned)p.stride_res : 0u, 0x00020000);
  const long long units = (long long)p.S * passes, step = (long long)gridDim.x * NW;
  for (long long unit = (long long)blockIdx.x * NW + wv; unit < units; unit += step) {
    const int stream = (int)(unit / passes), q = (int)(unit - (long long)stream * passes);
    const int pos = q * 512 + lane * 8;                     // the lane's first stream position = main column
    if (pos >= p.P) continue;
    // range-checked loads: the lane's twelve bytes may run past the stream's last index, and past the last stream
    const uint3v wm = __builtin_amdgcn_raw_buffer_load_b96(r_main, (unsigned)stream * (unsigned)p.stride + (unsigned)q * 768u + (unsigned)lane * 12u, 0, 0);
    unsigned r0 = 0u, r1 = 0u, r2 = 0u;
    if (RES_BITS == 12) {
      const uint3v wr = __builtin_amdgcn_raw_buffer_load_b96(r_res, (unsigned)stream * (unsigned)p.stride_res + (unsigned)q * 768u + (unsigned)lane * 12u, 0, 0);
      r0 = wr.x; r1 = wr.y; r2 = wr.z;
    }
    if (RES_BITS == 8) {
      const uint2v wr = __builtin_amdgcn_raw_buffer_load_b64(r_res, (unsigned)stream * (unsigned)p.stride_res + (unsigned)q * 512u + (unsigned)lane * 8u, 0, 0);
      r0 = wr.x; r1 = wr.y;
    }
    const unsigned mw[3] = {wm.x, wm.y, wm.z}, rw[3] = {r0, r1, r2};
    unsigned ex[8], ey[8], ez[8], fx[8], fy[8], fz[8];      // the eight centroids' dwords (main / residual)
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int bit = u * 12, i0 = bit >> 5, o = bit & 31;
      const unsigned idx = (o + 12 <= 32 ? mw[i0] >> o : __builtin_amdgcn_alignbit(mw[i0 + 1 < 3 ? i0 + 1 : i0], mw[i0], o)) & 0xFFFu;
      const uint4v e = *reinterpret_cast<const uint4v *>(lds + idx * 16);
      ex[u] = e.x; ey[u] = e.y; ez[u] = e.z;
      fx[u] = fy[u] = fz[u] = 0u;
      if (RES_BITS) {
        const int rbit = u * RB, j0 = rbit >> 5, ro = rbit & 31;
        const unsigned ridx = (ro + RB <= 32 ? rw[j0] >> ro : __builtin_amdgcn_alignbit(rw[j0 + 1 < 3 ? j0 + 1 : j0], rw[j0], ro)) & ((1u << RB) - 1u);
        const uint4v f = *reinterpret_cast<const uint4v *>(lds + lds_res + ridx * 16);
        fx[u] = f.x; fy[u] = f.y; fz[u] = f.z;
      }
    }
    const int n_valid = min(8, p.P - pos);
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      const int o = stream * 6 + j;
      if (o >= p.out_features) break;
      const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
      unsigned out[4];
#pragma unroll
      for (int h = 0; h < 4; ++h) {                         // columns 2h and 2h + 1: element j of centroids 2h, 2h + 1
        const unsigned ma = j < 2 ? ex[2 * h] : j < 4 ? ey[2 * h] : ez[2 * h], mb = j < 2 ? ex[2 * h + 1] : j < 4 ? ey[2 * h + 1] : ez[2 * h + 1];
        const unsigned ra = j < 2 ? fx[2 * h] : j < 4 ? fy[2 * h] : fz[2 * h], rb = j < 2 ? fx[2 * h + 1] : j < 4 ? fy[2 * h + 1] : fz[2 * h + 1];
        const unsigned sh = (j & 1) * 16;
        float da = __half2float(__ushort_as_half((unsigned short)(ma >> sh))), db = __half2float(__ushort_as_half((unsigned short)(mb >> sh)));
        if (RES_BITS) {
          da = __fadd_rn(da, __half2float(__ushort_as_half((unsigned short)(ra >> sh))));
          db = __fadd_rn(db, __half2float(__ushort_as_half((unsigned short)(rb >> sh))));
        }
        out[h] = (unsigned)__half_as_ushort(restore(da, sc, bi)) | ((unsigned)__half_as_ushort(restore(db, sc, bi)) << 16);
      }
      __half *dst = W + (long long)o * ldw + p.n_out + pos;
      if (wide && n_valid == 8) {
        uint4v pk; pk.x = out[0]; pk.y = out[1]; pk.z = out[2]; pk.w = out[3];
        *reinterpret_cast<uint4v *>(dst) = pk;
      } else {
        for (int c = 0; c < n_valid; ++c) dst[c] = __ushort_as_half((unsigned short)(out[c >> 1] >> ((c & 1) * 16)));
      }
    }
  }
}


template <int RES_BITS>
int launch_v6(const Params &p, DqPlan plan, unsigned lds_bytes, __half *W, long long ldw, hipStream_t s) {
  const int cus = cu_count();
  if (p.n_groups > cus) return VQ_ERR_UNSUPPORTED;
  auto kernel = dequant_v6_kernel<RES_BITS>;
  VQ_ALLOW_FULL_LDS(kernel);
  // the kernel needs few registers, so as many workgroups per compute unit as their LDS allows (at most two: 32 waves)
  const long long slots = (long long)cus * (2u * lds_bytes <= 160u * 1024u ? 2 : 1);
  if (p.n_groups > 1) {
    // the workgroups are shared out evenly over the groups; each group's chunk walk is worked out in the kernel
    const int wgs_per_group = (int)max(1LL, slots / p.n_groups);
    hipLaunchKernelGGL(kernel, dim3((unsigned)(wgs_per_group * p.n_groups)), dim3(NW * 64), lds_bytes, s, p, plan, W, ldw, wgs_per_group);
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  const long long want = (plan.total_chunks + NW - 1) / NW;
  const unsigned grid = (unsigned)(want < slots ? want : slots);
  const int cpr = plan.main_chunks + plan.out_chunks;
  plan.step = (long long)grid * NW;
  plan.step_rows = (int)(plan.step / cpr);
  plan.step_chunks = (int)(plan.step % cpr);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds_bytes, s, p, plan, W, ldw, 0);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// Orientation 1 with v = 8 (W[8s + j][c] = C[idx[s][c]][j]; Sec. 3.1, Algorithm 1), byte-aligned indices: one lane per
// (stream, main column); its entry's eight components go to eight rows of one column, so a wave writes 128 contiguous
// bytes of each of the eight rows.
template <int IB, int RB>
__global__ __launch_bounds__(256) void dequant_down_v8_kernel(Params p, __half *__restrict__ W, long long ldw, int blocks_per_stream) {
  const int stream = blockIdx.x / blocks_per_stream;
  const int pos = (blockIdx.x % blocks_per_stream) * 256 + threadIdx.x;
  if (pos >= p.P) return;
  const uint8_t *irow = p.idx + (long long)stream * p.stride;
  const unsigned raw = IB == 2 ? (unsigned)reinterpret_cast<const unsigned short *>(irow)[pos] : (unsigned)irow[pos];
  const size_t group = (size_t)(pos / p.Pg);
  const uint4v e = reinterpret_cast<const uint4v *>(p.cb)[group * (size_t)p.k + min(raw, (unsigned)p.k - 1u)];
  uint4v f = {0u, 0u, 0u, 0u};
  if (RB) {
    const uint8_t *rrow = p.idx_res + (long long)stream * p.stride_res;
    const unsigned rraw = RB == 2 ? (unsigned)reinterpret_cast<const unsigned short *>(rrow)[pos] : (unsigned)rrow[pos];
    f = reinterpret_cast<const uint4v *>(p.cb_res)[group * (size_t)p.k_res + min(rraw, (unsigned)p.k_res - 1u)];
  }
  const unsigned de[4] = {e.x, e.y, e.z, e.w}, df[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int o = stream * 8 + j;
    if (o < p.out_features) {
      float d = __half2float(__ushort_as_half((unsigned short)(de[j >> 1] >> ((j & 1) * 16))));
      if (RB) d = __fadd_rn(d, __half2float(__ushort_as_half((unsigned short)(df[j >> 1] >> ((j & 1) * 16)))));
      const float sc = p.scale ? __half2float(p.scale[o]) : 1.0f, bi = p.bias ? __half2float(p.bias[o]) : 0.0f;
      W[(long long)o * ldw + p.n_out + pos] = restore(d, sc, bi);
    }
  }
}

}  // namespace

// Main columns of a layer of orientation 1 (v = 6, 12-bit indices, one codebook group; or v = 8, 8- or 16-bit indices, any
// number of groups); VQ_ERR_UNSUPPORTED otherwise.
// The outlier columns, if any, are the caller's (generic kernel).
int launch_dequant_down_fast(const Params &p, __half *W, long long ldw, hipStream_t s) {
  const bool off = switches().dequant == 'g';
  if (off || p.orientation != 1) return VQ_ERR_UNSUPPORTED;
  {
    const int ib = p.bits == 16 ? 2 : p.bits == 8 ? 1 : 0, rbytes = !p.k_res ? 0 : p.bits_res == 16 ? 2 : p.bits_res == 8 ? 1 : -1;
    if (p.v == 8 && ib && rbytes >= 0 && (reinterpret_cast<uintptr_t>(p.cb) & 15) == 0 && (!p.k_res || (reinterpret_cast<uintptr_t>(p.cb_res) & 15) == 0) &&
        (p.stride & 1) == 0 && (!p.k_res || (p.stride_res & 1) == 0)) {
      const int bps = (p.P + 255) / 256;
      const long long blocks = (long long)bps * p.S;
      if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
#define VQ_CASE(IB, RB) \
      if (ib == IB && rbytes == RB) hipLaunchKernelGGL((dequant_down_v8_kernel<IB, RB>), dim3((unsigned)blocks), dim3(256), 0, s, p, W, ldw, bps);
      VQ_CASE(2, 0) VQ_CASE(2, 1) VQ_CASE(2, 2) VQ_CASE(1, 0) VQ_CASE(1, 1) VQ_CASE(1, 2)
#undef VQ_CASE
      return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
    }
  }
  if (p.v != 6 || p.bits != 12 || p.n_groups != 1) return VQ_ERR_UNSUPPORTED;
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return VQ_ERR_UNSUPPORTED;
  if ((long long)p.S * max(p.stride, p.stride_res) >= (1LL << 31)) return VQ_ERR_UNSUPPORTED;      // 32-bit buffer offsets
  const unsigned lds_res = 4096u * 16u;
  const unsigned lds_bytes = lds_res + (p.k_res ? (1u << p.bits_res) * 16u : 0u);
  const int wide = ((reinterpret_cast<uintptr_t>(W) & 15) == 0 && (ldw & 7) == 0 && (p.n_out & 7) == 0) ? 1 : 0;
  const long long units = (long long)p.S * ((p.P + 511) / 512);
  const long long want = (units + NW - 1) / NW, slots = (long long)cu_count() * (2u * lds_bytes <= 160u * 1024u ? 2 : 1);
  const unsigned grid = (unsigned)max(1LL, min(want, slots));
  const void *kernel = !p.k_res ? reinterpret_cast<const void *>(dequant_down_v6_kernel<0>)
                       : p.bits_res == 12 ? reinterpret_cast<const void *>(dequant_down_v6_kernel<12>)
                                          : reinterpret_cast<const void *>(dequant_down_v6_kernel<8>);
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return VQ_ERR_HIP;
  Params pc = p;
  unsigned lr = lds_res;
  int w = wide;
  void *args[] = {&pc, &lr, &W, &ldw, &w};
  return hipLaunchKernel(kernel, dim3(grid), dim3(NW * 64), args, lds_bytes, s) == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// Returns VQ_ERR_UNSUPPORTED when no fast kernel takes the layer (the caller then uses the generic kernel).
int launch_dequant_fast(const Params &p, __half *W, long long ldw, hipStream_t s) {
  const bool off = switches().dequant == 'g';
  if (off || p.orientation != 0) return VQ_ERR_UNSUPPORTED;
  const bool aligned16 = (reinterpret_cast<uintptr_t>(W) & 15) == 0 && (ldw & 7) == 0;
  const int ib = p.bits == 16 ? 2 : p.bits == 8 ? 1 : 0, rbytes = !p.k_res ? 0 : p.bits_res == 16 ? 2 : p.bits_res == 8 ? 1 : -1;
  if (p.v == 8 && ib && rbytes >= 0 && p.n_out == 0 && (reinterpret_cast<uintptr_t>(p.cb) & 15) == 0 &&
      (!p.k_res || (reinterpret_cast<uintptr_t>(p.cb_res) & 15) == 0) && (p.stride & 1) == 0 && (!p.k_res || (p.stride_res & 1) == 0)) {
    const int bpr = (p.P + 255) / 256;
    const long long blocks = (long long)bpr * p.out_features;
    if (blocks > 0x7fffffffLL) return VQ_ERR_UNSUPPORTED;
    const int wide = aligned16 ? 1 : 0;
#define VQ_CASE(IB, RB) \
    if (ib == IB && rbytes == RB) hipLaunchKernelGGL((dequant_v8_kernel<IB, RB>), dim3((unsigned)blocks), dim3(256), 0, s, p, W, ldw, wide, bpr);
    VQ_CASE(2, 0) VQ_CASE(2, 1) VQ_CASE(2, 2) VQ_CASE(1, 0) VQ_CASE(1, 1) VQ_CASE(1, 2)
#undef VQ_CASE
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  if (p.v != 6 || p.bits != 12) return VQ_ERR_UNSUPPORTED;
  if (p.k_res && p.bits_res != 12 && p.bits_res != 8) return VQ_ERR_UNSUPPORTED;
  if (p.n_out && (p.v_out != 4 || p.bits_out != 12)) return VQ_ERR_UNSUPPORTED;
  if (p.n_groups > 1 && (p.Pg & 7)) return VQ_ERR_UNSUPPORTED;    // a group must start on a dword of the index streams
  DqPlan plan{};
  unsigned offb = 4096u * 16u;
  plan.lds_res = offb; offb += p.k_res ? (1u << p.bits_res) * 16u : 0u;
  plan.lds_out = offb; offb += p.n_out ? 4096u * 8u : 0u;
  plan.lds_strip = offb; offb += NW * 768u;
  plan.main_chunks = (p.P + 63) / 64;
  plan.out_chunks = p.n_out ? (p.Q + 63) / 64 : 0;
  plan.total_chunks = (long long)(plan.main_chunks + plan.out_chunks) * p.out_features;
  plan.wide = (aligned16 && (p.n_out & 7) == 0) ? 1 : 0;
  const bool strip_only = switches().dequant == 's';            // 's': never the wide kernel
  const bool wide_route = plan.wide && p.n_groups == 1 && !strip_only && (long long)p.out_features * max(p.stride, p.stride_res) < (1LL << 31);
  // (the wide route keeps no outlier table in LDS: it also takes a 12-bit residual table together with outlier columns)
  if (offb > 160u * 1024u && !wide_route) return VQ_ERR_UNSUPPORTED;
  if (wide_route) {
    // aligned rows: the main columns by the wide kernel, the few outlier columns by the generic kernel
    const unsigned lds_res = 4096u * 16u, lds_strip = lds_res + (p.k_res ? (1u << p.bits_res) * 16u : 0u);
    const int waves = lds_strip + 16u * 3072u <= 160u * 1024u ? 16 : 8;
    const unsigned lds_bytes = lds_strip + (unsigned)waves * 3072u;
    const long long units = (long long)p.out_features * ((p.P + 255) / 256);
    const long long want = (units + waves - 1) / waves, slots = (long long)cu_count() * (2u * lds_bytes <= 160u * 1024u ? 2 : 1);
    const void *kernel = !p.k_res ? reinterpret_cast<const void *>(dequant_v6_wide_kernel<0>)
                         : p.bits_res == 12 ? reinterpret_cast<const void *>(dequant_v6_wide_kernel<12>)
                                            : reinterpret_cast<const void *>(dequant_v6_wide_kernel<8>);
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return VQ_ERR_HIP;
    Params pc = p;
    unsigned lr = lds_res, lst = lds_strip;
    void *args[] = {&pc, &lr, &lst, &W, &ldw};
    if (hipLaunchKernel(kernel, dim3((unsigned)max(1LL, min(want, slots))), dim3(waves * 64), args, lds_bytes, s) != hipSuccess) return VQ_ERR_HIP;
    return p.n_out ? launch_dequant_outliers(p, W, ldw, s) : VQ_OK;
  }
  const int rb = p.k_res ? p.bits_res : 0;
  if (rb == 0) return launch_v6<0>(p, plan, offb, W, ldw, s);
  if (rb == 12) return launch_v6<12>(p, plan, offb, W, ldw, s);
  return launch_v6<8>(p, plan, offb, W, ldw, s);
}

}  // namespace vq
