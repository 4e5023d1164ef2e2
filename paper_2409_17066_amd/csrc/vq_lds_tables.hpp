// What the decode kernels that keep codebooks in LDS as padded entries share (vq_gemv_lds.hip, vq_gemv_down_lds.hip): the
// window of index words a lane loads at a time, the padded entry, the staging of one table entry.
#pragma once
#include "vq_common.hpp"

namespace vq {
namespace lds_tables {

typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint3v __attribute__((ext_vector_type(3)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

// A window is the smallest run of vectors whose index bits fill whole dwords: 32 / gcd(32, bits) vectors in bits / gcd(32, bits)
// dwords (one dword for 4- and 8-bit indices, three for 12-bit ones).
constexpr int win_vectors(int bits) { return bits % 32 == 0 ? 1 : bits % 16 == 0 ? 2 : bits % 8 == 0 ? 4 : bits % 4 == 0 ? 8 : 32; }
// Halves a table entry takes in LDS: padded to 4, 8 or 16 bytes, so that an entry is one aligned read; v = 12 keeps its 24
// bytes (three 8-byte reads cost no more LDS time than two 16-byte ones, and 4096 entries are 96 KB instead of 128).
constexpr int entry_halfs(int v) { return v <= 2 ? 2 : v <= 4 ? 4 : v <= 8 ? 8 : (v + 3) / 4 * 4; }
// The (v, index width) pairs the kernels are compiled for.
inline bool compiled_pair(int v, int bits, bool with_v6_12) {
  return (v == 2 && bits == 4) || ((v == 4 || v == 6 || v == 8) && bits == 8) || ((v == 4 || v == 8 || v == 12 || (with_v6_12 && v == 6)) && bits == 12);
}

#ifdef __HIPCC__
__device__ __forceinline__ float dot2(unsigned a, unsigned b, float c) {
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b), c, false);
}

// v + (v moved between lanes by a DPP control word); lanes whose row is masked out add 0
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
// Sum over every aligned segment of `seg` lanes (8, 16, 32 or 64; the same for the whole wave): the segment's LAST lane holds it.
__device__ __forceinline__ float segment_sum_to_last(float v, int seg) {
  v = dpp_add<0xB1, 0xF>(v);                  // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xF>(v);                  // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xF>(v);                 // row_half_mirror: every lane of an 8-lane half holds the half's sum
  if (seg > 8) v = dpp_add<0x140, 0xF>(v);    // row_mirror: every lane of a 16-lane row holds the row's sum
  if (seg > 16) v = dpp_add<0x142, 0xA>(v);   // row_bcast15 into rows 1 and 3: lanes 31 and 63 hold 32 lanes' sums
  if (seg > 32) v = dpp_add<0x143, 0xC>(v);   // row_bcast31 into rows 2 and 3: lane 63 holds the wave's sum
  return v;
}

// ND dwords of a stream from byte offset `off`, range-checked (zeros past the buffer's end)
template <int ND>
__device__ __forceinline__ void load_window(unsigned (&w)[ND], __amdgpu_buffer_rsrc_t r, unsigned off) {
  if constexpr (ND == 1) w[0] = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0);
  else {
    static_assert(ND == 3, "windows of one or three dwords");
    const uint3v a = __builtin_amdgcn_raw_buffer_load_b96(r, off, 0, 0);
    w[0] = a.x; w[1] = a.y; w[2] = a.z;
  }
}
// index u of a window (u a compile-time constant after unrolling; NW >= the window's dwords)
template <int BITS, int NW>
__device__ __forceinline__ unsigned window_field(const unsigned (&w)[NW], int u) {
  const int bit = u * BITS, j = bit >> 5, sh = bit & 31;
  unsigned v = w[j] >> sh;
  if (sh + BITS > 32) v |= w[j + 1 < NW ? j + 1 : j] << (32 - sh);
  return v & ((1u << BITS) - 1u);
}

// Entry `en` of a [k][V] table of halves (16-byte aligned: entries of an even number of dwords are 8-byte aligned, of 4 or 8
// dwords 16-byte) into LDS as ED dwords, zero in the pad.
template <int V>
__device__ __forceinline__ void stage_entry(unsigned char *lds_table, const __half *cb, int en) {
  constexpr int VD = V / 2, ED = entry_halfs(V) / 2;
  const unsigned *src = reinterpret_cast<const unsigned *>(cb) + (long long)en * VD;
  unsigned v[ED];
#pragma unroll
  for (int d = 0; d < ED; ++d) v[d] = 0u;
  if constexpr (VD % 4 == 0) {
#pragma unroll
    for (int d = 0; d < VD; d += 4) { const uint4v a = *reinterpret_cast<const uint4v *>(src + d); v[d] = a.x; v[d + 1] = a.y; v[d + 2] = a.z; v[d + 3] = a.w; }
  } else if constexpr (VD % 2 == 0) {
#pragma unroll
    for (int d = 0; d < VD; d += 2) { const uint2v a = *reinterpret_cast<const uint2v *>(src + d); v[d] = a.x; v[d + 1] = a.y; }
  } else {
#pragma unroll
    for (int d = 0; d < VD; ++d) v[d] = src[d];
  }
  unsigned *dst = reinterpret_cast<unsigned *>(lds_table) + en * ED;
  if constexpr (ED % 4 == 0) {
#pragma unroll
    for (int d = 0; d < ED; d += 4) *reinterpret_cast<uint4v *>(dst + d) = uint4v{v[d], v[d + 1], v[d + 2], v[d + 3]};
  } else if constexpr (ED % 2 == 0) {
#pragma unroll
    for (int d = 0; d < ED; d += 2) *reinterpret_cast<uint2v *>(dst + d) = uint2v{v[d], v[d + 1]};
  } else {
#pragma unroll
    for (int d = 0; d < ED; ++d) dst[d] = v[d];
  }
}

// Entry i of a staged table: aligned reads of 16, 8 or 4 bytes.
template <int V>
__device__ __forceinline__ void read_entry(unsigned (&e)[entry_halfs(V) / 2], const unsigned char *lds_table, unsigned i) {
  constexpr int ED = entry_halfs(V) / 2;
  const unsigned *src = reinterpret_cast<const unsigned *>(lds_table) + i * ED;
  if constexpr (ED % 4 == 0) {
#pragma unroll
    for (int d = 0; d < ED; d += 4) { const uint4v a = *reinterpret_cast<const uint4v *>(src + d); e[d] = a.x; e[d + 1] = a.y; e[d + 2] = a.z; e[d + 3] = a.w; }
  } else if constexpr (ED % 2 == 0) {
#pragma unroll
    for (int d = 0; d < ED; d += 2) { const uint2v a = *reinterpret_cast<const uint2v *>(src + d); e[d] = a.x; e[d + 1] = a.y; }
  } else {
#pragma unroll
    for (int d = 0; d < ED; ++d) e[d] = src[d];
  }
}
#endif

}  // namespace lds_tables
}  // namespace vq
