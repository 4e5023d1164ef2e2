// Pieces shared by the prefill GEMM kernels that feed the FP16 matrix cores from swizzled LDS tiles (vq_gemm_fused.hip: v = 8
// layers gathered from L2 and the dense product; vq_gemm_v6.hip: v = 6 layers gathered from LDS tables): tile geometry, the
// LDS-only barrier, loads issued from inline assembly with counted waits, the bit-exact restore of two and eight weights.
#pragma once
#include "vq_common.hpp"

namespace vq {
namespace gemm_tiles {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));

constexpr int BN = 128;       // output channels per workgroup
constexpr int BK = 32;        // columns per step (4 vectors of 8)
constexpr int LDT = BK;       // W tile row pitch in halfs: 64-byte rows, chunks swizzled like the activation tile
constexpr int GD = 8;         // centroid gathers run this many steps ahead (one register slot per step); also the index group size
constexpr int XD = 3;         // activation copies run this many steps ahead
constexpr int NSX = XD + 1;   // activation stages in LDS

__device__ __forceinline__ unsigned restore2(unsigned packed, float s, float b) {
  const unsigned short l = (unsigned short)(packed & 0xFFFFu), h = (unsigned short)(packed >> 16);
  const __half rl = restore(__half2float(__ushort_as_half(l)), s, b);
  const __half rh = restore(__half2float(__ushort_as_half(h)), s, b);
  return (unsigned)__half_as_ushort(rl) | ((unsigned)__half_as_ushort(rh) << 16);
}

// eight halfs -> scale * d + bias in binary32 -> eight halfs (all zero when `on` is false)
__device__ __forceinline__ uint4v restore8(uint4v d, float s, float b, bool on) {
  uint4v out = {0u, 0u, 0u, 0u};
  if (on) {
    out.x = restore2(d.x, s, b);
    out.y = restore2(d.y, s, b);
    out.z = restore2(d.z, s, b);
    out.w = restore2(d.w, s, b);
  }
  return out;
}

// Workgroup barrier for the step loop.  __syncthreads() carries a release fence, for which the compiler waits
// until EVERY outstanding memory operation of the wave has completed (s_waitcnt vmcnt(0)): that drains the
// centroid gathers and activation copies that were issued steps ahead on purpose, and made each step cost a
// full memory round trip.  Here only LDS traffic is waited for; the caller waits for the global->LDS copies
// it needs by count.
__device__ __forceinline__ void step_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Loads whose completion the kernel tracks itself.  The compiler's own wait insertion cannot count memory
// operations across the unrolled, looping producer schedule and falls back to "wait for everything" at the
// first use of a loaded register, which again drains the prefetch queues every step.  These loads are
// therefore issued from inline assembly and consumed only after an explicit s_waitcnt with a counted bound.
__device__ __forceinline__ void async_load16(uint4v &dst, const void *base, unsigned byte_offset) {
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=&v"(dst) : "v"(byte_offset), "s"(base) : "memory");
}
__device__ __forceinline__ void async_load16(uint4v &dst, const void *address) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(dst) : "v"(address) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmem_at_most() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
template <class T> __device__ __forceinline__ void settle(T &v) { asm volatile("" : "+v"(v)); }

// Both tiles in LDS are [rows][32 halfs] with unpadded 64-byte rows (the asynchronous activation copy writes
// 64 lanes x 16 bytes contiguously).  An MFMA operand read is 16-lane groups of 16 consecutive rows, same
// 16-byte chunk; LDS serves 64 banks x 4 bytes per cycle, i.e. sixteen 16-byte groups, and row r's chunks
// start at group 4r mod 16: rows r, r+4, r+8, r+12 collide unless their chunks differ.  XOR-ing the chunk
// index with bits 2..3 of the row makes every such read, and the producers' writes, conflict-free.
__device__ __forceinline__ unsigned swz(unsigned row) { return (row >> 2) & 3u; }
__device__ __forceinline__ unsigned x_slot(unsigned row, unsigned chunk) {     // byte offset inside a stage / W buffer
  return row * 64u + ((chunk ^ swz(row)) << 4);
}

}  // namespace gemm_tiles
}  // namespace vq
