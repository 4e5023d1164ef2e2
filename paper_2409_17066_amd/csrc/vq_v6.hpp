// Device helpers shared by the v = 6 GEMV kernels (internal): bounds-checked index windows, field
// extraction, hand-issued LDS gathers and the LDS layout of the 16-byte-padded codebooks.
#pragma once
#include "vq_common.hpp"

namespace vq {
namespace v6 {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint3v __attribute__((ext_vector_type(3)));

static __device__ __forceinline__ float dot2(unsigned a, unsigned b, float c) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b), c, false);
}

static __device__ __forceinline__ float half_pair_sum(unsigned packed) {
  const half2v h = __builtin_bit_cast(half2v, packed);
  return (float)h.x + (float)h.y;
}

static __device__ __forceinline__ float dpp_add(float v, const int ctrl, const int row_mask) {
  // v + (lane-permuted v); lanes whose row is masked out add 0
  int moved;
  switch (ctrl) {   // the builtin wants literal control words
    case 0xB1: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false); break;
    case 0x4E: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false); break;
    case 0x141: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false); break;
    case 0x140: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false); break;
    case 0x142: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false); break;
    default: moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false); break;
  }
  (void)row_mask;
  return v + __builtin_bit_cast(float, moved);
}

// Sum over the 64 lanes of a wave; the total lands in lane 63.
static __device__ __forceinline__ float wave_reduce_to_lane63(float v) {
  v = dpp_add(v, 0xB1, 0xF);    // quad_perm [1,0,3,2]
  v = dpp_add(v, 0x4E, 0xF);    // quad_perm [2,3,0,1]
  v = dpp_add(v, 0x141, 0xF);   // row_half_mirror
  v = dpp_add(v, 0x140, 0xF);   // row_mirror: every lane of a 16-lane row now holds the row's sum
  v = dpp_add(v, 0x142, 0xA);   // row_bcast15 into rows 1 and 3
  v = dpp_add(v, 0x143, 0xC);   // row_bcast31 into rows 2 and 3
  return v;
}

static __device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// Index window of one lane: N dwords (4 or 6) starting at dword `dw` of the row at byte offset `row_off`.
// Buffer loads are range-checked per dword: dwords past the end of the stream read as zero, never fault.
template <int N> struct Window { unsigned w[N]; };

template <int N>
static __device__ __forceinline__ void load_window(Window<N> &r, __amdgpu_buffer_rsrc_t rsrc, unsigned row_off, unsigned dw) {
  static_assert(N >= 2 && N <= 6, "window of 2..6 dwords");
  const unsigned off = row_off + dw * 4u;
  if constexpr (N == 2) {
    uint2v a = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0);
    r.w[0] = a.x; r.w[1] = a.y;
  } else if constexpr (N == 3) {
    uint3v a = __builtin_amdgcn_raw_buffer_load_b96(rsrc, off, 0, 0);
    r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z;
  } else {
    uint4v a = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
    r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z; r.w[3] = a.w;
    if constexpr (N == 5) r.w[4] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off + 16u, 0, 0);
    if constexpr (N == 6) {
      uint2v b = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off + 16u, 0, 0);
      r.w[4] = b.x; r.w[5] = b.y;
    }
  }
}

// Shift the window right by `sh` bits (0..31) so that the lane's first index starts at bit 0.
template <int N>
static __device__ __forceinline__ void normalize_from(Window<N> &out, const Window<N> &in, unsigned sh) {
#pragma unroll
  for (int i = 0; i < N - 1; ++i) out.w[i] = __builtin_amdgcn_alignbit(in.w[i + 1], in.w[i], sh);
  out.w[N - 1] = in.w[N - 1] >> sh;
}

// Field u (BITS wide) of a normalized window.
template <int BITS, int N>
static __device__ __forceinline__ unsigned field(const Window<N> &win, int u) {
  const int bit = u * BITS, i = bit >> 5, o = bit & 31;
  if (o + BITS <= 32) return __builtin_amdgcn_ubfe(win.w[i], o, BITS);
  return __builtin_amdgcn_alignbit(win.w[i + 1 < N ? i + 1 : i], win.w[i], o) & ((1u << BITS) - 1u);
}

// Byte offset (index << SHIFT) of field u of a normalized window, in two VALU ops: one shift that lands the
// field SHIFT bits up, one mask.  (Fields that straddle two dwords cost one funnel shift more.)
template <int BITS, int SHIFT, int N>
static __device__ __forceinline__ unsigned field_addr(const Window<N> &win, int u) {
  const int bit = u * BITS, i = bit >> 5, o = bit & 31;
  constexpr unsigned mask = ((1u << BITS) - 1u) << SHIFT;
  if (o + BITS <= 32) {
    const unsigned w = win.w[i];
    return (o >= SHIFT ? (w >> (o - SHIFT)) : (w << (SHIFT - o))) & mask;
  }
  return (__builtin_amdgcn_alignbit(win.w[i + 1 < N ? i + 1 : i], win.w[i], o) << SHIFT) & mask;
}

// One centroid (12 bytes + 4 bytes of padding) from LDS, as one ds_read_b128 written by hand: measured on
// gfx950, random 16-byte reads run at ~5.1 per clock per CU, while the 12-byte read the compiler would
// narrow a plain load to (the padding is never used) runs at only ~3.2.  The read is asynchronous:
// lds_gather_wait() must come before the first use of the values.
template <int OFF>
static __device__ __forceinline__ void lds_gather16(uint4v &dst, unsigned lds_addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(lds_addr), "n"(OFF));
}
static __device__ __forceinline__ void lds_gather8(uint2v &dst, unsigned lds_addr) {
  asm volatile("ds_read_b64 %0, %1" : "=v"(dst) : "v"(lds_addr));
}
static __device__ __forceinline__ void lds_gather_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
template <class T> __device__ __forceinline__ void settle(T &v) { asm volatile("" : "+v"(v)); }

// 32-bit LDS address of a pointer into shared memory.
static __device__ __forceinline__ unsigned lds_address(const void *p) {
  return (unsigned)reinterpret_cast<size_t>((const __attribute__((address_space(3))) void *)p);
}


// Table layouts in LDS, all with 16-byte entries (a 32-byte interleave of main and residual entries was
// tried and lost: each table then only touches half of the banks).  The 8-bit residual table goes first so
// that both gathers are "index << 4" plus an immediate offset:
//   no residual:      main at 0
//   8-bit residual:   residual at 0 (4 KB), main at 4096
//   12-bit residual:  main at 0, residual at 65536 (one add per lookup: the offset field holds 16 bits)
template <int RES_BITS> struct Layout {
  static constexpr unsigned MAIN_OFF = RES_BITS == 8 ? 4096u : 0u, MAIN_SH = 4u;
  static constexpr unsigned RES_OFF = 0u, RES_SH = 4u, RES_ADD = RES_BITS == 12 ? 65536u : 0u;
  static constexpr unsigned BYTES = RES_BITS == 0 ? 65536u : RES_BITS == 8 ? 4096u + 65536u : 131072u;
};


// Barrier for LDS traffic only: __syncthreads() would also wait for the index and activation loads that are
// in flight for the next pass.
static __device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// The index words and activations that run ahead of the computation are loaded from inline assembly and
// waited for with counted s_waitcnt: the compiler's own wait insertion, across this kernel's control flow,
// falls back to "wait for everything" at the first use of a loaded register, which would serialise the
// prefetch ring.  Vector memory loads return in issue order, so "at most N outstanding" is exact when N is
// the number of loads known to have been issued after the one needed (more loads after it only make the
// wait stricter).  Descriptors are built by hand so that they can be passed as scalar operands: raw
// buffers with per-dword range checking, out-of-range dwords read as zero.
//
// Two rules keep this sound.  (1) Every asynchronous destination is a read-write ("+v") operand, refilled in
// straight-line code: the new value is tied to the register of the old one, so a slot keeps its register
// through every branch and loop edge.  With write-only operands, or a refill inside a branch, the compiler
// merges old and new values with register copies at the joins -- copies of a register whose load has not
// landed yet.  The build also refuses any spill in these kernels, for the same reason.  (2) Every load
// instruction keeps at least one lane in range.  A load whose lanes are all out of range fetches nothing and
// has been seen to complete ahead of older loads, which breaks the counting.
static __device__ __forceinline__ uint4v scalar_rsrc(const void *base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  uint4v r;
  r.x = (unsigned)a; r.y = (unsigned)(a >> 32) & 0xFFFFu; r.z = bytes; r.w = 0x00020000u;
  return r;
}
static __device__ __forceinline__ void async_load_b64(uint2v &dst, uint4v rsrc, unsigned off) {
  asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "+v"(dst) : "v"(off), "s"(rsrc) : "memory");
}
static __device__ __forceinline__ void async_load_b96(uint3v &dst, uint4v rsrc, unsigned off) {
  asm volatile("buffer_load_dwordx3 %0, %1, %2, 0 offen" : "+v"(dst) : "v"(off), "s"(rsrc) : "memory");
}
template <int N> static __device__ __forceinline__ void wait_vmem_at_most() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

template <int OFF>
static __device__ __forceinline__ void async_load_b128_at(uint4v &dst, uint4v rsrc, unsigned off) {
  asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:%3" : "+v"(dst) : "v"(off), "s"(rsrc), "n"(OFF) : "memory");
}

// Codebooks into LDS with entries padded to 16 bytes (v = 6) or as they are (v = 4, 8 bytes), by T threads, in
// two steps so that the index loads of the first passes can be issued in between: the table loads (hits in
// L2 for all but the first workgroups) then return first and need not wait behind loads from HBM.
// Range-checked loads return zeros past the k entries a table really has.
template <int RES_BITS, int T> struct TableStage {
  static constexpr int GROUPS = 1024 / T;       // groups of 4 entries (48 bytes) per thread and table of 4096
  uint4v m[GROUPS][3], r[RES_BITS == 12 ? GROUPS : 1][3], o[2048 / T];

  // `group` selects the main and residual tables of one codebook group; `outliers` = 0 leaves the outlier table out
  __device__ __forceinline__ void issue(const Params &p, int group = 0, bool outliers = true, unsigned tid = threadIdx.x) {
    const uint4v rm = scalar_rsrc(p.cb + (long long)group * p.k * 6, (unsigned)p.k * 12u);
#pragma unroll
    for (int gi = 0; gi < GROUPS; ++gi) {
      const unsigned off = (tid + gi * T) * 48u;
      async_load_b128_at<0>(m[gi][0], rm, off); async_load_b128_at<16>(m[gi][1], rm, off); async_load_b128_at<32>(m[gi][2], rm, off);
    }
    if (RES_BITS == 12) {
      const uint4v rr = scalar_rsrc(p.cb_res + (long long)group * p.k_res * 6, (unsigned)p.k_res * 12u);
#pragma unroll
      for (int gi = 0; gi < GROUPS; ++gi) {
        const unsigned off = (tid + gi * T) * 48u;
        async_load_b128_at<0>(r[gi][0], rr, off); async_load_b128_at<16>(r[gi][1], rr, off); async_load_b128_at<32>(r[gi][2], rr, off);
      }
    }
    if (RES_BITS == 8) {                         // 256 entries: every wave loads them, the first one stores them
      const uint4v rr = scalar_rsrc(p.cb_res + (long long)group * p.k_res * 6, (unsigned)p.k_res * 12u);
      const unsigned off = (tid & 63u) * 48u;
      async_load_b128_at<0>(r[0][0], rr, off); async_load_b128_at<16>(r[0][1], rr, off); async_load_b128_at<32>(r[0][2], rr, off);
    }
    if (p.Q && outliers) {                       // 4096 entries of 8 bytes
      const uint4v ro = scalar_rsrc(p.cb_out, (unsigned)p.k_out * 8u);
#pragma unroll
      for (int i = 0; i < 2048 / T; ++i) async_load_b128_at<0>(o[i], ro, (tid + i * T) * 16u);
    }
  }

  static __device__ __forceinline__ void put4(unsigned char *base, unsigned first_entry, uint4v (&v)[3]) {
    settle(v[0]); settle(v[1]); settle(v[2]);
    const unsigned d[12] = {v[0].x, v[0].y, v[0].z, v[0].w, v[1].x, v[1].y, v[1].z, v[1].w, v[2].x, v[2].y, v[2].z, v[2].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4v e; e.x = d[3 * i]; e.y = d[3 * i + 1]; e.z = d[3 * i + 2]; e.w = 0u;
      *reinterpret_cast<uint4v *>(base + (first_entry + i) * 16u) = e;
    }
  }

  // after a wait that covers the loads of issue()
  __device__ __forceinline__ void store(const Params &p, unsigned char *lds, unsigned lds_out, bool outliers = true, unsigned tid = threadIdx.x) {
    typedef Layout<RES_BITS> L;
#pragma unroll
    for (int gi = 0; gi < GROUPS; ++gi) put4(lds + L::MAIN_OFF, (tid + gi * T) * 4u, m[gi]);
    if (RES_BITS == 12) {
#pragma unroll
      for (int gi = 0; gi < GROUPS; ++gi) put4(lds + L::RES_ADD, (tid + gi * T) * 4u, r[gi]);
    }
    if (RES_BITS == 8 && tid < 64) put4(lds, tid * 4u, r[0]);
    if (p.Q && outliers) {
#pragma unroll
      for (int i = 0; i < 2048 / T; ++i) {
        settle(o[i]);
        *reinterpret_cast<uint4v *>(lds + lds_out + (tid + i * T) * 16u) = o[i];
      }
    }
  }
};


}  // namespace v6
}  // namespace vq
