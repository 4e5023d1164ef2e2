// vq_gemv, one activation row, for the long-row layers of the paper's 70B setting: v = 6 with 12-bit indices, a
// residual codebook of at most 256 entries (8-bit indices), optional outlier columns with v = 4 and 12-bit indices
// (App. "Parameter Description"; Table "Quantization parameters"; decode phase of App. "Our Dequantization
// Implementation").  Vector ALUs only.
//
// One workgroup of 16 waves per compute unit owns a block of rows and keeps every codebook in LDS with entries padded
// to 16 bytes, so that one ds_read_b128 fetches a centroid.  A main wave owns a column slice of 64 x U vectors and a
// row stream (rows s, s + RS, ...): each lane keeps the activations of its U vectors in registers, loaded straight
// from memory, and per row loads its 12 x U main and 8 x U residual index bits as two dword windows (range-checked
// buffer loads), shifts them to bit 0, extracts the indices, gathers the centroids and accumulates with
// v_dot2_f32_f16; row sums are reduced over the wave with DPP and over the slices through a small LDS array;
// y = scale * sum(d x) + bias * sum(x).
//
// What this kernel is built around (gfx950; probes/lds_gather_probe.hip gives nominal clocks per 64 lookups):
//  * the LDS gathers bind: a 16-byte gather at random entries costs 13.3 clocks, most of them bank conflicts, the same
//    read from a table stored as 16 interleaved replicas, lane l reading replica l % 16, costs 5.7.  The 256-entry
//    residual table is therefore stored 16 times (64 KB), which takes a quarter off the LDS time of such a layer;
//  * the fourth dword of a padded entry is never used by the gathers: the 2 x 4096 padding dwords of the two 64 KB
//    regions hold the 4096 x 8-byte outlier table, so all three tables fit 128 KB and nothing else needs LDS (the
//    activations of a 28672-column row, staged in LDS, would be 57 KB);
//  * the row loop is pipelined inside the wave: while one set of U centroids is multiplied the gathers of the other
//    set are in the LDS queue;
//  * index windows are kept as one vector value from load to use and refilled outside branches with clamped row
//    numbers: held as separate dwords a refilled slot is copied between registers at the loop's back edge, and such a
//    copy waits for every load in flight (the loop then runs at one memory latency per round).
#include "vq_common.hpp"
#include "vq_v6.hpp"

namespace vq {
namespace {

using namespace v6;

constexpr int NW = 16;                 // waves per workgroup
constexpr int D = 3;                   // rows of index windows a wave has in flight
constexpr int UO = 8;                  // outlier vectors per lane: 8 x 12 bits = three aligned dwords
constexpr unsigned RES_BASE = 65536u;  // the replicated residual table
constexpr int MAX_ROWS_PER_WG = 512;

struct Res8Plan {
  int W, U, RS, Wo;                    // main slices per row, vectors per lane, row streams, outlier slices
  int rows_per_wg;
  unsigned lds_part, lds_xsum;         // byte offsets of part[rows][W + Wo] and xsum[W + Wo]
  unsigned role[NW];                   // per wave: slice | stream << 8 | main << 16 | outlier << 17
};

// Dwords of a lane's index window: U fields of `bits` bits starting at bit (bits U L) % 32 for lane number L, i.e. at a
// multiple of g = gcd(bits U, 32); the worst start is 32 - g.
constexpr int gcd32(int a) { int g = 32; while (a % g) g >>= 1; return g; }
constexpr int window_dwords(int bits, int u) { return (32 - gcd32(bits * u) + bits * u + 31) / 32; }

template <int N> struct WinT;
template <> struct WinT<1> { typedef unsigned type; };
template <> struct WinT<2> { typedef uint2v type; };
template <> struct WinT<3> { typedef uint3v type; };
template <int N> struct Win { unsigned w[N]; };         // (unpacked, for the arithmetic)

template <int N>
__device__ __forceinline__ void load_win(typename WinT<N>::type &r, __amdgpu_buffer_rsrc_t rsrc, unsigned off) {
  if constexpr (N == 1) r = __builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0);
  else if constexpr (N == 2) r = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0);
  else r = __builtin_amdgcn_raw_buffer_load_b96(rsrc, off, 0, 0);
}
template <int N>
__device__ __forceinline__ void unpack_win(Win<N> &out, typename WinT<N>::type &r) {
  asm volatile("" : "+v"(r));            // pins the first use of the slot (and the compiler's wait for its load) here
  if constexpr (N == 1) { out.w[0] = r; }
  else {
    out.w[0] = r.x; out.w[1] = r.y;
    if constexpr (N >= 3) out.w[2] = r.z;
  }
}

// Shift the window right by `sh` bits (0..31) so that the lane's first index starts at bit 0.
template <int N>
__device__ __forceinline__ void shift_win(Win<N> &out, const Win<N> &in, unsigned sh) {
#pragma unroll
  for (int i = 0; i < N - 1; ++i) out.w[i] = __builtin_amdgcn_alignbit(in.w[i + 1], in.w[i], sh);
  out.w[N - 1] = in.w[N - 1] >> sh;
}

// Byte offset (index << SHIFT) of field u of a shifted window.
template <int BITS, int SHIFT, int N>
__device__ __forceinline__ unsigned field_off(const Win<N> &win, int u) {
  const int bit = u * BITS, i = bit >> 5, o = bit & 31;
  constexpr unsigned mask = ((1u << BITS) - 1u) << SHIFT;
  if (o + BITS <= 32) {
    const unsigned w = win.w[i];
    return (o >= SHIFT ? (w >> (o - SHIFT)) : (w << (SHIFT - o))) & mask;
  }
  return (__builtin_amdgcn_alignbit(win.w[i + 1 < N ? i + 1 : i], win.w[i], o) << SHIFT) & mask;
}

// A lane's activations: N consecutive dwords from a row of x, range-checked (zeros past the buffer).
template <int N>
__device__ __forceinline__ void load_dwords(unsigned (&dst)[N], __amdgpu_buffer_rsrc_t r, unsigned off) {
  constexpr int Q4 = N / 4, REM = N % 4;
#pragma unroll
  for (int i = 0; i < Q4; ++i) {
    const uint4v a = __builtin_amdgcn_raw_buffer_load_b128(r, off + 16u * i, 0, 0);
    dst[4 * i] = a.x; dst[4 * i + 1] = a.y; dst[4 * i + 2] = a.z; dst[4 * i + 3] = a.w;
  }
  if constexpr (REM == 3) {
    const uint3v a = __builtin_amdgcn_raw_buffer_load_b96(r, off + 16u * Q4, 0, 0);
    dst[4 * Q4] = a.x; dst[4 * Q4 + 1] = a.y; dst[4 * Q4 + 2] = a.z;
  } else if constexpr (REM == 2) {
    const uint2v a = __builtin_amdgcn_raw_buffer_load_b64(r, off + 16u * Q4, 0, 0);
    dst[4 * Q4] = a.x; dst[4 * Q4 + 1] = a.y;
  } else if constexpr (REM == 1) {
    dst[4 * Q4] = __builtin_amdgcn_raw_buffer_load_b32(r, off + 16u * Q4, 0, 0);
  }
}

static __device__ __forceinline__ void lds_read32_pad(unsigned &dst, unsigned lds_addr) {     // the fourth dword of a 16-byte entry
  asm volatile("ds_read_b32 %0, %1 offset:12" : "=v"(dst) : "v"(lds_addr));
}
template <int N> static __device__ __forceinline__ void lds_wait_at_most() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }

// LDS layout (bytes):
//   [0, 64K)       main table, entry i at 16 i; its fourth dword holds dword 0 of outlier entry i
//   [64K, 128K)    residual table: entry j, replica r at 64K + 256 j + 16 r; the fourth dword of slot s = 16 j + r holds
//                  dword 1 of outlier entry s
//   then           xsum[W + Wo], part[rows][W + Wo]
template <int U>
__device__ __forceinline__ void gemv_res8_body(const Params &p, const Res8Plan &plan, const __half *__restrict__ x,
                                               __half *__restrict__ y, int wg) {
  constexpr int NM = window_dwords(12, U);
  constexpr int NR = window_dwords(8, U);
  static_assert(NM == 3 || (NM == 2 && U == 4), "an outlier wave reads three dwords of a main slot");
  constexpr int NW3 = 3;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int row0 = wg * plan.rows_per_wg;
  const int rows_here = min(p.out_features - row0, plan.rows_per_wg);
  const int Wt = plan.W + plan.Wo;
  const bool has_out = plan.Wo != 0;
  float *part = reinterpret_cast<float *>(lds + plan.lds_part);     // [rows][Wt]
  float *xsum = reinterpret_cast<float *>(lds + plan.lds_xsum);     // [Wt]
  const unsigned a_base = lds_address(lds);

  const unsigned role = plan.role[wv];          // worked out on the host
  const bool is_main = (role >> 16) & 1u, is_out = (role >> 17) & 1u;
  const int slice = (int)(role & 0xFFu);
  const int stream = (int)((role >> 8) & 0xFFu);

  // ---- the loads of the start-up, oldest first (vector memory loads complete in issue order): activations, tables,
  // the first D rows of index windows, scale and bias

  // activations of this lane's vectors: main lanes 3 U dwords from column n_out + 6 U (64 slice + lane), outlier lanes
  // 2 UO dwords from column 4 UO (64 slice + lane); columns past the part they belong to read as zero
  constexpr int XN = 3 * U > 2 * UO ? 3 * U : 2 * UO;
  constexpr int XA = 3 * U < 2 * UO ? 3 * U : 2 * UO;           // dwords both kinds of wave need; the rest only the one with more
  const unsigned first_col = is_main ? (unsigned)p.n_out + (unsigned)(slice * 64 + lane) * (6u * U) : (unsigned)(slice * 64 + lane) * (4u * UO);
  unsigned xr[XN];
  if (p.perm) {
    // stored column c meets x[col_perm[c]] (Sec. 3.2.3): the lane's columns one by one, range-checked (zero for a column past
    // its part of the row or an entry outside the row).  Every workgroup looks the whole row up: what a caller without a
    // workspace pays; with one, a gather kernel does it once.
    const unsigned lim = is_main ? (unsigned)p.in_features : is_out ? (unsigned)p.n_out : 0u;
    const unsigned lim_rest = (3 * U > 2 * UO ? is_main : is_out) ? lim : 0u;
    unsigned pc[2 * XN];
    load_dwords<2 * XN>(pc, make_rsrc(p.perm, lim * 4u), first_col * 4u);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (unsigned)p.in_features * 2u);
#pragma unroll
    for (int i = 0; i < XN; ++i) {
      const unsigned l = i < XA ? lim : lim_rest;
      const bool ok0 = first_col + 2u * i < l && pc[2 * i] < (unsigned)p.in_features;
      const bool ok1 = first_col + 2u * i + 1u < l && pc[2 * i + 1] < (unsigned)p.in_features;
      const unsigned h0 = __builtin_amdgcn_raw_buffer_load_b16(rx, ok0 ? pc[2 * i] * 2u : 0xFFFFFFFEu, 0, 0);
      const unsigned h1 = __builtin_amdgcn_raw_buffer_load_b16(rx, ok1 ? pc[2 * i + 1] * 2u : 0xFFFFFFFEu, 0, 0);
      xr[i] = h0 | (h1 << 16);
    }
  } else {
    const unsigned bytes = is_main ? (unsigned)p.in_features * 2u : is_out ? (unsigned)p.n_out * 2u : 0u;
    const unsigned bytes_rest = (3 * U > 2 * UO ? is_main : is_out) ? bytes : 0u;
    unsigned head[XA];
    load_dwords<XA>(head, make_rsrc(x, bytes), first_col * 2u);
#pragma unroll
    for (int i = 0; i < XA; ++i) xr[i] = head[i];
    if constexpr (XN > XA) {
      unsigned rest[XN - XA];
      load_dwords<XN - XA>(rest, make_rsrc(x, bytes_rest), first_col * 2u + 4u * XA);
#pragma unroll
      for (int i = 0; i < XN - XA; ++i) xr[XA + i] = rest[i];
    }
  }

  // tables through registers: thread t loads entries 4t .. 4t+3 of the main table (48 bytes), entry t / 4 of the residual
  // table (which it stores as replicas 4 (t % 4) .. + 3), and outlier entries 4t .. 4t+3 (32 bytes).  Offsets are
  // clamped to the table's end where a thread's share lies past it (k < 4096): what such a thread stores are entries
  // that no valid index selects.
  uint4v tm[3], to[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) to[i] = uint4v{0u, 0u, 0u, 0u};
  {
    const __amdgpu_buffer_rsrc_t rm = make_rsrc(p.cb, (unsigned)p.k * 12u);
#pragma unroll
    for (int i = 0; i < 3; ++i) tm[i] = __builtin_amdgcn_raw_buffer_load_b128(rm, min(threadIdx.x * 48u + i * 16u, (unsigned)p.k * 12u - 4u), 0, 0);
  }
  const uint3v tr = __builtin_amdgcn_raw_buffer_load_b96(make_rsrc(p.cb_res, (unsigned)p.k_res * 12u),
                                                         min((threadIdx.x >> 2) * 12u, (unsigned)p.k_res * 12u - 12u), 0, 0);
  if (has_out) {
    const unsigned out_bytes = (unsigned)p.k_out * 8u;
    const __amdgpu_buffer_rsrc_t ro = make_rsrc(p.cb_out, out_bytes);
#pragma unroll
    for (int i = 0; i < 2; ++i) to[i] = __builtin_amdgcn_raw_buffer_load_b128(ro, min(threadIdx.x * 32u + i * 16u, out_bytes - 4u), 0, 0);
  }
  asm volatile("" ::: "memory");

  // index windows.  A main wave's rows are stream, stream + RS, ...; an outlier wave walks every row with three aligned
  // dwords per lane.  Both kinds run the same loads here, with their own buffer, stride and offset (no branch: after a
  // join the compiler waits as if the path with the fewest loads in flight had been taken).
  const int first_vec = (slice * 64 + lane) * U;
  const unsigned bit0 = (unsigned)first_vec * 12u;
  const unsigned off_main = is_main ? (bit0 >> 5) * 4u : (unsigned)(slice * 64 + lane) * 12u, sh_main = is_main ? bit0 & 31u : 0u;
  const unsigned bitr = (unsigned)first_vec * 8u;
  const unsigned off_res = (bitr >> 5) * 4u, sh_res = bitr & 31u;
  const unsigned st_main = (unsigned)(is_out ? p.stride_out : p.stride), st_res = (unsigned)p.stride_res;
  const __amdgpu_buffer_rsrc_t r_main = make_rsrc(is_out ? p.idx_out + (long long)row0 * p.stride_out : p.idx + (long long)row0 * p.stride,
                                                  (unsigned)rows_here * st_main);
  const __amdgpu_buffer_rsrc_t r_res = make_rsrc(p.idx_res + (long long)row0 * p.stride_res, is_main ? (unsigned)rows_here * st_res : 0u);
  const int last_row = rows_here - 1;
  const int step = is_main ? plan.RS : 1;
  const int my_first = is_main ? stream : 0;
  const int my_rows = (is_main || is_out) ? (rows_here - my_first + step - 1) / step : 0;   // rows my_first + i step, i < my_rows

  typename WinT<NW3>::type wm[D];
  typename WinT<NR>::type wr[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    const unsigned r = (unsigned)min(my_first + d * step, last_row);
    load_win<NW3>(wm[d], r_main, r * st_main + off_main);
    load_win<NR>(wr[d], r_res, r * st_res + off_res);
  }
  // scale and bias of the row this thread finishes (clamped row, empty buffer for a missing array: unconditional loads)
  const unsigned ep_off = (unsigned)min((int)threadIdx.x, rows_here - 1) * 2u;
  const unsigned ep_bytes = (unsigned)rows_here * 2u;
  const unsigned short ep_scale_h = __builtin_amdgcn_raw_buffer_load_b16(
      make_rsrc(p.scale ? (const void *)(p.scale + row0) : (const void *)p.cb, p.scale ? ep_bytes : 0u), ep_off, 0, 0);
  const unsigned short ep_bias_h = __builtin_amdgcn_raw_buffer_load_b16(
      make_rsrc(p.bias ? (const void *)(p.bias + row0) : (const void *)p.cb, p.bias ? ep_bytes : 0u), ep_off, 0, 0);
  asm volatile("" ::: "memory");

  // ---- tables into LDS (the compiler's wait covers the table loads only), then the one barrier of the start-up
  {
    const unsigned tid = threadIdx.x;
    const unsigned m[12] = {tm[0].x, tm[0].y, tm[0].z, tm[0].w, tm[1].x, tm[1].y, tm[1].z, tm[1].w, tm[2].x, tm[2].y, tm[2].z, tm[2].w};
    const unsigned o[8] = {to[0].x, to[0].y, to[0].z, to[0].w, to[1].x, to[1].y, to[1].z, to[1].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint4v e; e.x = m[3 * i]; e.y = m[3 * i + 1]; e.z = m[3 * i + 2]; e.w = o[2 * i];
      *reinterpret_cast<uint4v *>(lds + (tid * 4u + i) * 16u) = e;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {        // slots 4t .. 4t+3 = entry t / 4, replicas 4 (t % 4) .. + 3
      uint4v e; e.x = tr.x; e.y = tr.y; e.z = tr.z; e.w = o[2 * i + 1];
      *reinterpret_cast<uint4v *>(lds + RES_BASE + (tid * 4u + i) * 16u) = e;
    }
  }
  // activation sums: the main waves of stream 0 and the outlier waves cover every column once
  if ((is_main && stream == 0) || is_out) {
    float s0 = 0.0f;
#pragma unroll
    for (int i = 0; i < XN; ++i) s0 += half_pair_sum(xr[i]);
    const float s = wave_reduce_to_lane63(s0);
    if (lane == 63) xsum[is_main ? slice : plan.W + slice] = s;
  }
  lds_barrier();                                   // LDS traffic only: the index rows stay in flight

  if (is_out) {
    // ---- outlier columns: 8 vectors of 4 per lane and row; the table lives in the padding dwords of the two 64 KB
    // regions.  The slots are refilled from inline assembly into the same registers and waited for by count: with the
    // compiler's own loads this loop's slots were copied between registers at its back edge.
    const uint4v r_out_s = scalar_rsrc(p.idx_out + (long long)row0 * p.stride_out, (unsigned)rows_here * st_main);
    for (int i0 = 0; i0 < my_rows; i0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int i = i0 + d;
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(wm[d]) : "n"(D - 1) : "memory");   // (the slot's value is what this statement returns)
        Win<NW3> ow;
        unpack_win<NW3>(ow, wm[d]);
        const unsigned w0 = ow.w[0], w1 = ow.w[1], w2 = ow.w[2];
        async_load_b96(wm[d], r_out_s, (unsigned)min(i + D, last_row) * st_main + off_main);
        if (i < my_rows) {
          const unsigned f[UO] = {w0 & 0xFFFu, (w0 >> 12) & 0xFFFu, (w0 >> 24) | ((w1 & 0xFu) << 8), (w1 >> 4) & 0xFFFu,
                                  (w1 >> 16) & 0xFFFu, (w1 >> 28) | ((w2 & 0xFFu) << 4), (w2 >> 8) & 0xFFFu, w2 >> 20};
          float acc = 0.0f;
          unsigned e0[UO], e1[UO];
#pragma unroll
          for (int u = 0; u < UO; ++u) { lds_read32_pad(e0[u], a_base + f[u] * 16u); lds_read32_pad(e1[u], a_base + RES_BASE + f[u] * 16u); }
          lds_gather_wait();
#pragma unroll
          for (int u = 0; u < UO; ++u) { settle(e0[u]); settle(e1[u]); }
#pragma unroll
          for (int u = 0; u < UO; ++u) {
            acc = dot2(e0[u], xr[2 * u], acc);
            acc = dot2(e1[u], xr[2 * u + 1], acc);
          }
          const float s = wave_reduce_to_lane63(acc);
          if (lane == 63) part[i * Wt + plan.W + slice] = s;
        }
      }
    }
    wait_vmem_at_most<0>();
  } else if (is_main) {
    // ---- main columns.  Residual gathers go to this lane's replica of the table.
    // Two sets of U centroid registers, a row's main and residual centroids; while one set is multiplied the gathers of
    // the other are in the LDS queue.  LDS reads return in order: "at most U outstanding" means the older set is in.
    // Rows past the wave's last one (the ring's last round) are computed from a repeated row and not stored.
    const unsigned rep = RES_BASE + ((unsigned)(lane & 15) << 4);
    uint4v e[2][U];
#pragma unroll
    for (int u = 0; u < U; ++u) { e[0][u] = uint4v{0u, 0u, 0u, 0u}; e[1][u] = uint4v{0u, 0u, 0u, 0u}; }
    unsigned am[U], ar[U];
    // index windows of a slot (row number i of this wave) -> LDS addresses; the slot is then requested again
    auto consume = [&](typename WinT<NW3>::type &sm, typename WinT<NR>::type &sr, int i) {
      Win<NW3> raw3;
      Win<NM> cm, raw;
      Win<NR> cr, rawr;
      unpack_win<NW3>(raw3, sm);
#pragma unroll
      for (int j = 0; j < NM; ++j) raw.w[j] = raw3.w[j];
      shift_win(cm, raw, sh_main);
      unpack_win<NR>(rawr, sr);
      shift_win(cr, rawr, sh_res);
      const unsigned r = (unsigned)min(my_first + (i + D) * step, last_row);   // the row D steps ahead (the last row again once past the end)
      load_win<NW3>(sm, r_main, r * st_main + off_main);
      load_win<NR>(sr, r_res, r * st_res + off_res);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        am[u] = field_off<12, 4>(cm, u);
        ar[u] = field_off<8, 8>(cr, u) | rep;
      }
    };
    auto issue = [&](uint4v (&dst)[U], const unsigned (&addr)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) asm volatile("ds_read_b128 %0, %1" : "+v"(dst[u]) : "v"(addr[u]));
    };
    auto dots = [&](uint4v (&src)[U], float &acc) {
#pragma unroll
      for (int u = 0; u < U; ++u) settle(src[u]);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        acc = dot2(src[u].x, xr[3 * u], acc);
        acc = dot2(src[u].y, xr[3 * u + 1], acc);
        acc = dot2(src[u].z, xr[3 * u + 2], acc);
      }
    };
    consume(wm[0], wr[0], 0);
    issue(e[0], am); issue(e[1], ar);
    for (int i0 = 0; i0 < my_rows; i0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        const int i = i0 + d;
        float acc = 0.0f;
        consume(wm[(d + 1) % D], wr[(d + 1) % D], i + 1);
        lds_wait_at_most<U>();                           // in flight: main(i), residual(i)
        dots(e[0], acc);
        issue(e[0], am);
        lds_wait_at_most<U>();                           // in flight: residual(i), main(i + 1)
        dots(e[1], acc);
        issue(e[1], ar);
        const float s = wave_reduce_to_lane63(acc);
        if (lane == 63 && i < my_rows) part[(my_first + i * step) * Wt + slice] = s;
      }
    }
    lds_wait_at_most<0>();
  }
  __syncthreads();
  // ---- combine slices, apply scale and bias, store: thread t finishes row t (+ 1024, ...)
  for (int rl = (int)threadIdx.x; rl < rows_here; rl += NW * 64) {
    float s = 0.0f, xs_all = 0.0f;
    for (int w = 0; w < Wt; ++w) { s += part[rl * Wt + w]; xs_all += xsum[w]; }
    float sc, bi;
    if (rl < NW * 64) {
      sc = p.scale ? __half2float(__ushort_as_half(ep_scale_h)) : 1.0f; bi = p.bias ? __half2float(__ushort_as_half(ep_bias_h)) : 0.0f;
    } else {
      sc = p.scale ? __half2float(p.scale[row0 + rl]) : 1.0f; bi = p.bias ? __half2float(p.bias[row0 + rl]) : 0.0f;
    }
    y[row0 + rl] = __float2half_rn(__fmaf_rn(sc, s, bi * xs_all));
  }
}

template <int U>
__global__ __launch_bounds__(NW * 64) void gemv_res8_kernel(Params p, Res8Plan plan, const __half *__restrict__ x, __half *__restrict__ y) {
  warm_kernel_arguments<5>();                   // Params, the plan and two pointers: 270 bytes
  gemv_res8_body<U>(p, plan, x, y, (int)blockIdx.x);
}


template <int U>
int launch_one(const Params &p, const Res8Plan &plan, unsigned lds_bytes, unsigned grid, const __half *x, __half *y, hipStream_t s) {
  auto kernel = gemv_res8_kernel<U>;
  static const hipError_t configured =
      hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (configured != hipSuccess) return VQ_ERR_HIP;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds_bytes, s, p, plan, x, y);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Whether the kernel takes this layer and these activations (one activation row).
bool gemv_res8_applicable(const Params &p, const __half *x) {
  if (p.orientation != 0 || p.v != 6 || p.bits != 12 || p.n_groups > 1) return false;
  if (!p.k_res || p.bits_res != 8) return false;
  if (p.n_out && (p.v_out != 4 || p.bits_out != 12)) return false;
  if ((reinterpret_cast<uintptr_t>(x) & 3) || (p.in_features & 1)) return false;
  return true;
}

int launch_gemv_res8(const Params &p, const __half *x, __half *y, hipStream_t s) {
  static const int kU[] = {4, 5, 6};
  Res8Plan plan{};
  const int g = min(cu_count(), p.out_features);
  plan.rows_per_wg = min((p.out_features + g - 1) / g, MAX_ROWS_PER_WG);
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  const long long max_stride = max(p.stride, max(p.stride_res, p.stride_out));
  if ((long long)plan.rows_per_wg * max_stride >= (1LL << 31)) return VQ_ERR_UNSUPPORTED;       // 32-bit buffer offsets
  plan.Wo = p.Q ? (p.Q + 64 * UO - 1) / (64 * UO) : 0;
  if (plan.Wo >= NW) return VQ_ERR_UNSUPPORTED;
  // vectors per lane U and main slices W: fill the lanes, keep the waves busy, balance the rows over the row streams
  double best = -1.0;
  for (int U : kU) {
    const int W = (p.P + 64 * U - 1) / (64 * U);
    if (W + plan.Wo > NW) continue;
    const int RS = min((NW - plan.Wo) / W, plan.rows_per_wg);
    const int iters = (plan.rows_per_wg + RS - 1) / RS;
    const double eff = (double)p.P / (64.0 * W * U) * (double)(RS * W) / NW * (double)plan.rows_per_wg / ((double)iters * RS);
    if (eff > best) { best = eff; plan.W = W; plan.U = U; plan.RS = RS; }
  }
  if (best < 0.0) return VQ_ERR_UNSUPPORTED;
  for (int w = 0; w < NW; ++w) {
    const int n_main = plan.RS * plan.W;
    if (w < n_main) plan.role[w] = (unsigned)(w % plan.W) | ((unsigned)(w / plan.W) << 8) | (1u << 16);
    else if (w - n_main < plan.Wo) plan.role[w] = (unsigned)(w - n_main) | (1u << 17);
    else plan.role[w] = 0u;
  }
  const int Wt = plan.W + plan.Wo;
  unsigned off = 2u * RES_BASE;
  plan.lds_xsum = off; off += (unsigned)Wt * 4u;
  plan.lds_part = off; off += (unsigned)(plan.rows_per_wg * Wt) * 4u;
  if (off > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  if (plan.U == 4) return launch_one<4>(p, plan, off, grid, x, y, s);
  if (plan.U == 5) return launch_one<5>(p, plan, off, grid, x, y, s);
  return launch_one<6>(p, plan, off, grid, x, y, s);
}

}  // namespace vq
