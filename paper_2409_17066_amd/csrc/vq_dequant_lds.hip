// vq_dequant for the layers that have no restore kernel of their own (the paper's other (v, k) settings: App. "Impact of
// Vector Length", Table "Quantization parameters" -- v = 12 with two 4096-entry tables, v = 4 / k = 256, codebook groups) with
// the tables in LDS instead of behind the caches, where every lookup of the generic kernel drags a 128-byte line out of L2.
// Same arithmetic as everywhere (Sec. 2.2 lookup; Sec. 3.2.2: binary32 sum of main and residual centroid; one binary32 fma
// with scale and bias; round to nearest even to binary16), so the result is the same bits.
//
// One 1024-thread workgroup per compute unit owns a block of rows; a wave takes a row at a time, a lane a vector, so that a
// wave's stores cover one contiguous span of the row.  The tables sit in LDS as they are.  Where main and residual table of a
// codebook group fit together, one pass per group does everything.  Where they do not (two 4096 x 12 tables are 192 KB), the
// group takes two passes: the first writes the main centroids to W as they are -- binary16 values, exact -- and the second,
// with the residual table in the main table's place, reads them back (the same thread that wrote them), adds, restores and
// writes the final weights.  That scheme is the fallback (dequant=s): by default the residual entries of such layers are
// read from memory (the table stays in L2) while the main table is in LDS, one pass, which is faster (11008 x 4096, v = 12:
// 63 against 100 us).  Outlier columns are left to the caller (the generic kernel restores them afterwards).
#include "vq_common.hpp"

namespace vq {

namespace {

constexpr int DW = 16;           // waves per workgroup

struct DqLdsPlan {
  unsigned off_res, bytes;       // residual table behind the main table (both resident), LDS bytes
  int both, rows_per_wg;
  int res_global;                // the residual table does not fit beside the main one: its entries are read from memory
};

// index p of a row's stream: the two dwords that hold it, range-checked against the end of the stream array
template <int BITS>
__device__ __forceinline__ unsigned stream_index(__amdgpu_buffer_rsrc_t r, unsigned row_off, int pv) {
  typedef unsigned uint2v __attribute__((ext_vector_type(2)));
  const unsigned bit = (unsigned)pv * BITS;
  const uint2v w = __builtin_amdgcn_raw_buffer_load_b64(r, row_off + (bit >> 5) * 4u, 0, 0);
  return __builtin_amdgcn_alignbit(w.y, w.x, bit & 31u) & ((1u << BITS) - 1u);
}

// entry i of a [k][V] table in memory (16-byte aligned table: entries of an even number of dwords are 8-byte aligned)
template <int V>
__device__ __forceinline__ void global_entry(unsigned (&e)[V / 2], const __half *table, unsigned i) {
  constexpr int VD = V / 2;
  typedef unsigned uint2v __attribute__((ext_vector_type(2)));
  const unsigned *src = reinterpret_cast<const unsigned *>(table) + (long long)i * VD;
  if constexpr (VD % 2 == 0) {
#pragma unroll
    for (int d = 0; d < VD; d += 2) { const uint2v a = *reinterpret_cast<const uint2v *>(src + d); e[d] = a.x; e[d + 1] = a.y; }
  } else {
#pragma unroll
    for (int d = 0; d < VD; ++d) e[d] = src[d];
  }
}

template <int V, int BITS, bool A4>      // A4: W, ldw and the first main column allow dword stores
__global__ __launch_bounds__(DW * 64) void dequant_lds_kernel(Params p, DqLdsPlan plan, __half *__restrict__ W, long long ldw) {
  constexpr int VD = V / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const unsigned *T = reinterpret_cast<const unsigned *>(lds);
  const unsigned *Tr = reinterpret_cast<const unsigned *>(lds + plan.off_res);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int row0 = blockIdx.x * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.out_features * p.stride), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.k_res ? p.idx_res : p.idx), 0,
                                                                       p.k_res ? (unsigned)((long long)p.out_features * p.stride_res) : 0u, 0x00020000);
  const bool two = p.k_res && !plan.both && !plan.res_global;     // two passes per group
  const int per_group = two ? 2 : 1;
  for (int pass = 0; pass < p.n_groups * per_group; ++pass) {
    const int g = pass / per_group;
    const bool second = two && pass - g * per_group == 1;
    const int p_lo = g * p.Pg, p_hi = min(p.P, p_lo + p.Pg);
    __syncthreads();                                      // every wave has left the tables of the pass before
    {
      const unsigned *src = reinterpret_cast<const unsigned *>(second ? p.cb_res + (long long)g * p.k_res * V : p.cb + (long long)g * p.k * V);
      const int n = (second ? p.k_res : p.k) * VD;
      unsigned *dst = reinterpret_cast<unsigned *>(lds);
#pragma unroll 4
      for (int e = threadIdx.x; e < n; e += DW * 64) dst[e] = src[e];
      if (plan.both) {
        const unsigned *srcr = reinterpret_cast<const unsigned *>(p.cb_res + (long long)g * p.k_res * V);
        unsigned *dstr = reinterpret_cast<unsigned *>(lds + plan.off_res);
#pragma unroll 4
        for (int e = threadIdx.x; e < p.k_res * VD; e += DW * 64) dstr[e] = srcr[e];
      }
    }
    __syncthreads();

    const bool add_res = plan.both || second || plan.res_global;   // this pass adds a residual centroid
    const bool final_pass = !two || second;               // this pass writes final weights
    const unsigned k_main = (unsigned)(second ? p.k_res : p.k);
    for (int o = row0 + wv; o < row1; o += DW) {
      const float s = p.scale ? __half2float(p.scale[o]) : 1.0f, b = p.bias ? __half2float(p.bias[o]) : 0.0f;
      __half *wrow = W + (long long)o * ldw + p.n_out;
      const unsigned ro_i = (unsigned)o * (unsigned)p.stride, ro_r = (unsigned)o * (unsigned)p.stride_res;
      for (int pv = p_lo + lane; pv < p_hi; pv += 64) {
        // the table in LDS this pass: the main one, or (second pass) the residual one, looked up with the residual index
        const unsigned i = min(second ? stream_index<BITS>(r_r, ro_r, pv) : stream_index<BITS>(r_i, ro_i, pv), k_main - 1u);
        unsigned e[VD], f[VD];
#pragma unroll
        for (int d = 0; d < VD; ++d) e[d] = T[i * VD + d];
        if (plan.both) {
          const unsigned ir = min(stream_index<BITS>(r_r, ro_r, pv), (unsigned)p.k_res - 1u);
#pragma unroll
          for (int d = 0; d < VD; ++d) f[d] = Tr[ir * VD + d];
        } else if (plan.res_global) {
          const unsigned ir = min(stream_index<BITS>(r_r, ro_r, pv), (unsigned)p.k_res - 1u);
          global_entry<V>(f, p.cb_res + (long long)g * p.k_res * V, ir);
        }
        const int c0 = pv * V;                            // first main column of the vector (stored order, after the outlier columns)
        const int n_cols = min(V, p.in_features - p.n_out - c0);          // the row's last vector may stick out
        if (second) {                                     // the main centroid, written by this thread in the pass before
#pragma unroll
          for (int d = 0; d < VD; ++d) {
            f[d] = e[d];
            if (A4 && 2 * d + 1 < n_cols) e[d] = *reinterpret_cast<const unsigned *>(wrow + c0 + 2 * d);
            else {
              const unsigned lo = 2 * d < n_cols ? (unsigned)__half_as_ushort(wrow[c0 + 2 * d]) : 0u;
              const unsigned hi = 2 * d + 1 < n_cols ? (unsigned)__half_as_ushort(wrow[c0 + 2 * d + 1]) : 0u;
              e[d] = lo | (hi << 16);
            }
          }
        }
#pragma unroll
        for (int d = 0; d < VD; ++d) {
          unsigned out = e[d];
          if (final_pass) {
            float lo = __half2float(__ushort_as_half((unsigned short)(e[d] & 0xFFFFu)));
            float hi = __half2float(__ushort_as_half((unsigned short)(e[d] >> 16)));
            if (add_res) {
              lo = __fadd_rn(lo, __half2float(__ushort_as_half((unsigned short)(f[d] & 0xFFFFu))));
              hi = __fadd_rn(hi, __half2float(__ushort_as_half((unsigned short)(f[d] >> 16))));
            }
            out = (unsigned)__half_as_ushort(restore(lo, s, b)) | ((unsigned)__half_as_ushort(restore(hi, s, b)) << 16);
          }
          if (A4 && 2 * d + 1 < n_cols) *reinterpret_cast<unsigned *>(wrow + c0 + 2 * d) = out;
          else {
            if (2 * d < n_cols) wrow[c0 + 2 * d] = __ushort_as_half((unsigned short)(out & 0xFFFFu));
            if (2 * d + 1 < n_cols) wrow[c0 + 2 * d + 1] = __ushort_as_half((unsigned short)(out >> 16));
          }
        }
      }
    }
  }
}

template <int V, int BITS>
int launch_vb(const Params &p, const DqLdsPlan &plan, bool a4, __half *W, long long ldw, hipStream_t s) {
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  if (a4) {
    VQ_ALLOW_FULL_LDS((dequant_lds_kernel<V, BITS, true>));
    hipLaunchKernelGGL((dequant_lds_kernel<V, BITS, true>), dim3(grid), dim3(DW * 64), plan.bytes, s, p, plan, W, ldw);
  } else {
    VQ_ALLOW_FULL_LDS((dequant_lds_kernel<V, BITS, false>));
    hipLaunchKernelGGL((dequant_lds_kernel<V, BITS, false>), dim3(grid), dim3(DW * 64), plan.bytes, s, p, plan, W, ldw);
  }
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

// The same for layers stored with vectors down the output dimension (Sec. 3.1): a stream is V rows, an index a column.  The
// (stream, 128 columns) items of a workgroup's streams are dealt to its waves; a lane restores two adjacent columns of the
// stream's V rows, so that a wave's stores are dwords side by side in every row.
template <int V, int BITS, bool A4>
__global__ __launch_bounds__(DW * 64) void dequant_down_lds_kernel(Params p, DqLdsPlan plan, __half *__restrict__ W, long long ldw) {
  constexpr int VD = V / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const unsigned *T = reinterpret_cast<const unsigned *>(lds);
  const unsigned *Tr = reinterpret_cast<const unsigned *>(lds + plan.off_res);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int s0 = blockIdx.x * plan.rows_per_wg, s1 = min(p.S, s0 + plan.rows_per_wg);      // (streams per workgroup)
  const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.S * p.stride), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.k_res ? p.idx_res : p.idx), 0,
                                                                       p.k_res ? (unsigned)((long long)p.S * p.stride_res) : 0u, 0x00020000);
  const bool two = p.k_res && !plan.both && !plan.res_global;
  const int per_group = two ? 2 : 1;
  for (int pass = 0; pass < p.n_groups * per_group; ++pass) {
    const int g = pass / per_group;
    const bool second = two && pass - g * per_group == 1;
    const int p_lo = g * p.Pg, p_hi = min(p.P, p_lo + p.Pg);
    __syncthreads();
    {
      const unsigned *src = reinterpret_cast<const unsigned *>(second ? p.cb_res + (long long)g * p.k_res * V : p.cb + (long long)g * p.k * V);
      const int n = (second ? p.k_res : p.k) * VD;
      unsigned *dst = reinterpret_cast<unsigned *>(lds);
#pragma unroll 4
      for (int e = threadIdx.x; e < n; e += DW * 64) dst[e] = src[e];
      if (plan.both) {
        const unsigned *srcr = reinterpret_cast<const unsigned *>(p.cb_res + (long long)g * p.k_res * V);
        unsigned *dstr = reinterpret_cast<unsigned *>(lds + plan.off_res);
#pragma unroll 4
        for (int e = threadIdx.x; e < p.k_res * VD; e += DW * 64) dstr[e] = srcr[e];
      }
    }
    __syncthreads();

    const bool add_res = plan.both || second || plan.res_global, final_pass = !two || second;
    const unsigned k_main = (unsigned)(second ? p.k_res : p.k);
    const int chunks = (p_hi - p_lo + 127) / 128;
    for (int item = wv; item < (s1 - s0) * chunks; item += DW) {
      const int sl = item / chunks, st = s0 + sl, pos0 = p_lo + (item - sl * chunks) * 128 + 2 * lane;
      if (pos0 >= p_hi) continue;
      const bool two_cols = pos0 + 1 < p_hi;
      const unsigned ro_i = (unsigned)st * (unsigned)p.stride, ro_r = (unsigned)st * (unsigned)p.stride_res;
      unsigned e[2][VD], f[2][VD];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int pos = two_cols ? pos0 + c : pos0;
        const unsigned i = min(second ? stream_index<BITS>(r_r, ro_r, pos) : stream_index<BITS>(r_i, ro_i, pos), k_main - 1u);
#pragma unroll
        for (int d = 0; d < VD; ++d) e[c][d] = T[i * VD + d];
        if (plan.both) {
          const unsigned ir = min(stream_index<BITS>(r_r, ro_r, pos), (unsigned)p.k_res - 1u);
#pragma unroll
          for (int d = 0; d < VD; ++d) f[c][d] = Tr[ir * VD + d];
        } else if (plan.res_global) {
          const unsigned ir = min(stream_index<BITS>(r_r, ro_r, pos), (unsigned)p.k_res - 1u);
          global_entry<V>(f[c], p.cb_res + (long long)g * p.k_res * V, ir);
        }
      }
#pragma unroll
      for (int j = 0; j < V; ++j) {
        const int o = st * V + j;
        if (o >= p.out_features) break;
        __half *w = W + (long long)o * ldw + p.n_out + pos0;
        unsigned short h[2], r[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          h[c] = (unsigned short)((j & 1) ? e[c][j / 2] >> 16 : e[c][j / 2] & 0xFFFFu);
          r[c] = plan.both || plan.res_global ? (unsigned short)((j & 1) ? f[c][j / 2] >> 16 : f[c][j / 2] & 0xFFFFu) : (unsigned short)0;
        }
        if (second) {                                     // the main centroids, written by this thread in the pass before
          r[0] = h[0]; r[1] = h[1];
          if (A4 && two_cols) {
            const unsigned m = *reinterpret_cast<const unsigned *>(w);
            h[0] = (unsigned short)(m & 0xFFFFu); h[1] = (unsigned short)(m >> 16);
          } else {
            h[0] = __half_as_ushort(w[0]);
            if (two_cols) h[1] = __half_as_ushort(w[1]);
          }
        }
        if (final_pass) {
          const float s = p.scale ? __half2float(p.scale[o]) : 1.0f, b = p.bias ? __half2float(p.bias[o]) : 0.0f;
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            float d = __half2float(__ushort_as_half(h[c]));
            if (add_res) d = __fadd_rn(d, __half2float(__ushort_as_half(r[c])));
            h[c] = __half_as_ushort(restore(d, s, b));
          }
        }
        if (A4 && two_cols) *reinterpret_cast<unsigned *>(w) = (unsigned)h[0] | ((unsigned)h[1] << 16);
        else {
          w[0] = __ushort_as_half(h[0]);
          if (two_cols) w[1] = __ushort_as_half(h[1]);
        }
      }
    }
  }
}

template <int V, int BITS>
int launch_down_vb(const Params &p, const DqLdsPlan &plan, bool a4, __half *W, long long ldw, hipStream_t s) {
  const unsigned grid = (unsigned)((p.S + plan.rows_per_wg - 1) / plan.rows_per_wg);
  if (a4) {
    VQ_ALLOW_FULL_LDS((dequant_down_lds_kernel<V, BITS, true>));
    hipLaunchKernelGGL((dequant_down_lds_kernel<V, BITS, true>), dim3(grid), dim3(DW * 64), plan.bytes, s, p, plan, W, ldw);
  } else {
    VQ_ALLOW_FULL_LDS((dequant_down_lds_kernel<V, BITS, false>));
    hipLaunchKernelGGL((dequant_down_lds_kernel<V, BITS, false>), dim3(grid), dim3(DW * 64), plan.bytes, s, p, plan, W, ldw);
  }
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// The main columns of a layer with vectors along the rows, stored column order (the caller restores outlier columns and moves
// permuted columns); VQ_ERR_UNSUPPORTED for (v, index width) pairs without a compiled kernel or tables beyond LDS.
int launch_dequant_lds(const Params &p, __half *W, long long ldw, hipStream_t s) {
  if (switches().dequant == 'g' || p.orientation != 0 || (p.k_res && p.bits_res != p.bits)) return VQ_ERR_UNSUPPORTED;
  if ((long long)p.out_features * p.stride >= (1LL << 32) || (long long)p.out_features * p.stride_res >= (1LL << 32)) return VQ_ERR_UNSUPPORTED;
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  const size_t main = up16((size_t)p.k * p.v * 2), res = up16((size_t)p.k_res * p.v * 2);
  DqLdsPlan plan{};
  plan.both = p.k_res && main + res <= 160 * 1024;
  plan.off_res = (unsigned)main;
  plan.res_global = p.k_res && !plan.both && main <= 160 * 1024 && switches().dequant != 's';
  plan.bytes = (unsigned)(plan.both ? main + res : plan.res_global ? main : main > res ? main : res);
  if (plan.bytes > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  const int wgs = cu_count();
  plan.rows_per_wg = (p.out_features + wgs - 1) / wgs;
  if (plan.rows_per_wg < DW) plan.rows_per_wg = DW;
  const bool a4 = (reinterpret_cast<uintptr_t>(W) & 3) == 0 && (ldw & 1) == 0 && (p.n_out & 1) == 0;
#define VQ_PAIR(V, BITS) if (p.v == V && p.bits == BITS) return launch_vb<V, BITS>(p, plan, a4, W, ldw, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

// The main columns of a layer with vectors down the output dimension, stored column order (outlier streams and permuted
// columns are the caller's).
int launch_dequant_down_lds(const Params &p, __half *W, long long ldw, hipStream_t s) {
  if (switches().dequant == 'g' || p.orientation != 1 || (p.k_res && p.bits_res != p.bits)) return VQ_ERR_UNSUPPORTED;
  if ((long long)p.S * p.stride >= (1LL << 32) || (long long)p.S * p.stride_res >= (1LL << 32)) return VQ_ERR_UNSUPPORTED;
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  const size_t main = up16((size_t)p.k * p.v * 2), res = up16((size_t)p.k_res * p.v * 2);
  DqLdsPlan plan{};
  plan.both = p.k_res && main + res <= 160 * 1024;
  plan.off_res = (unsigned)main;
  plan.res_global = p.k_res && !plan.both && main <= 160 * 1024 && switches().dequant != 's';
  plan.bytes = (unsigned)(plan.both ? main + res : plan.res_global ? main : main > res ? main : res);
  if (plan.bytes > 160u * 1024u) return VQ_ERR_UNSUPPORTED;
  const int wgs = cu_count();
  plan.rows_per_wg = (p.S + wgs - 1) / wgs;                 // streams per workgroup
  if (plan.rows_per_wg < 1) plan.rows_per_wg = 1;
  // (pairs of columns as dwords: every group has to start on an even column)
  const bool a4 = (reinterpret_cast<uintptr_t>(W) & 3) == 0 && (ldw & 1) == 0 && (p.n_out & 1) == 0 && (p.n_groups == 1 || (p.Pg & 1) == 0);
#define VQ_PAIR(V, BITS) if (p.v == V && p.bits == BITS) return launch_down_vb<V, BITS>(p, plan, a4, W, ldw, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

}  // namespace vq
