// vq_gemv for the layers that have no kernel of their own but whose tables fit LDS: any vector length, any table sizes and
// index widths, residual and outlier tables, a column permutation -- the paper's other (v, k) settings (App. "Impact of
// Vector Length": v = 2 / k = 16, v = 4 / k = 256; Table "Quantization parameters") -- one to four activation rows a launch.
// (App. "Our Dequantization Implementation", decode phase: restore and multiply fused, the tables in fast memory.)
//
// One 1024-thread workgroup per compute unit owns a block of output rows.  Tables go into LDS as they are ([k][v] halves),
// the activation rows too, gathered into stored column order on the way when the layer has a column permutation, so the
// row loop never sees it.  A wave takes a row at a time; its lanes stride over the row's vectors, read their indices from
// the packed streams (two dwords and a shift), look the centroids up in LDS and accumulate d * x in binary32 -- in pairs
// with v_dot2_f32_f16 when vectors start on even columns, else element by element -- and the row ends in
// y = scale * sum(d x) + bias * sum(x), as in the other decode kernels.  No layout tricks: this kernel's job is to keep
// every such layer off the generic kernel, whose table reads go through the caches (about 90 GB/s).
#include "vq_lds_tables.hpp"

namespace vq {

namespace {

using namespace lds_tables;

constexpr int LW = 16;           // waves per workgroup

struct LdsPlan {
  unsigned off_res, off_out, off_x, off_xsum, off_ypart, bytes;   // byte offsets in dynamic LDS (main table at 0)
  int rows_per_wg;
  unsigned x_pitch;                                    // bytes per staged activation row
};

template <int B>
__global__ __launch_bounds__(LW * 64) void gemv_lds_kernel(Params p, LdsPlan plan, const __half *__restrict__ x, long long ldx,
                                                           __half *__restrict__ y, long long ldy) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const __half *T = reinterpret_cast<const __half *>(lds);
  const __half *Tr = reinterpret_cast<const __half *>(lds + plan.off_res);
  const __half *To = reinterpret_cast<const __half *>(lds + plan.off_out);
  float *xsum = reinterpret_cast<float *>(lds + plan.off_xsum);          // [B], then the waves' parts [B][LW]
  float *xpart = xsum + B;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;

  // ---- tables and activations into LDS
  {
    __half *dst = reinterpret_cast<__half *>(lds);
    const int n_main = p.k * p.v, n_res = p.k_res * p.v, n_out = p.k_out * p.v_out;
    for (int e = threadIdx.x; e < n_main; e += LW * 64) dst[e] = p.cb[e];
    dst = reinterpret_cast<__half *>(lds + plan.off_res);
    for (int e = threadIdx.x; e < n_res; e += LW * 64) dst[e] = p.cb_res[e];
    dst = reinterpret_cast<__half *>(lds + plan.off_out);
    for (int e = threadIdx.x; e < n_out; e += LW * 64) dst[e] = p.cb_out[e];
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < B; ++t) {
    __half *xs = reinterpret_cast<__half *>(lds + plan.off_x + t * plan.x_pitch);
    float part = 0.0f;
    for (int c = threadIdx.x; c < p.in_features; c += LW * 64) {
      int src = c;
      if (p.perm) src = p.perm[c];                      // stored column c meets x[perm[c]] (Sec. 3.2.3); entries outside the row count as zero
      const __half v = (unsigned)src < (unsigned)p.in_features ? x[(long long)t * ldx + src] : __float2half_rn(0.0f);
      xs[c] = v;
      part += __half2float(v);
    }
    // (the pad of the last vector: zeros)
    for (int c = p.in_features + threadIdx.x; c < (int)(plan.x_pitch / 2); c += LW * 64) xs[c] = __float2half_rn(0.0f);
    part = wave_sum(part);
    if (lane == 0) xpart[t * LW + wv] = part;
  }
  __syncthreads();
  if (threadIdx.x < B) {                                  // the waves' parts in a fixed order: the same bits every run
    float sum = 0.0f;
    for (int w = 0; w < LW; ++w) sum += xpart[threadIdx.x * LW + w];
    xsum[threadIdx.x] = sum;
  }
  __syncthreads();

  const int row0 = blockIdx.x * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const bool pairs = (p.v % 2 == 0) && (p.n_out % 2 == 0) && (p.v_out % 2 == 0 || p.Q == 0);   // every vector starts on an even column
  for (int o = row0 + wv; o < row1; o += LW) {
    float acc[B];
#pragma unroll
    for (int t = 0; t < B; ++t) acc[t] = 0.0f;
    const uint8_t *ri = p.idx + (long long)o * p.stride;
    const uint8_t *rr = p.k_res ? p.idx_res + (long long)o * p.stride_res : ri, *ro = p.Q ? p.idx_out + (long long)o * p.stride_out : ri;
    for (int slot = lane; slot < p.Q + p.P; slot += 64) {
      const __half *e, *er = nullptr;
      int c0, len;
      if (slot < p.Q) {
        const unsigned i = min(load_index(ro, slot, p.bits_out), (unsigned)p.k_out - 1u);
        e = To + i * p.v_out; c0 = slot * p.v_out; len = p.v_out;
      } else {
        const int pp = slot - p.Q;
        const unsigned i = min(load_index(ri, pp, p.bits), (unsigned)p.k - 1u);
        e = T + i * p.v;
        if (p.k_res) er = Tr + min(load_index(rr, pp, p.bits_res), (unsigned)p.k_res - 1u) * p.v;
        c0 = p.n_out + pp * p.v; len = p.v;             // (columns past in_features meet zeros in the staged row)
      }
      if (pairs) {
        for (int j = 0; j < len; j += 2) {
          const unsigned d = *reinterpret_cast<const unsigned *>(e + j);
          const unsigned r = er ? *reinterpret_cast<const unsigned *>(er + j) : 0u;
#pragma unroll
          for (int t = 0; t < B; ++t) {
            const unsigned xv = *reinterpret_cast<const unsigned *>(lds + plan.off_x + t * plan.x_pitch + (unsigned)(c0 + j) * 2u);
            acc[t] = dot2(d, xv, acc[t]);
            if (er) acc[t] = dot2(r, xv, acc[t]);
          }
        }
      } else {
        for (int j = 0; j < len; ++j) {
          float d = __half2float(e[j]);
          if (er) d = __fadd_rn(d, __half2float(er[j]));
#pragma unroll
          for (int t = 0; t < B; ++t)
            acc[t] = __fmaf_rn(d, __half2float(*reinterpret_cast<const __half *>(lds + plan.off_x + t * plan.x_pitch + (unsigned)(c0 + j) * 2u)), acc[t]);
        }
      }
    }
    const float s = p.scale ? __half2float(p.scale[o]) : 1.0f, b = p.bias ? __half2float(p.bias[o]) : 0.0f;
#pragma unroll
    for (int t = 0; t < B; ++t) {
      const float r = wave_sum(acc[t]);
      if (lane == 0) y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(s, r, b * xsum[t]));
    }
  }
}


// The same for the settings of the paper's tables when there are no outlier columns: vector length V and index width BITS
// (main and residual streams alike) fixed at compile time.  A lane takes a whole window of its row's index stream at a
// time -- 32 / gcd(32, BITS) vectors in BITS / gcd(32, BITS) dwords, consecutive lanes consecutive windows: one coalesced,
// range-checked load per window instead of two dwords per index -- and the table entries sit in LDS padded to 4, 8, 16 or
// 32 bytes, so that an entry is one aligned read (two for V = 12).
constexpr bool two_pass_compiled(int v, int bits) { return v >= 8 && bits == 12; }   // where two padded tables can exceed LDS

template <int V, int BITS, int MODE, int B>      // MODE 0: no residual; 1: both tables in LDS; 2: one table at a time, two passes over the rows
__global__ __launch_bounds__(LW * 64) void gemv_lds_window_kernel(Params p, LdsPlan plan, const __half *__restrict__ x, long long ldx,
                                                                  __half *__restrict__ y, long long ldy) {
  constexpr int U = win_vectors(BITS), ND = U * BITS / 32, EH = entry_halfs(V), ED = EH / 2, VD = V / 2;
  constexpr bool BOTH = MODE == 1;
  constexpr int PASSES = MODE == 2 ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  float *xsum = reinterpret_cast<float *>(lds + plan.off_xsum);          // [B], then the waves' parts [B][LW]
  float *xpart = xsum + B;
  float *ypart = reinterpret_cast<float *>(lds + plan.off_ypart);        // MODE 2: the first pass's row sums [rows_per_wg][B]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;

  const int row0 = blockIdx.x * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const int windows = (p.P + U - 1) / U;
  const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.out_features * p.stride), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(MODE ? p.idx_res : p.idx), 0,
                                                                       MODE ? (unsigned)((long long)p.out_features * p.stride_res) : 0u, 0x00020000);
  // The wave's rows go 64 windows at a time (`ipr` rounds a row), and the windows of the next round are loaded before the
  // current ones are used, so that a row's trip to memory hides behind the row before it; the first round's go out here,
  // ahead of the staging.  A round past the row's windows or past the wave's rows loads from an offset outside the buffer
  // (zeros, never looked at).
  const int ipr = (windows + 63) >> 6;
  auto offset_of = [&](int o, int it, unsigned stride) {
    const int w = lane + it * 64;
    return o < row1 && w < windows ? (unsigned)o * stride + (unsigned)w * (ND * 4u) : 0xFFFFFFF0u;
  };
  unsigned wm[ND], wr[ND];
  float s_row = 1.0f, b_row = 0.0f;                                       // scale and bias of the current row, loaded ahead like the windows
  auto first_loads = [&](bool second) {
    const int o = row0 + wv;
    load_window<ND>(wm, second ? r_r : r_i, offset_of(o, 0, (unsigned)(second ? p.stride_res : p.stride)));
    if (BOTH) load_window<ND>(wr, r_r, offset_of(o, 0, (unsigned)p.stride_res));
    s_row = 1.0f; b_row = 0.0f;
    if (o < row1) {
      if (p.scale) s_row = __half2float(p.scale[o]);
      if (p.bias) b_row = __half2float(p.bias[o]);
    }
  };
  first_loads(false);

  // ---- activations into LDS as in the kernel above (windows of U * V columns side by side: a lane's reads of consecutive
  // columns stay aligned and wide; an odd pitch per window, tried against bank conflicts, made them narrow and twice as slow)
#pragma unroll
  for (int t = 0; t < B; ++t) {
    __half *xs = reinterpret_cast<__half *>(lds + plan.off_x + t * plan.x_pitch);
    float part = 0.0f;
    for (int c = threadIdx.x; c < p.in_features; c += LW * 64) {
      int src = c;
      if (p.perm) src = p.perm[c];
      const __half v = (unsigned)src < (unsigned)p.in_features ? x[(long long)t * ldx + src] : __float2half_rn(0.0f);
      xs[c] = v;
      part += __half2float(v);
    }
    for (int c = p.in_features + threadIdx.x; c < (int)(plan.x_pitch / 2); c += LW * 64) xs[c] = __float2half_rn(0.0f);
    part = wave_sum(part);
    if (lane == 0) xpart[t * LW + wv] = part;
  }
  __syncthreads();
  if (threadIdx.x < B) {
    float sum = 0.0f;
    for (int w = 0; w < LW; ++w) sum += xpart[threadIdx.x * LW + w];
    xsum[threadIdx.x] = sum;
  }

  for (int pass = 0; pass < PASSES; ++pass) {
    // ---- this pass's table(s) into LDS as padded entries (zero past the table's last entry and in the pad)
    const bool second = pass == 1;                                        // (MODE 2 only) the residual table takes the main table's place
    const int k_a = second ? p.k_res : p.k;
    const __half *cb_a = second ? p.cb_res : p.cb;
    if (second) {
      first_loads(true);
      __syncthreads();                                                    // every wave has left the first pass's table
    }
    // (an entry per thread and round: its V / 2 dwords loaded together, stored as one padded entry; four rounds in flight)
#pragma unroll 4
    for (int en = threadIdx.x; en < k_a + (BOTH ? p.k_res : 0); en += LW * 64) {
      const bool res = BOTH && en >= k_a;
      if (res) stage_entry<V>(lds + plan.off_res, p.cb_res, en - k_a);
      else stage_entry<V>(lds, cb_a, en);
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t r_a = second ? r_r : r_i;
    const unsigned stride_a = (unsigned)(second ? p.stride_res : p.stride);
    int o = row0 + wv, it = 0;
    float acc[B];
#pragma unroll
    for (int t = 0; t < B; ++t) acc[t] = 0.0f;
    while (o < row1) {
      int on = o, itn = it + 1;
      if (itn == ipr) { itn = 0; on = o + LW; }
      float s_next = s_row, b_next = b_row;
      if (itn == 0 && on < row1) {
        if (p.scale) s_next = __half2float(p.scale[on]);
        if (p.bias) b_next = __half2float(p.bias[on]);
      }
      unsigned nm[ND], nr[ND];
      load_window<ND>(nm, r_a, offset_of(on, itn, stride_a));
      if (BOTH) load_window<ND>(nr, r_r, offset_of(on, itn, (unsigned)p.stride_res));
      const int wdx = lane + it * 64;
      if (wdx < windows) {
        const unsigned xbase = plan.off_x + (unsigned)wdx * (U * V * 2u);          // the window's U * V columns of the staged rows
#pragma unroll
        for (int u = 0; u < U; ++u) {
          // (a vector past the row's last one: some entry of the table times the zeros that end the staged row)
          const unsigned i = min(window_field<BITS, ND>(wm, u), (unsigned)k_a - 1u);
          unsigned e[ED], f[ED];
          read_entry<V>(e, lds, i);
          if (BOTH) {
            const unsigned ir = min(window_field<BITS, ND>(wr, u), (unsigned)p.k_res - 1u);
            read_entry<V>(f, lds + plan.off_res, ir);
          }
#pragma unroll
          for (int t = 0; t < B; ++t) {
#pragma unroll
            for (int d = 0; d < VD; ++d) {
              const unsigned xv = *reinterpret_cast<const unsigned *>(lds + xbase + t * plan.x_pitch + (unsigned)(u * V + 2 * d) * 2u);
              acc[t] = dot2(e[d], xv, acc[t]);
              if (BOTH) acc[t] = dot2(f[d], xv, acc[t]);
            }
          }
        }
      }
      if (itn == 0) {                                                     // the row is complete
        const float s = s_row, b = b_row;
#pragma unroll
        for (int t = 0; t < B; ++t) {
          float r = segment_sum_to_last(acc[t], 64);
          acc[t] = 0.0f;
          if (lane == 63) {
            if (MODE == 2 && !second) ypart[(o - row0) * B + t] = r;       // the same lane of the same wave picks it up in the second pass
            else {
              if (MODE == 2) r = __fadd_rn(ypart[(o - row0) * B + t], r);
              y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(s, r, b * xsum[t]));
            }
          }
        }
      }
#pragma unroll
      for (int d = 0; d < ND; ++d) { wm[d] = nm[d]; if (BOTH) wr[d] = nr[d]; }
      o = on; it = itn; s_row = s_next; b_row = b_next;
    }
  }
}

// (two_pass: the residual table takes the main table's place for a second pass over the rows, whose first-pass sums wait in LDS)
bool make_window_plan(const Params &p, int batch, int u, int eh, bool two_pass, LdsPlan *plan) {
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  const size_t main = up16((size_t)p.k * eh * 2), res = up16((size_t)p.k_res * eh * 2);
  const size_t tables = two_pass ? (main > res ? main : res) : main + res;
  const size_t windows = ((size_t)p.P + u - 1) / u;
  const size_t pitch = up16(windows * u * p.v * 2);
  const int wgs = cu_count();
  plan->rows_per_wg = (p.out_features + wgs - 1) / wgs;
  if (plan->rows_per_wg < LW) plan->rows_per_wg = LW;
  const size_t sums = up16(4 * 4 * (1 + LW));
  const size_t total = tables + pitch * batch + sums + (two_pass ? (size_t)plan->rows_per_wg * batch * 4 : 0);
  if (total > 160 * 1024) return false;
  if ((long long)p.out_features * p.stride >= (1LL << 32) || (long long)p.out_features * p.stride_res >= (1LL << 32)) return false;
  plan->off_res = (unsigned)main; plan->off_out = (unsigned)tables; plan->off_x = (unsigned)tables;
  plan->off_xsum = (unsigned)(tables + pitch * batch); plan->off_ypart = (unsigned)(tables + pitch * batch + sums);
  plan->bytes = (unsigned)total; plan->x_pitch = (unsigned)pitch;
  return true;
}

template <int V, int BITS, int MODE, int B>
int launch_window(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  LdsPlan plan;
  if (!make_window_plan(p, B, win_vectors(BITS), entry_halfs(V), MODE == 2, &plan)) return VQ_ERR_UNSUPPORTED;
  auto kernel = gemv_lds_window_kernel<V, BITS, MODE, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int V, int BITS>
int launch_window_vb(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (batch != 1 && batch != 2 && batch != 4) return VQ_ERR_UNSUPPORTED;
  if (p.k_res == 0)
    return batch == 1 ? launch_window<V, BITS, 0, 1>(p, x, ldx, y, ldy, s) : batch == 2 ? launch_window<V, BITS, 0, 2>(p, x, ldx, y, ldy, s)
                                                                                         : launch_window<V, BITS, 0, 4>(p, x, ldx, y, ldy, s);
  int rc = batch == 1 ? launch_window<V, BITS, 1, 1>(p, x, ldx, y, ldy, s) : batch == 2 ? launch_window<V, BITS, 1, 2>(p, x, ldx, y, ldy, s)
                                                                                          : launch_window<V, BITS, 1, 4>(p, x, ldx, y, ldy, s);
  if (rc != VQ_ERR_UNSUPPORTED) return rc;
  // both tables do not fit: one after the other (v = 12 with two 4096-entry tables, Table "Quantization parameters")
  if constexpr (!two_pass_compiled(V, BITS)) return VQ_ERR_UNSUPPORTED;
  else return batch == 1 ? launch_window<V, BITS, 2, 1>(p, x, ldx, y, ldy, s) : batch == 2 ? launch_window<V, BITS, 2, 2>(p, x, ldx, y, ldy, s)
                                                                                        : launch_window<V, BITS, 2, 4>(p, x, ldx, y, ldy, s);
}

// the (V, BITS) pairs with a compiled kernel: no outlier columns, a residual stream (if any) of the same index width
bool window_pair(const Params &p) {
  if (p.Q != 0 || (p.k_res && p.bits_res != p.bits)) return false;
  return compiled_pair(p.v, p.bits, false);
}
int launch_window_any(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (p.Q != 0 || (p.k_res && p.bits_res != p.bits)) return VQ_ERR_UNSUPPORTED;
#define VQ_PAIR(V, BITS) if (p.v == V && p.bits == BITS) return launch_window_vb<V, BITS>(p, x, ldx, batch, y, ldy, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

// The layers of the paper's 2.07- to 2.26-bit settings (Table "Quantization parameters": v = 12 with two 4096-entry tables,
// 1 % outlier columns of v = 4, one to sixteen codebook groups) and whatever else the kernels above refuse for outlier
// columns, codebook groups (Sec. 3.1) or size: one table in LDS at a time.  A pass is (group, main or residual table) or the
// outlier table; the workgroup stages the pass's table (and, where groups differ, the activations with zeros outside the
// group's columns, so that a window that straddles two groups needs no masks), walks its rows over the pass's windows, and
// adds the row sums to those of the passes before, which wait in LDS; the dot product is linear in the sum of centroids, so
// y = scale * (sum of the passes) + bias * sum(x).  Outlier vectors have v_out = 4 and any index width.
struct PassPlan {
  unsigned off_x, off_xo, off_xsum, off_ypart, bytes;     // byte offsets in dynamic LDS (the pass's table at 0)
  unsigned x_pitch, xo_pitch;                             // bytes per staged row of main / outlier columns
  int rows_per_wg;
  // With a workspace on loan a workgroup takes one "slot" -- a codebook group (its main and residual table; the first group's
  // workgroups also the outlier columns) -- and a block of rows, and leaves its sums in the workspace for the kernel that adds
  // the slots up:
  int n_slots, batch_total;                               // 0: every workgroup walks all passes and writes y
  float *part, *part_xs;                                  // [n_slots][batch_total][out_features] sums, [n_slots][16] activation sums
};

template <int V, int BITS, int B>
__global__ __launch_bounds__(LW * 64) void gemv_lds_passes_kernel(Params p, PassPlan plan, const __half *__restrict__ x, long long ldx,
                                                                  __half *__restrict__ y, long long ldy) {
  constexpr int U = win_vectors(BITS), ND = U * BITS / 32, EH = entry_halfs(V), ED = EH / 2, VD = V / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  float *xsum = reinterpret_cast<float *>(lds + plan.off_xsum);          // [B], then the waves' parts [B][LW]
  float *xpart = xsum + B;
  float *ypart = reinterpret_cast<float *>(lds + plan.off_ypart);        // row sums of the passes so far [rows_per_wg][B]
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const bool slots = plan.n_slots != 0;
  const int slot = slots ? (int)blockIdx.x % plan.n_slots : 0;
  const int row0 = (slots ? (int)blockIdx.x / plan.n_slots : (int)blockIdx.x) * plan.rows_per_wg;
  const int row1 = min(p.out_features, row0 + plan.rows_per_wg);
  const int windows = (p.P + U - 1) / U;
  const __amdgpu_buffer_rsrc_t r_i = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.idx), 0, (unsigned)((long long)p.out_features * p.stride), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.k_res ? p.idx_res : p.idx), 0,
                                                                       p.k_res ? (unsigned)((long long)p.out_features * p.stride_res) : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_o = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.Q ? p.idx_out : p.idx), 0,
                                                                       p.Q ? (unsigned)((long long)p.out_features * p.stride_out) : 0u, 0x00020000);
  auto x_at = [&](int t, int c) {                         // activation of stored column c (Sec. 3.2.3), zero outside the row
    int src = c;
    if (p.perm) src = p.perm[c];
    return (unsigned)src < (unsigned)p.in_features ? x[(long long)t * ldx + src] : __float2half_rn(0.0f);
  };

  // ---- once: the activations of the outlier columns and their sum (with slots: the first slot's workgroups only); the main
  // columns are added to the sums as the passes restage them
  const int once_cols = slot == 0 ? p.n_out : 0;
#pragma unroll
  for (int t = 0; t < B; ++t) {
    __half *xo = reinterpret_cast<__half *>(lds + plan.off_xo + t * plan.xo_pitch);
    float part = 0.0f;
    for (int c = threadIdx.x; c < once_cols; c += LW * 64) {
      const __half v = x_at(t, c);
      if (c < p.n_out) xo[c] = v;
      part += __half2float(v);
    }
    part = wave_sum(part);
    if (lane == 0) xpart[t * LW + wv] = part;
  }

  const int tables_per_group = p.k_res ? 2 : 1;
  const int table_passes = p.n_groups * tables_per_group;
  const int pass_begin = slots ? slot * tables_per_group : 0;
  const int my_table_passes = slots ? tables_per_group : table_passes;
  const int my_passes = my_table_passes + (p.Q && slot == 0 ? 1 : 0);
  for (int ip = 0; ip < my_passes; ++ip) {
    const int pass = ip < my_table_passes ? pass_begin + ip : table_passes;
    const bool outlier = pass == table_passes;
    const int g = pass / tables_per_group;
    const bool second = !outlier && pass - g * tables_per_group == 1;
    // the pass's vectors [p_lo, p_hi) of the row, its windows [w_lo, w_hi) (outlier pass: its Q vectors, one per "window")
    const int p_lo = outlier ? 0 : g * p.Pg, p_hi = outlier ? p.Q : min(p.P, p_lo + p.Pg);
    const int w_lo = outlier ? 0 : p_lo / U, w_hi = outlier ? p.Q : (p_hi + U - 1) / U;
    // few windows (a narrow codebook group, the outlier vectors): segments of SEG lanes take a row each, 64 / SEG rows a round
    const int nw = w_hi - w_lo;
    const int SEG = nw > 32 ? 64 : nw > 16 ? 32 : nw > 8 ? 16 : 8;
    // (a wave's segments take consecutive rows, so that a block of few rows keeps few waves busy instead of a segment of each)
    const int lane_w = lane & (SEG - 1), row_step = (64 / SEG) * LW;
    const int o_lane_off = lane / SEG;                                    // this lane's row within the round's rows
    const int ipr = max((nw + 63) >> 6, 1);
    const int k_a = outlier ? p.k_out : second ? p.k_res : p.k;
    const __half *cb_a = outlier ? p.cb_out : second ? p.cb_res + (long long)g * p.k_res * V : p.cb + (long long)g * p.k * V;
    const __amdgpu_buffer_rsrc_t r_a = outlier ? r_o : second ? r_r : r_i;
    const unsigned stride_a = (unsigned)(outlier ? p.stride_out : second ? p.stride_res : p.stride);
    // index words of a round: a window of U vectors (ND dwords), or the two dwords that hold an outlier index
    auto offset_of = [&](int o, int it) {
      const int w = w_lo + lane_w + it * 64;
      o += o_lane_off;
      if (!(o < row1 && w < w_hi)) return 0xFFFFFFF0u;
      return (unsigned)o * stride_a + (outlier ? (((unsigned)w * (unsigned)p.bits_out) >> 5) * 4u : (unsigned)w * (ND * 4u));
    };
    auto load_round = [&](unsigned (&w)[ND < 2 ? 2 : ND], int o, int it) {
      const unsigned off = offset_of(o, it);
      if (outlier) {
        const uint2v a = __builtin_amdgcn_raw_buffer_load_b64(r_a, off, 0, 0);
        w[0] = a.x; w[1] = a.y;
      } else {
        unsigned v[ND];
        load_window<ND>(v, r_a, off);
#pragma unroll
        for (int d = 0; d < ND; ++d) w[d] = v[d];
      }
    };
    int o = row0 + wv * (64 / SEG), it = 0;
    unsigned wm[ND < 2 ? 2 : ND];
    load_round(wm, o, 0);                                                 // the first round's words go out ahead of the staging

    __syncthreads();                                                      // every wave has left the table and rows of the pass before
    // ---- the pass's table into LDS: padded entries, an entry per thread and round (outlier entries: 8 bytes as they are)
    if (outlier) {
      for (int en = threadIdx.x; en < k_a; en += LW * 64)
        *reinterpret_cast<uint2v *>(lds + (unsigned)en * 8u) = *reinterpret_cast<const uint2v *>(cb_a + (long long)en * 4);
    } else {
#pragma unroll 4
      for (int en = threadIdx.x; en < k_a; en += LW * 64) stage_entry<V>(lds, cb_a, en);
    }
    // ---- the activations of the pass's windows: a new group's, with zeros outside the group (and past the row)
    if (!outlier && !second) {
#pragma unroll
      for (int t = 0; t < B; ++t) {
        __half *xs = reinterpret_cast<__half *>(lds + plan.off_x + t * plan.x_pitch);
        float part = 0.0f;
        for (int j = w_lo * (U * V) + (int)threadIdx.x; j < w_hi * (U * V); j += LW * 64) {
          const int c = p.n_out + j, pv = j / V;
          const __half v = pv >= p_lo && pv < p_hi && c < p.in_features ? x_at(t, c) : __float2half_rn(0.0f);
          xs[j] = v;
          part += __half2float(v);
        }
        part = wave_sum(part);                                            // the group's share of sum(x)
        if (lane == 0) xpart[t * LW + wv] += part;
      }
    }
    __syncthreads();

    // ---- the wave's rows, 64 windows a round, the next round's words loaded before the current ones are used
    float acc[B];
#pragma unroll
    for (int t = 0; t < B; ++t) acc[t] = 0.0f;
    while (o < row1) {
      int on = o, itn = it + 1;
      if (itn == ipr) { itn = 0; on = o + row_step; }
      unsigned nm[ND < 2 ? 2 : ND];
      load_round(nm, on, itn);
      const int wdx = w_lo + lane_w + it * 64;
      if (wdx < w_hi && o + o_lane_off < row1) {
        if (outlier) {
          const unsigned sh = ((unsigned)wdx * (unsigned)p.bits_out) & 31u;
          unsigned i = wm[0] >> sh;
          if (sh + (unsigned)p.bits_out > 32u) i |= wm[1] << (32u - sh);
          i = min(i & ((1u << p.bits_out) - 1u), (unsigned)k_a - 1u);
          const uint2v e = *reinterpret_cast<const uint2v *>(lds + i * 8u);
#pragma unroll
          for (int t = 0; t < B; ++t) {
            const uint2v xv = *reinterpret_cast<const uint2v *>(lds + plan.off_xo + t * plan.xo_pitch + (unsigned)wdx * 8u);
            acc[t] = dot2(e.x, xv.x, acc[t]);
            acc[t] = dot2(e.y, xv.y, acc[t]);
          }
        } else {
          const unsigned xbase = plan.off_x + (unsigned)wdx * (U * V * 2u);
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const unsigned i = min(window_field<BITS, ND < 2 ? 2 : ND>(wm, u), (unsigned)k_a - 1u);
            unsigned e[ED];
            read_entry<V>(e, lds, i);
#pragma unroll
            for (int t = 0; t < B; ++t) {
#pragma unroll
              for (int d = 0; d < VD; ++d) {
                const unsigned xv = *reinterpret_cast<const unsigned *>(lds + xbase + t * plan.x_pitch + (unsigned)(u * V + 2 * d) * 2u);
                acc[t] = dot2(e[d], xv, acc[t]);
              }
            }
          }
        }
      }
      if (itn == 0) {                                                     // the row's part of this pass is complete
#pragma unroll
        for (int t = 0; t < B; ++t) {
          const float r = segment_sum_to_last(acc[t], SEG);
          acc[t] = 0.0f;
          if (lane_w == SEG - 1 && o + o_lane_off < row1) {                     // (a row changes hands between passes; barriers lie between)
            float *yp = ypart + (o + o_lane_off - row0) * B + t;
            *yp = pass != pass_begin ? __fadd_rn(*yp, r) : r;
          }
        }
      }
#pragma unroll
      for (int d = 0; d < (ND < 2 ? 2 : ND); ++d) wm[d] = nm[d];
      o = on; it = itn;
    }
  }
  // ---- scale, bias, store: a lane per row
  __syncthreads();
  if (threadIdx.x < B) {                                                  // the waves' parts of sum(x) in a fixed order
    float sum = 0.0f;
    for (int w = 0; w < LW; ++w) sum += xpart[threadIdx.x * LW + w];
    xsum[threadIdx.x] = sum;
  }
  __syncthreads();
  if (slots) {
    for (int r = threadIdx.x; r < row1 - row0; r += LW * 64)
#pragma unroll
      for (int t = 0; t < B; ++t) plan.part[((long long)slot * plan.batch_total + t) * p.out_features + row0 + r] = ypart[r * B + t];
    if (row0 == 0 && threadIdx.x < B) plan.part_xs[slot * 16 + threadIdx.x] = xsum[threadIdx.x];
    return;
  }
  for (int r = threadIdx.x; r < row1 - row0; r += LW * 64) {
    const int o = row0 + r;
    const float s = p.scale ? __half2float(p.scale[o]) : 1.0f, b = p.bias ? __half2float(p.bias[o]) : 0.0f;
#pragma unroll
    for (int t = 0; t < B; ++t) y[(long long)t * ldy + o] = __float2half_rn(__fmaf_rn(s, ypart[r * B + t], b * xsum[t]));
  }
}

bool make_pass_plan(const Params &p, int batch, int u, int eh, PassPlan *plan, int n_slots = 0) {
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  size_t table = up16((size_t)p.k * eh * 2);
  if (up16((size_t)p.k_res * eh * 2) > table) table = up16((size_t)p.k_res * eh * 2);
  if (p.Q && up16((size_t)p.k_out * 8) > table) table = up16((size_t)p.k_out * 8);
  const size_t windows = ((size_t)p.P + u - 1) / u;
  const size_t pitch = up16(windows * u * p.v * 2), xo_pitch = up16((size_t)p.n_out * 2);
  const int wgs = n_slots ? (cu_count() / n_slots > 0 ? cu_count() / n_slots : 1) : cu_count();     // workgroups per slot
  plan->rows_per_wg = (p.out_features + wgs - 1) / wgs;
  if (plan->rows_per_wg < LW) plan->rows_per_wg = LW;
  plan->n_slots = n_slots; plan->batch_total = 0; plan->part = nullptr; plan->part_xs = nullptr;
  const size_t sums = up16(4 * 4 * (1 + LW));
  const size_t total = table + (pitch + xo_pitch) * batch + sums + (size_t)plan->rows_per_wg * batch * 4;
  if (total > 160 * 1024) return false;
  if ((long long)p.out_features * p.stride >= (1LL << 32) || (long long)p.out_features * p.stride_res >= (1LL << 32) ||
      (long long)p.out_features * p.stride_out >= (1LL << 32)) return false;
  plan->off_x = (unsigned)table; plan->off_xo = (unsigned)(table + pitch * batch);
  plan->off_xsum = (unsigned)(table + (pitch + xo_pitch) * batch); plan->off_ypart = plan->off_xsum + (unsigned)sums;
  plan->bytes = (unsigned)total; plan->x_pitch = (unsigned)pitch; plan->xo_pitch = (unsigned)xo_pitch;
  return true;
}

// layers the pass kernel takes: a compiled (V, BITS) pair, a residual stream of the same width, outlier vectors of four
bool pass_pair(const Params &p) {
  if ((p.k_res && p.bits_res != p.bits) || (p.Q && (p.v_out != 4 || p.bits_out > 16))) return false;
  return compiled_pair(p.v, p.bits, true);
}

template <int V, int BITS, int B>
int launch_passes(const Params &p, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  PassPlan plan;
  if (!make_pass_plan(p, B, win_vectors(BITS), entry_halfs(V), &plan)) return VQ_ERR_UNSUPPORTED;
  auto kernel = gemv_lds_passes_kernel<V, BITS, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

template <int V, int BITS, int B>
int launch_slots(const Params &p, const __half *x, long long ldx, int n_slots, int batch_total, float *part, float *part_xs, hipStream_t s) {
  PassPlan plan;
  if (!make_pass_plan(p, B, win_vectors(BITS), entry_halfs(V), &plan, n_slots)) return VQ_ERR_UNSUPPORTED;
  plan.batch_total = batch_total; plan.part = part; plan.part_xs = part_xs;
  auto kernel = gemv_lds_passes_kernel<V, BITS, B>;
  VQ_ALLOW_FULL_LDS(kernel);
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg) * (unsigned)n_slots;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, static_cast<__half *>(nullptr), 0LL);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

int launch_slots_any(const Params &p, const __half *x, long long ldx, int batch, int n_slots, int batch_total, float *part, float *part_xs,
                     hipStream_t s) {
  if (!pass_pair(p) || (batch != 1 && batch != 2 && batch != 4)) return VQ_ERR_UNSUPPORTED;
#define VQ_PAIR(V, BITS)                                                                                                     \
  if (p.v == V && p.bits == BITS)                                                                                            \
    return batch == 1   ? launch_slots<V, BITS, 1>(p, x, ldx, n_slots, batch_total, part, part_xs, s)                         \
           : batch == 2 ? launch_slots<V, BITS, 2>(p, x, ldx, n_slots, batch_total, part, part_xs, s)                         \
                        : launch_slots<V, BITS, 4>(p, x, ldx, n_slots, batch_total, part, part_xs, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(6, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

int launch_passes_any(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (!pass_pair(p) || (batch != 1 && batch != 2 && batch != 4)) return VQ_ERR_UNSUPPORTED;
#define VQ_PAIR(V, BITS)                                                                                              \
  if (p.v == V && p.bits == BITS)                                                                                     \
    return batch == 1 ? launch_passes<V, BITS, 1>(p, x, ldx, y, ldy, s) : batch == 2 ? launch_passes<V, BITS, 2>(p, x, ldx, y, ldy, s) \
                                                                                     : launch_passes<V, BITS, 4>(p, x, ldx, y, ldy, s);
  VQ_PAIR(2, 4) VQ_PAIR(4, 8) VQ_PAIR(6, 8) VQ_PAIR(8, 8) VQ_PAIR(4, 12) VQ_PAIR(6, 12) VQ_PAIR(8, 12) VQ_PAIR(12, 12)
#undef VQ_PAIR
  return VQ_ERR_UNSUPPORTED;
}

bool make_plan(const Params &p, int batch, LdsPlan *plan) {
  auto up16 = [](size_t v) { return (v + 15) / 16 * 16; };
  const size_t main = up16((size_t)p.k * p.v * 2), res = up16((size_t)p.k_res * p.v * 2), out = up16((size_t)p.k_out * p.v_out * 2);
  // a staged row covers every column a vector can name: the outlier columns, then P whole vectors
  const size_t pitch = up16(((size_t)p.n_out + (size_t)p.P * p.v) * 2);
  const size_t total = main + res + out + pitch * batch + 4 * 4 * (1 + LW);
  if (total > 160 * 1024) return false;
  plan->off_res = (unsigned)main; plan->off_out = (unsigned)(main + res); plan->off_x = (unsigned)(main + res + out);
  plan->off_xsum = (unsigned)(main + res + out + pitch * batch); plan->bytes = (unsigned)total; plan->x_pitch = (unsigned)pitch;
  const int wgs = cu_count();
  plan->rows_per_wg = (p.out_features + wgs - 1) / wgs;
  if (plan->rows_per_wg < LW) plan->rows_per_wg = LW;       // at least a row per wave
  return true;
}

template <int B>
int launch_b(const Params &p, const LdsPlan &plan, const __half *x, long long ldx, __half *y, long long ldy, hipStream_t s) {
  VQ_ALLOW_FULL_LDS(gemv_lds_kernel<B>);
  const unsigned grid = (unsigned)((p.out_features + plan.rows_per_wg - 1) / plan.rows_per_wg);
  hipLaunchKernelGGL(gemv_lds_kernel<B>, dim3(grid), dim3(LW * 64), plan.bytes, s, p, plan, x, ldx, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

}  // namespace

// Vectors along the rows, one codebook group, tables and `batch` activation rows within LDS.
bool gemv_lds_applicable(const Params &p, int batch) {
  LdsPlan plan;
  PassPlan pplan;
  if (p.orientation != 0) return false;
  if (p.n_groups == 1) {
    if (make_plan(p, batch, &plan)) return true;
    if (window_pair(p) && (batch == 1 || batch == 2 || batch == 4) && make_window_plan(p, batch, win_vectors(p.bits), entry_halfs(p.v), false, &plan))
      return true;
  }
  return pass_pair(p) && (batch == 1 || batch == 2 || batch == 4) && make_pass_plan(p, batch, win_vectors(p.bits), entry_halfs(p.v), &pplan);
}

// batch in {1, 2, 4}
int launch_gemv_lds(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  LdsPlan plan;
  if (p.orientation != 0) return VQ_ERR_UNSUPPORTED;
  if (p.n_groups == 1) {
    if (batch == 1 || batch == 2 || batch == 4) {           // the compile-time variants first
      const int rc = launch_window_any(p, x, ldx, batch, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    {                                                       // then one table at a time, where a (V, BITS) pair is compiled
      const int rc = launch_passes_any(p, x, ldx, batch, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    if (make_plan(p, batch, &plan)) {
      if (batch == 1) return launch_b<1>(p, plan, x, ldx, y, ldy, s);
      if (batch == 2) return launch_b<2>(p, plan, x, ldx, y, ldy, s);
      if (batch == 4) return launch_b<4>(p, plan, x, ldx, y, ldy, s);
      return VQ_ERR_UNSUPPORTED;
    }
  }
  return launch_passes_any(p, x, ldx, batch, y, ldy, s);      // outlier columns, codebook groups, tables that do not fit together
}

// Layers that the pass kernel takes and that have at least two codebook groups: with a workspace of
// slots x (batch x out_features + 16) binary32 sums every workgroup takes one slot; 0 when that does not apply.
size_t gemv_lds_slots_workspace_bytes(const Params &p, int batch) {
  PassPlan plan;
  const int n_slots = p.n_groups;
  if (p.orientation != 0 || n_slots < 2 || n_slots > 64 || !pass_pair(p)) return 0;
  if (!make_pass_plan(p, 1, win_vectors(p.bits), entry_halfs(p.v), &plan, n_slots)) return 0;
  return ((size_t)n_slots * ((size_t)batch * (size_t)p.out_features + 16) * sizeof(float) + 255) / 256 * 256;
}

// The slots' sums into part [slots][batch][out_features] and part_xs [slots][16]; the caller adds them up.
int launch_gemv_lds_slots(const Params &p, const __half *x, long long ldx, int batch, float *part, float *part_xs, hipStream_t s) {
  const int n_slots = p.n_groups;
  int done = 0, g_max = 4;
  while (done < batch) {
    int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
    if (g > g_max) g = g_max;
    const int rc = launch_slots_any(p, x + done * ldx, ldx, g, n_slots, batch, part + (size_t)done * p.out_features, part_xs + done, s);
    if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
    if (rc != VQ_OK) return done ? VQ_ERR_HIP : rc;
    done += g;
  }
  return VQ_OK;
}

}  // namespace vq
