// vq_gemv: decode-phase fused restore + matrix-vector product for batch 1..16
// (paper App. "Our Dequantization Implementation", second phase: the FP16 weights are never written).
#include "vq_common.hpp"
#include <cstdlib>

namespace vq {

// The activation that stored column c meets (Sec. 3.2.3: the stored order of the columns may be a permutation of the
// layer's); entries outside the row count as zero.
__device__ __forceinline__ float x_at(const Params &p, const __half *xrow, int c) {
  if (!p.perm) return __half2float(xrow[c]);
  const int t = p.perm[c];
  return (unsigned)t < (unsigned)p.in_features ? __half2float(xrow[t]) : 0.0f;
}

// Any layer: one wave per output row, lanes stride over the row's vectors, tables read through the
// cache hierarchy.  Slow but complete; the specialised kernels below take the common shapes.
__global__ __launch_bounds__(256) void gemv_generic_kernel(Params p, const __half *__restrict__ x, long long ldx, int batch,
                                                           __half *__restrict__ y, long long ldy) {
  const int lane = threadIdx.x & 63;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= p.out_features) return;
  const float s = p.scale ? __half2float(p.scale[o]) : 1.0f;
  const float b = p.bias ? __half2float(p.bias[o]) : 0.0f;
  float acc[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) acc[t] = 0.0f;
  for (int slot = lane; slot < p.Q + p.P; slot += 64) {
    const __half *e, *er = nullptr;
    int c0, len;
    if (slot < p.Q) {
      unsigned i = min(load_index(p.idx_out + (long long)o * p.stride_out, slot, p.bits_out), (unsigned)p.k_out - 1u);
      e = p.cb_out + (long long)i * p.v_out;
      c0 = slot * p.v_out; len = p.v_out;
    } else {
      const int pp = slot - p.Q;
      unsigned i = min(load_index(p.idx + (long long)o * p.stride, pp, p.bits), (unsigned)p.k - 1u);
      const long long group = pp / p.Pg;
      e = p.cb + (group * p.k + i) * p.v;
      if (p.k_res) {
        unsigned r = min(load_index(p.idx_res + (long long)o * p.stride_res, pp, p.bits_res), (unsigned)p.k_res - 1u);
        er = p.cb_res + (group * p.k_res + r) * p.v;
      }
      c0 = p.n_out + pp * p.v; len = min(p.v, p.in_features - c0);
    }
    for (int j = 0; j < len; ++j) {
      float d = __half2float(e[j]);
      if (er) d = __fadd_rn(d, __half2float(er[j]));
      const float w = __half2float(restore(d, s, b));
#pragma unroll
      for (int t = 0; t < 16; ++t)
        if (t < batch) acc[t] = __fmaf_rn(w, x_at(p, x + t * ldx, c0 + j), acc[t]);
    }
  }
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    if (t < batch) {
      const float r = wave_sum(acc[t]);
      if (lane == 0) y[t * ldy + o] = __float2half_rn(r);
    }
  }
}

// Orientation 1 (vectors down the output dimension; Sec. 3.1, Algorithm 1): one wave per main stream, i.e. per block of v
// output rows; lanes stride over the columns and keep one sum per row of the block; the outlier columns of each of these
// rows come from the outlier stream that holds the row.  One token at a time.  Slow but complete.
__global__ __launch_bounds__(256) void gemv_down_kernel(Params p, const __half *__restrict__ x, long long ldx, int batch,
                                                        __half *__restrict__ y, long long ldy) {
  const int lane = threadIdx.x & 63;
  const int stream = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (stream >= p.S) return;
  const int o0 = stream * p.v;
  float sc[16], bi[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const bool on = j < p.v && o0 + j < p.out_features;
    sc[j] = on && p.scale ? __half2float(p.scale[o0 + j]) : 1.0f;
    bi[j] = on && p.bias ? __half2float(p.bias[o0 + j]) : 0.0f;
  }
  for (int t = 0; t < batch; ++t) {
    const __half *xt = x + (long long)t * ldx;
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0f;
    for (int pos = lane; pos < p.P; pos += 64) {
      unsigned i = min(load_index(p.idx + (long long)stream * p.stride, pos, p.bits), (unsigned)p.k - 1u);
      const long long group = pos / p.Pg;
      const __half *e = p.cb + (group * p.k + i) * p.v, *er = nullptr;
      if (p.k_res) {
        unsigned r = min(load_index(p.idx_res + (long long)stream * p.stride_res, pos, p.bits_res), (unsigned)p.k_res - 1u);
        er = p.cb_res + (group * p.k_res + r) * p.v;
      }
      const float xv = x_at(p, xt, p.n_out + pos);
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < p.v && o0 + j < p.out_features) {
          float d = __half2float(e[j]);
          if (er) d = __fadd_rn(d, __half2float(er[j]));
          acc[j] = __fmaf_rn(__half2float(restore(d, sc[j], bi[j])), xv, acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j < p.v && o0 + j < p.out_features) {
        const int o = o0 + j, sq = p.Q ? o / p.v_out : 0, jo = p.Q ? o - sq * p.v_out : 0;
        for (int pos = lane; pos < p.Q; pos += 64) {
          unsigned i = min(load_index(p.idx_out + (long long)sq * p.stride_out, pos, p.bits_out), (unsigned)p.k_out - 1u);
          const float w = __half2float(restore(__half2float(p.cb_out[(long long)i * p.v_out + jo]), sc[j], bi[j]));
          acc[j] = __fmaf_rn(w, x_at(p, xt, pos), acc[j]);
        }
        const float r = wave_sum(acc[j]);
        if (lane == 0) y[(long long)t * ldy + o] = __float2half_rn(r);
      }
  }
}

bool gemv_fast_applicable(const Params &p, const __half *x, long long ldx);
bool gemv_res8_applicable(const Params &p, const __half *x);
bool gemv_lds_applicable(const Params &p, int batch);
int launch_gemv_lds(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
size_t gemv_lds_slots_workspace_bytes(const Params &p, int batch);
bool gemv_down_lds_applicable(const Params &p, int batch);
size_t gemv_down_lds_slots_workspace_bytes(const Params &p, int batch);
int launch_gemv_down_lds_slots(const Params &p, const __half *x, long long ldx, int batch, float *part, float *part_xs, hipStream_t s);
int launch_gemv_down_lds(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
int launch_gemv_lds_slots(const Params &p, const __half *x, long long ldx, int batch, float *part, float *part_xs, hipStream_t s);
int launch_gemv_res8(const Params &p, const __half *x, __half *y, hipStream_t s);
int launch_gemv_fast(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);

int launch_gemv_mfma(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
bool gemv_down_applicable(const Params &p, const __half *x, long long ldx);
bool gemv_down_fits(const Params &p);
bool gemv_v8_applicable(const Params &p, const __half *x, long long ldx);
int launch_gemv_v8(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
bool gemv_v8_down_applicable(const Params &p);
int launch_gemv_v8_down(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s);
int launch_gemv_down(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s,
                     float *part = nullptr, float *part_xs = nullptr, int part_batch = 0);
int launch_groups_finish(const float *part, const float *part_xs, int n_groups, int batch, const Params &p, __half *y, long long ldy,
                         hipStream_t s);
bool gemv_down_mfma_applicable(const Params &p, const __half *x, long long ldx, int batch);
int gemv_down_mfma_parts(const Params &p);
int launch_gemv_down_mfma(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s,
                          float *part, float *part_xs, int parts);

// Switch gemv=g forces the generic kernel, =m the matrix-core kernel, =d the dot-product kernels (testing and
// measurement; unset: chosen by batch and shape).
static char forced_kernel() { return switches().gemv; }
static bool force_generic() { return forced_kernel() == 'g'; }

static bool down_mfma_wanted(const Params &p, const __half *x, long long ldx, int batch) {
  const char fk = forced_kernel();
  return fk != 'g' && fk != 'd' && gemv_down_applicable(p, x, ldx) && gemv_down_mfma_applicable(p, x, ldx, batch);
}
// With a workspace (column parts, one workgroup per block of 16 streams and part): from two rows on, and for any batch
// when there are codebook groups (measured, 4096 x 4096: one row 12.8 against 10.5 us, two rows 13.0 against 12.7 us and
// level from there; 16 groups, one row: 15.5 against 17.4 us).
// (and for one row of a layer whose activations do not fit the other kernel's LDS beside the tables)
static bool down_mfma_parts_wanted(const Params &p, const __half *x, long long ldx, int batch) {
  return down_mfma_wanted(p, x, ldx, batch) && (batch >= 2 || p.n_groups > 1 || forced_kernel() == 'm' || !gemv_down_fits(p));
}
// Without a workspace a block of 16 streams is one workgroup over all the columns: with few blocks and three or four rows the
// other kernel, which spreads single streams over the chip, is still ahead (4096 x 11008, 43 blocks: 26 against 34 us).
static bool down_mfma_alone_wanted(const Params &p, const __half *x, long long ldx, int batch) {
  if (!down_mfma_wanted(p, x, ldx, batch)) return false;
  if (p.n_groups > 1) return true;                        // the only fast kernel of this orientation that walks codebook groups by itself
  // (with a 12-bit residual stream the other kernel pays twice per row, and three rows are enough: 4096 x 11008, 54 against 46 us)
  return batch >= 5 || (batch >= 3 && (p.S >= 64 * 16 || (p.k_res && p.bits_res == 12))) || forced_kernel() == 'm';
}

// Whether vq_gemv would run this layer on the kernels that keep one table in LDS at a time (no kernel of its own, tables that fit).
bool gemv_has_lds_kernel(const Params &p, const __half *x, long long ldx) {
  if (forced_kernel() != '\0') return false;
  if (p.orientation == 1) return !gemv_down_applicable(p, x, ldx) && !gemv_v8_down_applicable(p) && gemv_down_lds_applicable(p, 1);
  return !gemv_fast_applicable(p, x, ldx) && !gemv_v8_applicable(p, x, ldx) && gemv_lds_applicable(p, 1);
}

// Whether vq_gemv has one of its specialised kernels for this layer and these activations (vq_gemm sends small token
// counts, and layers its own kernels do not take, through vq_gemv sixteen rows at a time).
bool gemv_has_fast_kernel(const Params &p, const __half *x, long long ldx) {
  if (forced_kernel() != '\0') return false;
  if (p.orientation == 1) return down_mfma_wanted(p, x, ldx, 16) || gemv_v8_down_applicable(p);
  return gemv_fast_applicable(p, x, ldx) || gemv_v8_applicable(p, x, ldx);
}

// Layers without a kernel of their own whose tables fit LDS (vq_gemv_lds.hip): batch rows in launches of 4, 2 or 1, fewer
// when that many activation rows do not fit beside the tables.  VQ_ERR_UNSUPPORTED when the kernel does not take the layer.
static int gemv_through_lds_tables(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  const bool down = p.orientation == 1;
  if (force_generic() || !(down ? gemv_down_lds_applicable(p, 1) : gemv_lds_applicable(p, 1))) return VQ_ERR_UNSUPPORTED;
  int done = 0, g_max = 4, rc = VQ_OK;
  while (done < batch) {
    int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
    if (g > g_max) g = g_max;
    rc = down ? launch_gemv_down_lds(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s) : launch_gemv_lds(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
    if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
    if (rc != VQ_OK) return rc;
    done += g;
  }
  return VQ_OK;
}

int launch_gemv(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, hipStream_t s) {
  if (p.perm) {
    // Permuted column order without a workspace: the dot-product kernels for v = 6 gather the activations while they stage
    // them in LDS (or load them into registers: long rows); everything else runs on the generic kernels, which look every
    // activation up.
    if (p.orientation == 0 && !force_generic()) {
      if (p.in_features >= 16384 && gemv_res8_applicable(p, x) && (ldx & 1) == 0) {
        // the long-row kernel gathers into its registers; more rows one after the other (still far ahead of the generic kernel)
        int rc = VQ_OK;
        for (int t = 0; t < batch && rc == VQ_OK; ++t) rc = launch_gemv_res8(p, x + t * ldx, y + t * ldy, s);
        if (rc != VQ_ERR_UNSUPPORTED) return rc;
      }
      if (gemv_fast_applicable(p, x, ldx) && p.n_groups == 1) {
        int done = 0, rc = VQ_OK, g_max = 4;
        while (done < batch) {
          int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
          if (g > g_max) g = g_max;
          rc = launch_gemv_fast(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
          if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
          if (rc != VQ_OK) break;
          done += g;
        }
        if (rc == VQ_OK) return VQ_OK;
        if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
      }
    }
    {
      const int rc = gemv_through_lds_tables(p, x, ldx, batch, y, ldy, s);       // gathers the activations while it stages them
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    if (p.orientation == 1) hipLaunchKernelGGL(gemv_down_kernel, dim3((unsigned)((p.S + 3) / 4)), dim3(256), 0, s, p, x, ldx, batch, y, ldy);
    else hipLaunchKernelGGL(gemv_generic_kernel, dim3((unsigned)((p.out_features + 3) / 4)), dim3(256), 0, s, p, x, ldx, batch, y, ldy);
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  // Matrix-core kernel: one launch for any batch, at about the cost of a batch-1 launch of the dot-product
  // kernels; those are still a little faster for one row (and for two rows of a layer with few output rows
  // per compute unit), so they keep these cases.  Layers with codebook groups always go to the matrix-core kernel:
  // it is the one that swaps the tables in LDS group by group.
  if (p.orientation == 1) {
    // from three to five rows on the matrix-core kernel of this orientation is ahead (six multiply-adds per gather and row
    // bind the other one); gemv=m sends every batch there, =d none
    if (down_mfma_alone_wanted(p, x, ldx, batch)) {
      const int rc = launch_gemv_down_mfma(p, x, ldx, batch, y, ldy, s, nullptr, nullptr, 1);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    if (!force_generic() && p.n_groups == 1 && gemv_down_applicable(p, x, ldx)) {
      // batch rows go in groups of 4, 2 or 1 (fewer when the rows do not fit LDS beside the tables)
      int done = 0, g_max = 4, rc = VQ_OK;
      while (done < batch) {
        int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
        if (g > g_max) g = g_max;
        rc = launch_gemv_down(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
        if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
        if (rc != VQ_OK) break;
        done += g;
      }
      if (rc == VQ_OK) return VQ_OK;
      if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
      if (down_mfma_wanted(p, x, ldx, batch)) {   // a row too long for that kernel's LDS (28672 columns beside two 64 KB tables)
        rc = launch_gemv_down_mfma(p, x, ldx, batch, y, ldy, s, nullptr, nullptr, 1);
        if (rc != VQ_ERR_UNSUPPORTED) return rc;
      }
    }
    if (!force_generic() && gemv_v8_down_applicable(p)) {
      // 8-component vectors, tables read through L2: batch rows in launches of 4, 2 or 1
      int done = 0, rc = VQ_OK;
      while (done < batch && rc == VQ_OK) {
        const int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
        rc = launch_gemv_v8_down(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
        if (rc == VQ_OK) done += g;
      }
      if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
    }
    {
      const int rc = gemv_through_lds_tables(p, x, ldx, batch, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
    hipLaunchKernelGGL(gemv_down_kernel, dim3((unsigned)((p.S + 3) / 4)), dim3(256), 0, s, p, x, ldx, batch, y, ldy);
    return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
  }
  // one activation row of a long-row layer with an 8-bit residual stream (the 8192 x 28672 layer of the 70B setting): the
  // kernel that replicates the residual table in LDS and keeps the activations out of it.  Measured against the other
  // dot-product kernel: 28672 columns 33.5 against 37.0 us; 8192 columns 16.0 against 14.7 us, hence the threshold
  // (gemv=d takes it for every layer it accepts, for the tests).
  if (batch == 1 && gemv_res8_applicable(p, x) && ((forced_kernel() == '\0' && p.in_features >= 16384) || forced_kernel() == 'd')) {
    const int rc = launch_gemv_res8(p, x, y, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  const bool fast = !force_generic() && gemv_fast_applicable(p, x, ldx);
  const bool many_rows = p.out_features > 16 * 256;
  // (and layers with outlier columns, whose part of the dot-product kernels is the slower one: 11008 x 4096 with 128 of
  // them, one row: 10.7 against 17.1 us; from 16384 columns on a single row is level or a little behind)
  const bool outliers_first = p.Q > 0 && (batch >= 2 || p.in_features < 16384);
  if (fast && forced_kernel() != 'd' && (batch >= 3 || (batch == 2 && many_rows) || forced_kernel() == 'm' || p.n_groups > 1 || outliers_first)) {
    const int rc = launch_gemv_mfma(p, x, ldx, batch, y, ldy, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  if (fast && p.n_groups == 1) {
    // batch rows go in groups of 4, 2 or 1; every group streams the indices once
    int done = 0, rc = VQ_OK;
    int g_max = 4;                      // largest group the layer's plan admits (found on the first group)
    while (done < batch) {
      int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
      if (g > g_max) g = g_max;
      rc = launch_gemv_fast(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
      if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
      if (rc != VQ_OK) break;
      done += g;
    }
    if (rc == VQ_OK) return VQ_OK;
    if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
    if (forced_kernel() != 'd') {       // a shape the dot-product kernels do not take
      rc = launch_gemv_mfma(p, x, ldx, batch, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
  }
  if (!force_generic() && gemv_v8_applicable(p, x, ldx)) {
    // 8-component vectors, tables read through L2: batch rows in launches of 8, 4, 2 or 1
    int done = 0, rc = VQ_OK;
    while (done < batch && rc == VQ_OK) {
      const int g = batch - done >= 8 ? 8 : batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
      rc = launch_gemv_v8(p, x + done * ldx, ldx, g, y + done * ldy, ldy, s);
      if (rc == VQ_OK) done += g;
    }
    if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
  }
  {
    const int rc = gemv_through_lds_tables(p, x, ldx, batch, y, ldy, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  const unsigned blocks = (unsigned)((p.out_features + 3) / 4);
  hipLaunchKernelGGL(gemv_generic_kernel, dim3(blocks), dim3(256), 0, s, p, x, ldx, batch, y, ldy);
  return hipGetLastError() == hipSuccess ? VQ_OK : VQ_ERR_HIP;
}

size_t gemv_mfma_groups_workspace_bytes(const Params &p, int batch);
int launch_gemv_mfma_groups(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, void *workspace,
                            hipStream_t s);

// A workspace serves layers with codebook groups on the matrix-core kernel: one group per workgroup, then a sum over
// the groups.  groups=loop keeps every workgroup walking all groups (measurement and tests).
// Layers with a permuted column order: the activations, gathered into stored order, come first in the workspace
// (batch rows of in_features rounded up to 8 halfs, the whole rounded up to 256 bytes); the rest is what the layer needs
// without the permutation.
static size_t permuted_x_bytes(const Params &p, int rows) { return ((size_t)rows * (size_t)((p.in_features + 7) & ~7) * sizeof(__half) + 255) / 256 * 256; }
// One row of a layer that the gathering dot-product kernel takes is faster without the extra launch, as long as the row
// is short: every workgroup gathers the whole row (64 lookups a wave instruction), a gather kernel does it once.
static bool permuted_in_kernel(const Params &p, const __half *x, long long ldx, int batch) {
  return batch == 1 && p.orientation == 0 && p.n_groups == 1 && forced_kernel() != 'm' && p.in_features < 16384 && gemv_fast_applicable(p, x, ldx);
}

size_t gemv_workspace_bytes(const Params &p, const __half *x, long long ldx, int batch) {
  if (force_generic()) return 0;
  if (p.perm) {
    if (permuted_in_kernel(p, x, ldx, batch)) return 0;
    Params q = p;
    q.perm = nullptr;
    return permuted_x_bytes(p, batch) + gemv_workspace_bytes(q, nullptr, (p.in_features + 7) & ~7, batch);
  }
  if (p.orientation == 1 && down_mfma_parts_wanted(p, x, ldx, batch)) {   // the matrix cores: the workspace lets parts of the columns run side by side
    const int parts = gemv_down_mfma_parts(p);            // the outlier columns are one more set of sums to add up
    return parts > 1 ? ((size_t)(parts + (p.Q ? 1 : 0)) * ((size_t)batch * (size_t)p.out_features + 16) * sizeof(float) + 255) / 256 * 256 : 0;
  }
  if (p.orientation == 1) {         // vectors down the output dimension: the same workspace layout, filled by that orientation's kernel
    if (p.n_groups > 1 && p.n_groups <= 256 && gemv_down_applicable(p, x, ldx))
      return ((size_t)(p.n_groups + (p.Q ? 1 : 0)) * ((size_t)batch * (size_t)p.out_features + 16) * sizeof(float) + 255) / 256 * 256;
    // (the other settings, on the kernel that keeps one table in LDS at a time: a group per workgroup)
    return gemv_down_applicable(p, x, ldx) || gemv_v8_down_applicable(p) ? 0 : gemv_down_lds_slots_workspace_bytes(p, batch);
  }
  if (!gemv_fast_applicable(p, x, ldx))       // the LDS-table kernels, when the layer gets that far: a slot per workgroup
    return gemv_v8_applicable(p, x, ldx) ? 0 : gemv_lds_slots_workspace_bytes(p, batch);
  if (forced_kernel() == 'd') return 0;
  return gemv_mfma_groups_workspace_bytes(p, batch);
}

int launch_gemv_ws(const Params &p, const __half *x, long long ldx, int batch, __half *y, long long ldy, void *workspace,
                   size_t workspace_bytes, hipStream_t s) {
  const size_t need = gemv_workspace_bytes(p, x, ldx, batch);
  if (p.perm) {
    if (!need || !workspace || workspace_bytes < need) return launch_gemv(p, x, ldx, batch, y, ldy, s);
    // gather the activations into stored order, then the layer is an unpermuted one
    Params q = p;
    q.perm = nullptr;
    __half *xp = static_cast<__half *>(workspace);
    const long long ldxp = (p.in_features + 7) & ~7;
    const int rc = launch_gather_cols(x, ldx, batch, p.in_features, p.perm, xp, ldxp, s);
    if (rc != VQ_OK) return rc;
    const size_t head = permuted_x_bytes(p, batch);
    return launch_gemv_ws(q, xp, ldxp, batch, y, ldy, static_cast<unsigned char *>(workspace) + head, workspace_bytes - head, s);
  }
  if (need && workspace && workspace_bytes >= need && p.orientation == 1 && down_mfma_parts_wanted(p, x, ldx, batch)) {
    const int parts = gemv_down_mfma_parts(p), slots = parts + (p.Q ? 1 : 0);
    float *part = static_cast<float *>(workspace), *part_xs = part + (size_t)slots * (size_t)batch * (size_t)p.out_features;
    int rc = launch_gemv_down_mfma(p, x, ldx, batch, nullptr, 0, s, part, part_xs, parts);
    if (rc == VQ_OK) return launch_groups_finish(part, part_xs, slots, batch, p, y, ldy, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  } else if (need && workspace && workspace_bytes >= need && p.orientation == 1 && !gemv_down_applicable(p, x, ldx)) {
    if (!switches().groups_loop) {                            // the LDS-table kernel of this orientation: a group per workgroup
      float *part = static_cast<float *>(workspace), *part_xs = part + (size_t)p.n_groups * (size_t)batch * (size_t)p.out_features;
      const int rc = launch_gemv_down_lds_slots(p, x, ldx, batch, part, part_xs, s);
      if (rc == VQ_OK) return launch_groups_finish(part, part_xs, p.n_groups, batch, p, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
  } else if (need && workspace && workspace_bytes >= need && p.orientation == 1) {
    const int slots = p.n_groups + (p.Q ? 1 : 0);             // the outlier columns are one more set of sums to add up
    float *part = static_cast<float *>(workspace), *part_xs = part + (size_t)slots * (size_t)batch * (size_t)p.out_features;
    int done = 0, g_max = 4, rc = VQ_OK;
    while (done < batch) {                                // batch rows in launches of 4, 2 or 1, as without groups
      int g = batch - done >= 4 ? 4 : batch - done >= 2 ? 2 : 1;
      if (g > g_max) g = g_max;
      rc = launch_gemv_down(p, x + done * ldx, ldx, g, nullptr, 0, s, part + (size_t)done * p.out_features, part_xs + done, batch);
      if (rc == VQ_ERR_UNSUPPORTED && g > 1) { g_max = g / 2; continue; }
      if (rc != VQ_OK) break;
      done += g;
    }
    if (rc == VQ_OK) return launch_groups_finish(part, part_xs, slots, batch, p, y, ldy, s);
    if (rc != VQ_ERR_UNSUPPORTED || done != 0) return rc;
  } else if (need && workspace && workspace_bytes >= need && !gemv_fast_applicable(p, x, ldx)) {
    if (!switches().groups_loop) {
      const int slots = p.n_groups;                         // (the first group's workgroups also take the outlier columns)
      float *part = static_cast<float *>(workspace), *part_xs = part + (size_t)slots * (size_t)batch * (size_t)p.out_features;
      const int rc = launch_gemv_lds_slots(p, x, ldx, batch, part, part_xs, s);
      if (rc == VQ_OK) return launch_groups_finish(part, part_xs, slots, batch, p, y, ldy, s);
      if (rc != VQ_ERR_UNSUPPORTED) return rc;
    }
  } else if (need && workspace && workspace_bytes >= need && !switches().groups_loop) {
    const int rc = launch_gemv_mfma_groups(p, x, ldx, batch, y, ldy, workspace, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  return launch_gemv(p, x, ldx, batch, y, ldy, s);
}

int launch_gemv_mfma_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys,
                           const long long *ldys, hipStream_t s);
int launch_gemv_fast_multi(const Params *ps, int n, const __half *x, __half *const *ys, hipStream_t s);
int launch_gemv_down_mfma_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys,
                                const long long *ldys, hipStream_t s);

// Several layers on the same activations: one launch of the dot-product kernel (one row) or of the matrix-core kernel
// (more rows; gemv=m: always) when all of them take it together, else (and with multi=0, for measurement and tests) one vq_gemv after the other.
int launch_gemv_multi(const Params *ps, int n, const __half *x, long long ldx, int batch, __half *const *ys, const long long *ldys,
                      hipStream_t s) {
  bool fused = n >= 2 && !switches().multi_off && forced_kernel() != 'g' && forced_kernel() != 'd';
  for (int i = 0; i < n; ++i) fused = fused && !ps[i].perm;      // permuted column orders: one layer after the other
  // layers with vectors down the output dimension: the matrix-core kernel of that orientation, any batch (a block of 16
  // streams per workgroup over all columns; the blocks of all the layers together are what fills the chip)
  bool down = fused;
  for (int i = 0; down && i < n; ++i) down = ps[i].orientation == 1 && ps[i].n_groups == 1 && down_mfma_wanted(ps[i], x, ldx, batch);
  if (down) {
    const int rc = launch_gemv_down_mfma_multi(ps, n, x, ldx, batch, ys, ldys, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  for (int i = 0; fused && i < n; ++i) fused = gemv_fast_applicable(ps[i], x, ldx);
  if (fused && batch == 1 && forced_kernel() != 'm') {     // a single row: the dot-product kernel is the faster body
    const int rc = launch_gemv_fast_multi(ps, n, x, ys, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  if (fused) {
    const int rc = launch_gemv_mfma_multi(ps, n, x, ldx, batch, ys, ldys, s);
    if (rc != VQ_ERR_UNSUPPORTED) return rc;
  }
  for (int i = 0; i < n; ++i) {
    const int rc = launch_gemv(ps[i], x, ldx, batch, ys[i], ldys[i], s);
    if (rc != VQ_OK) return rc;
  }
  return VQ_OK;
}

}  // namespace vq
