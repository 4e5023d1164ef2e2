// CPU oracle for the vector-quantized linear layer -- TEST INFRASTRUCTURE ONLY.
// Plain loops, fp64 accumulation, no blocking or fusion; see vq_oracle.h.
#include "vq_oracle.h"
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>
#include <atomic>
#include <algorithm>

extern "C" float vq_oracle_half_to_float(uint16_t h) {
  // binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
  const int sign = (h >> 15) & 1;
  const int exponent = (h >> 10) & 0x1F;
  const int fraction = h & 0x3FF;
  double value;
  if (exponent == 0x1F) {
    value = fraction ? NAN : INFINITY;
  } else if (exponent == 0) {
    value = std::ldexp((double)fraction, -24);             // subnormal: fraction * 2^-24
  } else {
    value = std::ldexp(1.0 + fraction / 1024.0, exponent - 15);
  }
  return (float)(sign ? -value : value);                    // every binary16 value is exact in binary32
}

extern "C" uint16_t vq_oracle_float_to_half(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  if (std::isnan(f)) return (uint16_t)(sign | 0x7E00u);
  const double a = std::fabs((double)f);
  if (std::isinf(f) || a >= 65520.0) return (uint16_t)(sign | 0x7C00u);   // 65520 is the tie that rounds up to infinity
  if (a == 0.0) return sign;
  // Spacing of binary16 values around a: 2^-24 below 2^-14, else 2^(e-10).
  int e;
  std::frexp(a, &e);                 // a = m * 2^e, m in [0.5, 1)
  int exp2 = e - 1;                  // a in [2^exp2, 2^(exp2+1))
  if (exp2 < -14) exp2 = -14;        // subnormal range shares the spacing of the smallest normal binade
  const double ulp = std::ldexp(1.0, exp2 - 10);
  const double q = a / ulp;          // exact: division by a power of two
  double n = std::floor(q);
  const double r = q - n;
  if (r > 0.5 || (r == 0.5 && std::fmod(n, 2.0) == 1.0)) n += 1.0;        // nearest, ties to even
  // n counts ulps; n in [0, 2048].  Bits = n + (exp2+14)*1024 handles the carry into the next binade.
  const uint32_t bits = (uint32_t)n + (uint32_t)(exp2 + 14) * 1024u;
  return (uint16_t)(sign | bits);
}

extern "C" int vq_oracle_index_bits(int32_t k) {
  int b = 1;
  while (((int64_t)1 << b) < (int64_t)k) ++b;
  return b;
}

extern "C" int vq_oracle_unpack_row(const uint8_t *row, int bits, int64_t count, int32_t *out) {
  if (!row || !out || bits < 1 || bits > 16 || count < 0) return VQO_ERR_ARG;
  for (int64_t p = 0; p < count; ++p) {
    int32_t value = 0;
    for (int j = 0; j < bits; ++j) {
      const int64_t t = p * bits + j;                 // bit t of the row's stream
      const int bit = (row[t >> 3] >> (t & 7)) & 1;    // is bit (t mod 8) of byte (t div 8)
      value |= bit << j;
    }
    out[p] = value;
  }
  return VQO_OK;
}

namespace {

struct RowDecoder {
  const vq_oracle_layer *L;
  int b, b_res, b_out;
  int64_t P, Q, Pg;            // indices per main / outlier stream; Pg: stream positions per codebook group
  bool down;                   // orientation 1: vectors run down the output dimension
  std::vector<int32_t> i_main, i_res, i_out;
  explicit RowDecoder(const vq_oracle_layer *layer) : L(layer) {
    b = vq_oracle_index_bits(L->k);
    b_res = L->k_res ? vq_oracle_index_bits(L->k_res) : 0;
    b_out = L->n_outlier_cols ? vq_oracle_index_bits(L->k_out) : 0;
    down = L->orientation == 1;
    const int64_t main_cols = (int64_t)L->in_features - L->n_outlier_cols;
    P = down ? main_cols : (main_cols + L->v - 1) / L->v;
    Q = !L->n_outlier_cols ? 0 : down ? L->n_outlier_cols : L->n_outlier_cols / L->v_out;
    Pg = L->group_vectors > 0 ? L->group_vectors : (P > 0 ? P : 1);
    i_main.resize(P); i_res.resize(L->k_res ? P : 0); i_out.resize(Q);
  }
  // Restored row o as fp16 bits, w16[c] for c < in_features.
  int decode(int64_t o, uint16_t *w16) {
    // the streams that hold row o: its own (orientation 0), or the one of its block of v (v_out) rows
    const int64_t s_main = down ? o / L->v : o, s_out = down && Q ? o / L->v_out : o;
    vq_oracle_unpack_row(L->idx + s_main * L->idx_row_stride, b, P, i_main.data());
    if (L->k_res) vq_oracle_unpack_row(L->idx_res + s_main * L->idx_res_row_stride, b_res, P, i_res.data());
    if (Q) vq_oracle_unpack_row(L->idx_out + s_out * L->idx_out_row_stride, b_out, Q, i_out.data());
    const float s = L->scale ? vq_oracle_half_to_float(L->scale[o]) : 1.0f;
    const float bias = L->bias ? vq_oracle_half_to_float(L->bias[o]) : 0.0f;
    for (int64_t c = 0; c < L->in_features; ++c) {
      float d;
      if (c < L->n_outlier_cols) {
        // which index of the outlier stream, which element of its centroid
        const int64_t q = down ? c : c / L->v_out, j = down ? o % L->v_out : c % L->v_out;
        const int32_t i = i_out[q];
        if (i >= L->k_out) return VQO_ERR_INDEX_RANGE;
        d = vq_oracle_half_to_float(L->codebook_out[(int64_t)i * L->v_out + j]);
      } else {
        const int64_t cc = c - L->n_outlier_cols;
        const int64_t p = down ? cc : cc / L->v, j = down ? o % L->v : cc % L->v;
        const int32_t i = i_main[p];
        if (i >= L->k) return VQO_ERR_INDEX_RANGE;
        const int64_t group = p / Pg;                        // this vector's tables
        d = vq_oracle_half_to_float(L->codebook[(group * L->k + i) * L->v + j]);
        if (L->k_res) {
          const int32_t r = i_res[p];
          if (r >= L->k_res) return VQO_ERR_INDEX_RANGE;
          volatile float sum = d + vq_oracle_half_to_float(L->codebook_res[(group * L->k_res + r) * L->v + j]);  // binary32 add
          d = sum;
        }
      }
      const float w32 = std::fmaf(s, d, bias);          // scale*d + bias, one rounding
      w16[L->col_perm ? L->col_perm[c] : c] = vq_oracle_float_to_half(w32);     // stored column c is the layer's column col_perm[c]
    }
    return VQO_OK;
  }
};

int check_layer(const vq_oracle_layer *L) {
  if (!L || !L->codebook || !L->idx) return VQO_ERR_ARG;
  if (L->group_vectors < 0 || (L->orientation != 0 && L->orientation != 1)) return VQO_ERR_ARG;
  if (L->out_features < 0 || L->in_features < 0 || L->v < 1 || L->k < 1) return VQO_ERR_ARG;
  if (L->k_res && (!L->codebook_res || !L->idx_res)) return VQO_ERR_ARG;
  if (L->n_outlier_cols) {
    if (!L->codebook_out || !L->idx_out || L->v_out < 1 || L->k_out < 1) return VQO_ERR_ARG;
    if ((L->orientation == 0 && L->n_outlier_cols % L->v_out) || L->n_outlier_cols > L->in_features) return VQO_ERR_ARG;
  }
  if (L->col_perm) {                                  // every column number exactly once
    std::vector<char> seen(L->in_features, 0);
    for (int64_t c = 0; c < L->in_features; ++c) {
      const int32_t t = L->col_perm[c];
      if (t < 0 || t >= L->in_features || seen[t]) return VQO_ERR_ARG;
      seen[t] = 1;
    }
  }
  return VQO_OK;
}

template <class F>
int parallel_rows(int64_t n, int n_threads, F body) {
  if (n_threads < 1) n_threads = 1;
  if ((int64_t)n_threads > n) n_threads = n > 0 ? (int)n : 1;
  std::atomic<int> status(VQO_OK);
  std::vector<std::thread> pool;
  for (int t = 0; t < n_threads; ++t) {
    pool.emplace_back([&, t]() {
      const int64_t lo = n * t / n_threads, hi = n * (t + 1) / n_threads;
      const int rc = body(lo, hi);
      if (rc != VQO_OK) status.store(rc);
    });
  }
  for (auto &th : pool) th.join();
  return status.load();
}

}  // namespace

extern "C" int vq_oracle_dequant(const vq_oracle_layer *L, uint16_t *W, int64_t ldw, int n_threads) {
  int rc = check_layer(L);
  if (rc != VQO_OK || !W || ldw < L->in_features) return VQO_ERR_ARG;
  return parallel_rows(L->out_features, n_threads, [&](int64_t lo, int64_t hi) {
    RowDecoder dec(L);
    for (int64_t o = lo; o < hi; ++o) {
      const int r = dec.decode(o, W + o * ldw);
      if (r != VQO_OK) return r;
    }
    return (int)VQO_OK;
  });
}

extern "C" int vq_oracle_matmul(const vq_oracle_layer *L, const uint16_t *x, int64_t ldx, int32_t n_tokens,
                                const int32_t *rows, int32_t n_rows, double *y, int64_t ldy, int n_threads) {
  int rc = check_layer(L);
  if (rc != VQO_OK || !x || !y || n_tokens < 0 || ldx < L->in_features) return VQO_ERR_ARG;
  if (!rows) n_rows = L->out_features;
  if (ldy < n_rows) return VQO_ERR_ARG;
  for (int32_t j = 0; rows && j < n_rows; ++j)
    if (rows[j] < 0 || rows[j] >= L->out_features) return VQO_ERR_ARG;
  const int64_t N = L->in_features;
  std::vector<double> xd((size_t)n_tokens * N);            // activations widened once: fp16 -> fp64 is exact
  for (int32_t t = 0; t < n_tokens; ++t)
    for (int64_t c = 0; c < N; ++c) xd[(size_t)t * N + c] = (double)vq_oracle_half_to_float(x[(int64_t)t * ldx + c]);
  return parallel_rows(n_rows, n_threads, [&](int64_t lo, int64_t hi) {
    RowDecoder dec(L);
    std::vector<uint16_t> w16(N);
    std::vector<double> w(N);
    for (int64_t j = lo; j < hi; ++j) {
      const int64_t o = rows ? rows[j] : j;
      const int r = dec.decode(o, w16.data());
      if (r != VQO_OK) return r;
      for (int64_t c = 0; c < N; ++c) w[c] = (double)vq_oracle_half_to_float(w16[c]);
      for (int32_t t = 0; t < n_tokens; ++t) {
        const double *xt = xd.data() + (int64_t)t * N;
        double acc = 0.0;
        for (int64_t c = 0; c < N; ++c) acc += w[c] * xt[c];
        y[(int64_t)t * ldy + j] = acc;
      }
    }
    return (int)VQO_OK;
  });
}

// Eq. 2 (Sec. 2.2) and the residual stage's equation (Sec. 3.2.2): index of the nearest centroid, every vector
// against every centroid.  The header states the arithmetic; volatile keeps each binary32 step a step of its own.
extern "C" int vq_oracle_assign(const uint16_t *W, const uint16_t *B, int64_t ld, int32_t rows, int32_t cols,
                                const uint16_t *codebook, int32_t v, int32_t k, int32_t *out, int n_threads) {
  if (!W || !codebook || !out || rows < 0 || cols < 1 || ld < cols || v < 1 || k < 1) return VQO_ERR_ARG;
  const int64_t P = ((int64_t)cols + v - 1) / v;
  std::vector<float> C((size_t)k * v);
  for (int64_t e = 0; e < (int64_t)k * v; ++e) C[e] = vq_oracle_half_to_float(codebook[e]);
  return parallel_rows(rows, n_threads, [&](int64_t lo, int64_t hi) {
    std::vector<float> t(v);
    for (int64_t o = lo; o < hi; ++o)
      for (int64_t p = 0; p < P; ++p) {
        const int64_t c0 = p * v;
        const int len = (int)std::min<int64_t>(v, cols - c0);
        for (int j = 0; j < len; ++j) {
          volatile float tj = vq_oracle_half_to_float(W[o * ld + c0 + j]);
          if (B) tj = tj - vq_oracle_half_to_float(B[o * ld + c0 + j]);
          t[j] = tj;
        }
        int32_t best = 0;
        float best_d = 0.0f;
        for (int32_t i = 0; i < k; ++i) {
          volatile float d = 0.0f;
          for (int j = 0; j < len; ++j) {
            volatile float diff = t[j] - C[(size_t)i * v + j];
            d = std::fmaf(diff, diff, d);
          }
          if (i == 0 || d < best_d) { best = i; best_d = d; }        // strict: the first of equal distances stays
        }
        out[o * P + p] = best;
      }
    return (int)VQO_OK;
  });
}

// Eq. 2 with the paper's own vectors: v consecutive rows of one column (Sec. 3.1; Algorithm 1).
extern "C" int vq_oracle_assign_down(const uint16_t *W, const uint16_t *B, int64_t ld, int32_t rows, int32_t cols,
                                     const uint16_t *codebook, int32_t v, int32_t k, int32_t *out, int n_threads) {
  if (!W || !codebook || !out || rows < 1 || cols < 1 || ld < cols || v < 1 || k < 1) return VQO_ERR_ARG;
  const int64_t S = ((int64_t)rows + v - 1) / v;
  std::vector<float> C((size_t)k * v);
  for (int64_t e = 0; e < (int64_t)k * v; ++e) C[e] = vq_oracle_half_to_float(codebook[e]);
  return parallel_rows(S, n_threads, [&](int64_t lo, int64_t hi) {
    std::vector<float> t(v);
    for (int64_t p = lo; p < hi; ++p) {
      const int len = (int)std::min<int64_t>(v, rows - p * v);
      for (int64_t n = 0; n < cols; ++n) {
        for (int j = 0; j < len; ++j) {
          volatile float tj = vq_oracle_half_to_float(W[(p * v + j) * ld + n]);
          if (B) tj = tj - vq_oracle_half_to_float(B[(p * v + j) * ld + n]);
          t[j] = tj;
        }
        int32_t best = 0;
        float best_d = 0.0f;
        for (int32_t i = 0; i < k; ++i) {
          volatile float d = 0.0f;
          for (int j = 0; j < len; ++j) {
            volatile float diff = t[j] - C[(size_t)i * v + j];
            d = std::fmaf(diff, diff, d);
          }
          if (i == 0 || d < best_d) { best = i; best_d = d; }
        }
        out[p * cols + n] = best;
      }
    }
    return (int)VQO_OK;
  });
}

// Algorithm 1 (Sec. 3.1): the quantizer's column loop, in the algorithm's order and notation.  See the header.
extern "C" int vq_oracle_quantize_columns(const double *W0, const double *Hinv, int32_t M, int32_t N, const uint16_t *codebook, int32_t v,
                                          int32_t k, const uint16_t *codebook_res, int32_t k_res, int32_t B, const int32_t *given_idx,
                                          const int32_t *given_idx_res, int32_t *idx, int32_t *idx_res, double *What, double *T) {
  if (!W0 || !Hinv || !codebook || !idx || !What || M < 1 || N < 1 || v < 1 || k < 1 || B < 1) return VQO_ERR_ARG;
  if (k_res && (!codebook_res || !idx_res)) return VQO_ERR_ARG;
  std::vector<double> W(W0, W0 + (size_t)M * N);           // the working copy that takes the error updates
  std::vector<double> E((size_t)M * N, 0.0);
  std::vector<double> C((size_t)k * v), R((size_t)k_res * v);
  for (size_t e = 0; e < C.size(); ++e) C[e] = (double)vq_oracle_half_to_float(codebook[e]);
  for (size_t e = 0; e < R.size(); ++e) R[e] = (double)vq_oracle_half_to_float(codebook_res[e]);
  // index of the nearest of `count` centroids to t[0 .. len)
  auto nearest = [&](const std::vector<double> &table, int32_t count, const double *t, int len) {
    int32_t best = 0;
    double best_d = 0.0;
    for (int32_t i = 0; i < count; ++i) {
      double d = 0.0;
      for (int j = 0; j < len; ++j) d += (t[j] - table[(size_t)i * v + j]) * (t[j] - table[(size_t)i * v + j]);
      if (i == 0 || d < best_d) { best = i; best_d = d; }
    }
    return best;
  };
  std::vector<double> t(v), r(v);
  for (int32_t s = 0; s < N; s += B) {                     // column blocks
    const int32_t s_end = std::min(N, s + B);
    for (int32_t n = s; n < s_end; ++n) {                  // one column at a time
      for (int32_t m = 0, p = 0; m < M; m += v, ++p) {     // the column's vectors
        const int len = std::min(v, M - m);
        for (int j = 0; j < len; ++j) t[j] = W[(size_t)(m + j) * N + n];
        const int32_t i = given_idx ? given_idx[(size_t)p * N + n] : nearest(C, k, t.data(), len);
        if (i < 0 || i >= k) return VQO_ERR_INDEX_RANGE;
        idx[(size_t)p * N + n] = i;
        int32_t ir = 0;
        if (k_res) {
          for (int j = 0; j < len; ++j) r[j] = t[j] - C[(size_t)i * v + j];
          ir = given_idx_res ? given_idx_res[(size_t)p * N + n] : nearest(R, k_res, r.data(), len);
          if (ir < 0 || ir >= k_res) return VQO_ERR_INDEX_RANGE;
          idx_res[(size_t)p * N + n] = ir;
        }
        for (int j = 0; j < len; ++j) {
          double q = C[(size_t)i * v + j];
          if (k_res) {
            volatile float sum = (float)q + (float)R[(size_t)ir * v + j];       // what inference restores: binary32 sum, then binary16
            q = (double)vq_oracle_half_to_float(vq_oracle_float_to_half(sum));
          }
          What[(size_t)(m + j) * N + n] = q;
        }
      }
      for (int32_t o = 0; o < M; ++o) {
        if (T) T[(size_t)o * N + n] = W[(size_t)o * N + n];
        E[(size_t)o * N + n] = (W[(size_t)o * N + n] - What[(size_t)o * N + n]) / Hinv[(size_t)n * N + n];
        for (int32_t c = n; c < s_end; ++c) W[(size_t)o * N + c] -= E[(size_t)o * N + n] * Hinv[(size_t)n * N + c];
      }
    }
    for (int32_t o = 0; o < M; ++o)                        // all the remaining columns
      for (int32_t c = s_end; c < N; ++c) {
        double acc = 0.0;
        for (int32_t n = s; n < s_end; ++n) acc += E[(size_t)o * N + n] * Hinv[(size_t)n * N + c];
        W[(size_t)o * N + c] -= acc;
      }
  }
  return VQO_OK;
}
