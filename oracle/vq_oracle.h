/* CPU oracle for the vector-quantized linear layer -- TEST INFRASTRUCTURE ONLY.
 *
 * A slow, plain restatement of what the layer computes, used to check the GPU
 * library and as the timed CPU baseline.  It shares no code, header or table
 * with the GPU library, and nothing in the product path may call it.
 *
 * What is computed follows the paper's description of inference: a weight
 * vector is restored by looking its index up in the codebook (Sec. 2.2,
 * "Vector Quantization"), the residual codebook's centroid is added to it
 * (Sec. 3.2.2, "Residual Vector Quantization"), a small set of outlier
 * columns uses a codebook of its own (Sec. 3.2.3, "Outlier Elimination";
 * parameters v0,k0,v1,k1,k2 of App. "Parameter Description"; the columns are
 * picked by the Hessian's diagonal, hence a column permutation), the weight
 * matrix may be split into groups that each have a codebook of their own
 * (Sec. 3.1, the paragraph on groups; "group num" in the parameter tables), and
 * the restored FP16 matrix multiplies the activations (App. "Our Dequantization
 * Implementation").  Per-output-channel scale and bias are applied to the
 * restored weight before it is rounded to FP16.
 *
 * All pointers are HOST pointers.  Parity status: every function here is
 * pinned by tests that do not depend on the oracle itself (hand-written byte
 * streams, one-hot lookups, W*e_j = column j, an independent triple-loop
 * matmul on unpacked indices, the compiler's own FP16 conversions; for the
 * quantizer's column loop: a test-local restatement without blocks, the
 * identity Hinv, independence of the block size, and the second-order loss
 * identity of the Cholesky factor).
 */
#ifndef VQ_ORACLE_H
#define VQ_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct vq_oracle_layer {
  int32_t out_features, in_features;      /* M rows (outputs), N columns (inputs)             */
  int32_t v, k;                           /* main codebook: vector length, entries            */
  int32_t k_res;                          /* residual codebook entries (same v); 0 = none     */
  int32_t n_outlier_cols, v_out, k_out;   /* first n columns use the outlier codebook; 0=none */
  const uint16_t *codebook;               /* fp16 bits [k][v]                                 */
  const uint16_t *codebook_res;           /* fp16 bits [k_res][v]                             */
  const uint16_t *codebook_out;           /* fp16 bits [k_out][v_out]                         */
  const uint8_t *idx;      int64_t idx_row_stride;      /* per-row bitstreams, stride in bytes */
  const uint8_t *idx_res;  int64_t idx_res_row_stride;
  const uint8_t *idx_out;  int64_t idx_out_row_stride;
  const uint16_t *scale, *bias;           /* fp16 bits [out_features]; NULL = 1.0 / 0.0       */
  /* Groups: with group_vectors > 0 the main vectors of a row are split into consecutive ranges of group_vectors
   * vectors (the last range may be shorter), ceil(P / group_vectors) groups in all, and each group has its own
   * main table and, if there is a residual codebook, its own residual table: vector p reads the tables of group
   * p / group_vectors.  codebook is then [groups][k][v] and codebook_res [groups][k_res][v].  0 means one
   * group.  Outlier columns keep their single table.                                            */
  int32_t group_vectors;
  /* Orientation of the vectors.  0: along the input dimension of an output row, as described above.
   * 1: the paper's own (Sec. 3.1: a quantized column is a stack of centroids; Algorithm 1 quantizes W[m:m+v, n]): a
   * vector covers v consecutive output rows of one input column.  Stream p of idx (and idx_res) then belongs to output
   * rows [p v, p v + v), the last one cut at out_features, and holds one index per main column: position t is column
   * n_outlier_cols + t, and W[p v + j][n_outlier_cols + t] comes from element j of its centroid.  There are
   * ceil(out_features / v) such streams.  Stream q of idx_out belongs to rows [q v_out, q v_out + v_out) and holds one
   * index per outlier column (n_outlier_cols need not be a multiple of v_out here).  Codebook groups are ranges of
   * group_vectors stream positions, i.e. of main columns.  Scale and bias stay per output row.                  */
  int32_t orientation;
  /* Column order.  The columns that get the outlier codebook are the ones the Hessian's diagonal singles out (Sec.
   * 3.2.3), wherever they lie, so the stored order of the columns is a permutation of the layer's: with col_perm != NULL
   * (int32 [in_features], every column number exactly once) everything said above about "column c" describes STORED
   * column c, which is column col_perm[c] of the layer: W[o][col_perm[c]] is the value restored for (o, c), and stored
   * column c meets x[col_perm[c]].  The outlier columns of the layer are col_perm[0 .. n_outlier_cols).  NULL: the
   * identity.                                                                                                  */
  const int32_t *col_perm;
} vq_oracle_layer;

enum { VQO_OK = 0, VQO_ERR_ARG = -1, VQO_ERR_INDEX_RANGE = -2 };

/* IEEE binary16 <-> binary32, round-to-nearest-even, subnormals kept, overflow to infinity. */
float    vq_oracle_half_to_float(uint16_t h);
uint16_t vq_oracle_float_to_half(float f);

/* ceil(log2 k), at least 1: bits of one stored index. */
int vq_oracle_index_bits(int32_t k);

/* Read `count` indices of `bits` bits from one row's little-endian bitstream. */
int vq_oracle_unpack_row(const uint8_t *row, int bits, int64_t count, int32_t *out);

/* Restored weight matrix as fp16 bits, W[o*ldw + c] for c < in_features. */
int vq_oracle_dequant(const vq_oracle_layer *L, uint16_t *W, int64_t ldw, int n_threads);

/* y[t*ldy + j] = sum_c W[rows[j]][c] * x[t*ldx + c] in fp64, c ascending.
 * rows == NULL means all rows (n_rows = out_features, j = o).                                */
int vq_oracle_matmul(const vq_oracle_layer *L, const uint16_t *x, int64_t ldx, int32_t n_tokens,
                     const int32_t *rows, int32_t n_rows, double *y, int64_t ldy, int n_threads);

/* Nearest-centroid assignment, the encode side of the lookup (Eq. 2 of Sec. 2.2; with B, the residual stage's
 * equation in Sec. 3.2.2, B being the first stage's restored values).  W, B: fp16 bits [rows][ld]; vectors run along a
 * row, vector p = columns [p v, p v + v), the last one cut at `cols`; codebook: fp16 bits [k][v].
 * t_j = W[o][p v + j] (- B[o][p v + j]),  d_i = sum_j (t_j - C[i][j])^2,  out[o * P + p] = the smallest i among those
 * with the smallest d_i, P = ceil(cols / v).
 * The paper fixes no precision for the distance, and a distance decides an integer, so the arithmetic is spelled out
 * and the HIP kernel follows the same: everything in binary32, round to nearest even; t_j is one subtraction of the
 * two widened binary16 values; every term is one subtraction and one fused multiply-add into the running sum, which
 * starts at +0 and takes j in ascending order.                                                                      */
int vq_oracle_assign(const uint16_t *W, const uint16_t *B, int64_t ld, int32_t rows, int32_t cols,
                     const uint16_t *codebook, int32_t v, int32_t k, int32_t *out, int n_threads);

/* The same for vectors that run down the columns of W (orientation 1 of vq_oracle_layer; Sec. 3.1, Algorithm 1's
 * Q(W[m:m+V, n])): vector (p, n) = W[p v + j][n], j < v, the last block of rows cut at `rows` and compared over its own
 * elements; out[p * cols + n], p < ceil(rows / v).  Same arithmetic, j ascending.                                  */
int vq_oracle_assign_down(const uint16_t *W, const uint16_t *B, int64_t ld, int32_t rows, int32_t cols,
                          const uint16_t *codebook, int32_t v, int32_t k, int32_t *out, int n_threads);

/* The column loop of the quantizer (Algorithm 1, Sec. 3.1 "VPTQ Algorithm"; the error update is the Delta W equation of
 * that section): columns are quantized one at a time, every column as a stack of length-v vectors that each take their
 * nearest centroid (Eq. 2; with a residual codebook, a second nearest centroid for what the first leaves, Sec. 3.2.2), the
 * column's error divided by the diagonal entry of the matrix the algorithm calls H^-1 is spread over the columns of its
 * block of B columns that are still to come, and at the end of a block over all later columns:
 *     for s = 0, B, 2B, ...:   for n = s .. min(s + B, N) - 1:
 *         What[:, n] = Q(W[:, n]);   E[:, n] = (W[:, n] - What[:, n]) / Hinv[n][n];
 *         W[:, n : s + B] -= E[:, n] * Hinv[n][n : s + B]
 *       W[:, s + B :] -= E[:, s : s + B] * Hinv[s : s + B][s + B :]
 * Hinv is an input: the algorithm only reads rows of it (callers in the GPTQ tradition pass the upper Cholesky factor of
 * the inverse Hessian, for which the sum of squared E is the second-order loss).  Everything is fp64: the paper fixes no
 * precision.  The distance is sum_j (t_j - C[i][j])^2, j ascending, the smallest i among the smallest distances; the last
 * vector of a column is cut at M and compared over its own elements.  What is what inference restores: the centroid, or
 * with a residual codebook the binary32 sum of the two centroids rounded to binary16.
 * W: [M][N] (not modified); Hinv: [N][N]; idx, idx_res (NULL without residual): int32 [ceil(M / v)][N]; What, T: [M][N],
 * T[:, n] = column n as it stood when it was quantized (NULL: not wanted).  With given_idx (and given_idx_res) those
 * choices are taken instead of the nearest centroids: the propagation that follows from somebody else's choices.      */
int vq_oracle_quantize_columns(const double *W, const double *Hinv, int32_t M, int32_t N, const uint16_t *codebook, int32_t v, int32_t k,
                               const uint16_t *codebook_res, int32_t k_res, int32_t B, const int32_t *given_idx,
                               const int32_t *given_idx_res, int32_t *idx, int32_t *idx_res, double *What, double *T);

#ifdef __cplusplus
}
#endif
#endif
