/* vq.h -- C ABI of the MI355X (gfx950) vector-quantized linear layer.
 *
 * The layer stores, per length-v weight vector, an index into a codebook of k
 * FP16 centroids (paper Sec. 2.2 "Vector Quantization": a weight vector is
 * restored by reading the centroid its index names out of the lookup table;
 * index bits = log2(k) per vector).  Optional extras, all from the paper's parameter list
 * (App. "Parameter Description": v0,k0 / v1,k1 / k2):
 *   - a residual codebook of k_res entries with the same v, whose centroid is
 *     ADDED to the main one (Sec. 3.2.2 "Residual Vector Quantization");
 *   - outlier columns: the first n_outlier_cols input columns (of the stored
 *     order: see col_perm) are coded with a codebook of their own (v_out,
 *     k_out) and have no residual (Sec. 3.2.3 "Outlier Elimination").
 * Per-output-channel FP16 scale and bias are applied to the restored weight:
 *     W[o][c] = fp16( fma( scale[o], d[o][c], bias[o] ) ),  d in binary32.
 * Inference is two-phase (App. "Our Dequantization Implementation"): prompts
 * restore W and run a matrix product (vq_dequant, vq_gemm); decoding fuses
 * restore and matrix-vector product (vq_gemv).
 *
 * Orientation: W is [out_features][in_features] (rows = outputs).  Vector p of
 * row o covers input columns n_outlier_cols + p*v ... + v-1; P = ceil((in -
 * n_outlier_cols)/v) vectors per row; elements past in_features in the last
 * vector are decoded and dropped.
 *
 * Index streams: one per codebook.  Row o of a stream starts at byte
 * o*row_stride and is a little-endian bitstream: index p occupies bits
 * [p*b, (p+1)*b), b = ceil(log2 k) (at least 1); bit t is bit (t mod 8) of byte
 * (t div 8).  b = 8 / 16 are plain uint8 / little-endian uint16 arrays.
 * row_stride is a multiple of 16 and at least ceil(P*b/8); pad bits are
 * ignored.  An index >= k (possible only when k is not a power of two) decodes
 * to an unspecified centroid of the same table; it never causes an
 * out-of-bounds access.
 *
 * Every pointer is a DEVICE pointer owned by the caller (the descriptor itself
 * is host memory, read during the call only).  Calls enqueue work on
 * `hip_stream` (NULL = the default stream) and return without synchronising;
 * nothing is allocated, freed or retained.  Output elements outside the
 * logical extents (columns >= in_features of W, columns >= out_features of y)
 * are not written.  Return value: VQ_OK or a negative vq_status; no exception
 * crosses the boundary.  Thread-safe: the library keeps no mutable state beyond
 * once-per-process initialisations (compute-unit count, per-kernel LDS limits,
 * the device address of vq_gemv_static_workspace's array), all of them guarded.
 * The environment variable VQ_SWITCHES ("name=value,..."; read once at the
 * start of every call) forces kernel choices for tests and measurements:
 * gemv=g|m|d (generic / matrix-core / dot-product kernels), groups=loop, multi=0,
 * gemm=g|f|w|r|6, dense=0|1, dequant=g|s; unset, every choice is the library's own.
 */
#ifndef VQ_H
#define VQ_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum vq_status {
  VQ_OK = 0,
  VQ_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  VQ_ERR_SHAPE = -2,       /* a size, stride or leading dimension is out of range           */
  VQ_ERR_ALIGNMENT = -3,   /* a pointer or stride misses its required alignment             */
  VQ_ERR_UNSUPPORTED = -4, /* valid layer, but no kernel handles it                         */
  VQ_ERR_HIP = -5,         /* the HIP runtime reported a launch error                       */
  VQ_ERR_WORKSPACE = -6    /* workspace missing or smaller than vq_gemm_workspace_bytes     */
} vq_status;

typedef struct vq_layer_desc {
  uint32_t struct_size;                    /* = sizeof(vq_layer_desc), or VQ_LAYER_DESC_SIZE_V1     */
  int32_t out_features, in_features;       /* M, N (logical, unpadded); 1 .. 2^24                  */
  int32_t v, k;                            /* main codebook: v in [1,16], k in [2,65536]           */
  int32_t k_res;                           /* residual entries, 0 = none; same v                   */
  int32_t n_outlier_cols, v_out, k_out;    /* 0 = none; n % v_out == 0; n < in_features            */
  const void *codebook;                    /* fp16 [k][v] row-major, 16-byte aligned               */
  const void *codebook_res;                /* fp16 [k_res][v]                                      */
  const void *codebook_out;                /* fp16 [k_out][v_out]                                  */
  const void *idx;      int64_t idx_row_stride;       /* bytes; 16-byte aligned base and stride    */
  const void *idx_res;  int64_t idx_res_row_stride;
  const void *idx_out;  int64_t idx_out_row_stride;
  const void *scale;                       /* fp16 [out_features], 2-byte aligned; NULL = 1.0      */
  const void *bias;                        /* fp16 [out_features]; NULL = 0.0                      */
  /* Codebook groups (Sec. 3.1, the paragraph on groups; "group num" in App. "Parameter Description"): with
   * group_vectors > 0 every range of group_vectors consecutive main vectors of a row (the last range may be
   * shorter) has its own main table and, with a residual codebook, its own residual table; vector p reads the
   * tables of group p / group_vectors.  codebook is then fp16 [groups][k][v] and codebook_res fp16
   * [groups][k_res][v], groups = ceil(P / group_vectors), P = ceil((in_features - n_outlier_cols) / v).
   * 0 = one group.  Outlier columns keep their single table.  The fast kernels take group_vectors % 8 == 0.
   * A caller that sets struct_size to VQ_LAYER_DESC_SIZE_V1 (the layout up to `bias`) gets one group.    */
  int32_t group_vectors;
  /* Orientation of the vectors.  0: along the input dimension of an output row (everything above).  1: the paper's own
   * (Sec. 3.1: a quantized column is a stack of centroids; Algorithm 1 quantizes W[m:m+v, n]): a vector covers v
   * consecutive output rows of one input column.  Stream p of idx (and idx_res), p < ceil(out_features / v), belongs
   * to output rows [p v, p v + v), cut at out_features, and holds one index per main column: position t is column
   * n_outlier_cols + t, and W[p v + j][n_outlier_cols + t] is element j of its centroid.  Stream q of idx_out,
   * q < ceil(out_features / v_out), belongs to rows [q v_out, q v_out + v_out) and holds one index per outlier column
   * (n_outlier_cols need not be a multiple of v_out).  Codebook groups are ranges of group_vectors stream positions,
   * i.e. of main columns.  Scale and bias stay per output row.  This field occupies what used to be padding after
   * group_vectors: descriptors that were zeroed as a whole keep orientation 0.  Layers of orientation 1 with v = 6 /
   * 12-bit indices or v = 8 / 8- or 16-bit indices have fast vq_gemv and vq_dequant kernels of their own; others, and
   * vq_gemm without a workspace, run on the generic kernels.                                                        */
  int32_t orientation;
  /* Column order (Sec. 3.2.3: the columns that get the outlier codebook are the ones the Hessian's diagonal singles
   * out, wherever they lie; Algorithm 2's outlier step).  NULL: the stored order of the columns is the layer's.
   * Otherwise int32 [in_features] in device memory, 4-byte aligned, every column number exactly once: everything this
   * header says about "column c" then describes STORED column c, which is column col_perm[c] of the layer --
   * vq_dequant writes the value restored for (o, c) to W[o][col_perm[c]], the products multiply it with
   * x[col_perm[c]] -- and the layer's outlier columns are col_perm[0 .. n_outlier_cols).  The library does not check
   * that the array is a permutation: entries outside [0, in_features) read as zero activations and are not stored
   * by vq_dequant, repeated entries give unspecified values in the columns involved; neither leaves the buffers.
   * Kernels: vq_gemv gathers the activations itself in its one- and two-row kernels for v = 6 layers, in the kernels
   * that keep other layers' tables in LDS, and in the generic kernels; with a workspace (vq_gemv_with_workspace,
   * vq_gemv_static_workspace, vq_gemm) the activations are first gathered into it (vq_gemv_workspace_bytes / vq_gemm_fast_workspace_bytes count that copy) and every kernel of
   * the library then runs as for an unpermuted layer; vq_dequant restores in stored order and then reorders each
   * row in place through LDS.  A caller that sets struct_size to VQ_LAYER_DESC_SIZE_V2 (the layout up to
   * `orientation`) gets the identity.                                                                             */
  const int32_t *col_perm;
} vq_layer_desc;

#define VQ_LAYER_DESC_SIZE_V1 ((uint32_t)offsetof(vq_layer_desc, group_vectors))
#define VQ_LAYER_DESC_SIZE_V2 ((uint32_t)offsetof(vq_layer_desc, col_perm))

/* Host-only check of a descriptor (no GPU work): the status any entry point would return for it. */
int vq_validate(const vq_layer_desc *desc);

/* Restore the weight matrix (Sec. 2.2; App. "Our Dequantization Implementation", first phase).
 * W: fp16 [out_features][ldw], ldw >= in_features (elements), 2-byte aligned.  Bit-exact definition:
 * binary32 add of main and residual centroid, one binary32 fma with scale/bias, round-to-nearest-even
 * to binary16 (subnormals kept, overflow to infinity).                                              */
int vq_dequant(const vq_layer_desc *desc, void *W, int64_t ldw, void *hip_stream);

/* Decode-phase fused restore + matrix-vector product ("QGemv", App. "Our Dequantization
 * Implementation", second phase): y[b][o] = sum_c W[o][c] * x[b][c], binary32 accumulation, fp16
 * result.  One or two activation rows run on the vector ALUs (v_dot2_f32_f16, DPP reductions); from
 * three rows on, and for layers with codebook groups or outlier columns, the fp16 matrix cores do the
 * multiplications (the LDS lookups cost the same and the vector ALUs stop binding); VQ_SWITCHES gemv=d
 * keeps every batch on the vector ALUs.  That is the v = 6 / 12-bit layers; v = 8 with 8- or 16-bit indices gathers its
 * table from L2; the paper's other settings (v = 12 with two 4096-entry tables, v = 4 / k = 256, v = 2 / k = 16, ..., with
 * codebook groups and outlier columns of v = 4, in either orientation) run four rows a launch on the vector ALUs with
 * one table in LDS at a time; what is left runs on generic kernels.
 * x: fp16 [batch][ldx], ldx >= in_features; y: fp16 [batch][ldy],
 * ldy >= out_features; batch in [1,16]; x and y 2-byte aligned (a 16-byte aligned x with ldx % 8 == 0
 * lets the fastest kernels run).  y must not alias x.                                               */
int vq_gemv(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch,
            void *y, int64_t ldy, void *hip_stream);

/* vq_gemv with a workspace on loan (device memory, 256-byte aligned, owned by the caller, contents undefined
 * afterwards).  Only layers with codebook groups (Sec. 3.1) use it (v = 6 layers on the matrix-core kernel, the other
 * settings on the kernel that keeps one table in LDS at a time): with vq_gemv_workspace_bytes(desc, batch) bytes
 * every workgroup takes one group, whose tables it loads once, and a share of the rows, writes binary32 sums to the
 * workspace, and a second kernel adds the groups up in ascending order and applies scale and bias -- instead of every
 * workgroup walking all groups and swapping its tables for each.  Layers of orientation 1 with one group use it from
 * two rows on (from one row when a row of x does not fit the one-row kernel's LDS beside the tables: about 15000
 * columns with a 12-bit residual table): the matrix-core kernel of that orientation works in blocks of 16 index streams (96 output rows), too few
 * to fill the chip on most layers, so with a workspace it also cuts the columns into parts, one workgroup per (block,
 * part), and the same second kernel adds the parts up.  vq_gemv_workspace_bytes returns 0 when no kernel
 * would use a workspace for this layer.  With workspace NULL or smaller than that, and for every other layer, the
 * call is vq_gemv.  Same arguments, bar and errors as vq_gemv; a workspace that is not 256-byte aligned is
 * VQ_ERR_ALIGNMENT.  Calls that share a workspace must not overlap.                                          */
size_t vq_gemv_workspace_bytes(const vq_layer_desc *desc, int32_t batch);
int vq_gemv_with_workspace(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch, void *y, int64_t ldy,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/* vq_gemv_with_workspace for callers that cannot allocate device memory or hand a workspace over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a device array inside this library,
 * VQ_GEMV_STATIC_WORKSPACE_BYTES per GPU, which the GPU holds from the library's load to the end of the process; the call
 * allocates and frees nothing.  A layer and batch whose vq_gemv_workspace_bytes exceeds that size is refused with
 * VQ_ERR_WORKSPACE (nothing is launched); otherwise arguments, results and errors are those of vq_gemv_with_workspace
 * with a workspace of the size it asks for.  The kernels write every workspace element before they read it, so nothing
 * has to be cleared between calls.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams or threads) race on it and must be ordered by the caller.                                     */
#define VQ_GEMV_STATIC_WORKSPACE_BYTES (16u << 20)
int vq_gemv_static_workspace(const vq_layer_desc *desc, const void *x, int64_t ldx, int32_t batch, void *y, int64_t ldy,
                             void *hip_stream);

/* vq_gemv for several layers that read the same activations -- the query, key and value projections of a
 * decoder layer, or its gate and up projections -- as one launch: y[i][b][o] = sum_c W_i[o][c] * x[b][c] for
 * i < n_layers, each result to vq_gemv's bar for that layer (the same kernel bodies run; deterministic run to run).
 * The operation is the decode-phase product of App. "Our Dequantization Implementation", once per layer.  On this
 * GPU a decode-sized product spends more time on launch and start-up than on streaming its indices, so launching
 * less often is what speeds up decoding (the paper's own tok/s figures were taken without such measures: footnote
 * to its table of 2-bit LLaMA-2 results).
 * descs: host array of n_layers descriptor pointers, all with the same in_features; y, ldy: host arrays of
 * n_layers device pointers / leading dimensions (ldy[i] >= out_features of layer i); the outputs must not overlap
 * each other or x.  n_layers in [1, 8].  Layers that the fused kernel does not take together (different residual
 * kinds, codebook groups, both orientations, shapes outside the fast kernels) are launched one after the other on the same stream:
 * the results are the same.  Errors as for vq_gemv; nothing is launched when any argument is rejected.       */
int vq_gemv_multi(const vq_layer_desc *const *descs, int32_t n_layers, const void *x, int64_t ldx, int32_t batch,
                  void *const *y, const int64_t *ldy, void *hip_stream);

/* Encode side of the lookup: the index of the nearest centroid of every length-v vector along the rows of a weight
 * matrix (Eq. 2 of Sec. 2.2), written as the packed index stream that the entry points above read.  With B, the
 * vectors of W - B are assigned: the residual stage of Sec. 3.2.2, B being what the first stage restores.
 * W, B: fp16 [rows][ld], ld >= cols, 2-byte aligned, B may be NULL; vector p of a row = columns [p v, p v + v), the
 * last one cut at cols and compared over its own elements only.  codebook: fp16 [k][v], v in [1,16], k in [2,65536].
 * idx: [rows][idx_row_stride] bytes, 16-byte aligned base and stride, stride >= ceil(P * b / 8) rounded up to 4,
 * P = ceil(cols / v), b = ceil(log2 k); every dword that holds one of the P * b bits of a row is written (bits past
 * them zero), the rest of the stride is left alone.
 * The distance decides an integer, so its arithmetic is part of the definition: binary32, round to nearest even;
 * t_j = W - B is one subtraction; d_i = sum_j (t_j - C[i][j])^2 with one subtraction and one fused multiply-add per
 * element into a sum that starts at +0, j ascending; the result is the smallest i among the smallest d_i.      */
int vq_assign(const void *W, const void *B, int64_t ld, int32_t rows, int32_t cols, const void *codebook, int32_t v, int32_t k,
              void *idx, int64_t idx_row_stride, void *hip_stream);

/* vq_assign for the paper's own vectors (orientation 1 of the descriptor; Sec. 3.1, Algorithm 1's Q(W[m:m+V, n])):
 * vector (p, n) = W[p v + j][n], j < v, the last block of rows cut at `rows` and compared over its own elements.  idx:
 * [ceil(rows / v)][idx_row_stride] bytes, stream p holds one index per column, stride >= ceil(cols * b / 8) rounded up
 * to 4.  Everything else -- B, the arithmetic of the distance, ties, alignment, errors -- as for vq_assign.        */
int vq_assign_down(const void *W, const void *B, int64_t ld, int32_t rows, int32_t cols, const void *codebook, int32_t v,
                   int32_t k, void *idx, int64_t idx_row_stride, void *hip_stream);

/* The column loop of the quantizer (Algorithm 1, Sec. 3.1 "VPTQ Algorithm"; its error update is the Delta W equation of
 * that section): the columns of W are quantized one at a time, every column as a stack of length-v vectors (orientation 1
 * of the descriptor) that each take their nearest centroid (Eq. 2) and, with a residual codebook, a second nearest centroid
 * for what the first leaves (Sec. 3.2.2); then
 *     E[:, n] = (W[:, n] - What[:, n]) / Hinv[n][n],   W[:, n+1 : s+B] -= E[:, n] * Hinv[n][n+1 : s+B]
 * inside the block [s, s+B) of `block` columns that holds n, and W[:, s+B :] -= E[:, s : s+B] * Hinv[s : s+B][s+B :] at the
 * end of every block.  Hinv is the matrix the algorithm calls H^-1, an input: binary32 [cols][ldh], only entries on and
 * above the diagonal are read (callers in the GPTQ tradition pass the upper Cholesky factor of the inverse Hessian);
 * its diagonal must not hold zeros.
 * W: binary32 [rows][ldw], in: the weights, out: the quantized weights What -- the centroid, or with a residual codebook
 * the binary32 sum of the two centroids rounded to binary16, i.e. what vq_dequant restores from the indices with scale 1
 * and bias 0.  idx / idx_res: the packed index streams of orientation 1, [ceil(rows / v)][stride] bytes, one index per
 * column, written as vq_assign_down writes them (same stride and alignment rules; idx_res and codebook_res NULL and
 * k_res 0 without a residual codebook).  T, optional (NULL): binary32 [rows][ldt], column n as it stood when it was
 * quantized.  block in [1, 128].  workspace: vq_quantize_columns_workspace_bytes(rows, v, k, k_res) bytes of device
 * memory, 256-byte aligned, contents undefined afterwards, else VQ_ERR_WORKSPACE.
 * Arithmetic: binary32 throughout.  The distance is the one of vq_assign (one subtraction and one fused multiply-add per
 * element into a sum that starts at +0, elements ascending; the smallest index among the smallest distances; a cut-off
 * last vector is compared over its own elements); the residual vector is one subtraction per element; E is one
 * subtraction and one division; the update inside a block is one fused multiply-add per element and column; the update at
 * the end of a block is a binary32 matrix product on the matrix cores, summed in the hardware's order, then one
 * subtraction.  Several summation orders are legitimate, so results are deterministic run to run but need not equal
 * another implementation's index for index: what holds is that every index is a nearest centroid of the column as this
 * call propagated it (T), and that T follows from the call's own earlier choices by the recurrence above.            */
size_t vq_quantize_columns_workspace_bytes(int32_t rows, int32_t v, int32_t k, int32_t k_res);
int vq_quantize_columns(void *W, int64_t ldw, int32_t rows, int32_t cols, const void *Hinv, int64_t ldh, const void *codebook,
                        int32_t v, int32_t k, const void *codebook_res, int32_t k_res, int32_t block, void *idx,
                        int64_t idx_row_stride, void *idx_res, int64_t idx_res_row_stride, void *T, int64_t ldt, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

/* Prompt-phase product for many tokens: Y[t][o] = sum_c W[o][c] * X[t][c] on the FP16 matrix cores,
 * binary32 accumulation, fp16 result (the paper's prompt phase, its section on inference throughput:
 * restore the weights, then multiply).  X: fp16 [tokens][ldx], 16-byte aligned, ldx % 8 == 0; Y: fp16
 * [tokens][ldy], ldy >= out_features; tokens >= 1.
 * Workspace (device memory, 16-byte aligned, owned by the caller, contents undefined afterwards):
 *  - it must hold at least vq_gemm_workspace_bytes(desc, tokens) bytes (currently 0: NULL is fine),
 *    else VQ_ERR_WORKSPACE;
 *  - if it holds vq_gemm_fast_workspace_bytes(desc, tokens) bytes (non-zero when in_features is a
 *    multiple of 256), the call restores W into it once (as vq_dequant does) and multiplies from
 *    there, which is the faster route on this GPU; with less, the restored weights go straight from
 *    on-chip tiles into the matrix cores and W is never written to memory (kernels of their own for
 *    v = 8 / 16-bit indices, gathered from L2, and for v = 6 / 12-bit indices with one codebook group
 *    and outlier columns in multiples of 16, whose tables sit in LDS; other layers restore through the
 *    generic tile kernel).
 * Small token counts (too few tiles to fill the chip), and layers whose only tile kernel without a
 * workspace is the generic one, are computed as vq_gemv computes them, sixteen rows of X at a time,
 * where that is the faster way on this GPU: same result bar, nothing for the caller to do.          */
int vq_gemm(const vq_layer_desc *desc, const void *X, int64_t ldx, int32_t tokens,
            void *Y, int64_t ldy, void *workspace, size_t workspace_bytes, void *hip_stream);
size_t vq_gemm_workspace_bytes(const vq_layer_desc *desc, int32_t tokens);
size_t vq_gemm_fast_workspace_bytes(const vq_layer_desc *desc, int32_t tokens);

/* Text for a status code (static storage).  */
const char *vq_status_string(int status);
/* Library version, major*10000 + minor*100 + patch. */
int vq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VQ_H */
