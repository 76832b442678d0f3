/*
 * bigcn.h - C ABI of the MI355X (gfx950) Bi-GCN forward library.
 *
 * The library implements the inference path of a binary graph convolutional network
 * ("Bi-GCN", arXiv 2210.13149, Sec. 4.2): per layer, node activations are sign-binarised
 * and bit-packed with one scale per node, weights are sign-binarised with one scale per
 * output channel, the +-1 inner products are evaluated with XOR / population count, and
 * the rescaled result is aggregated with the normalised adjacency
 * A~ = D^-1/2 (A + I) D^-1/2 stored in CSR.
 *
 * Conventions common to every entry point
 *  - Pointers marked DEVICE must be device (HBM) addresses valid on the current device,
 *    allocated by the caller (e.g. torch.empty(..., device="cuda").data_ptr()).  Pointers
 *    marked HOST are ordinary host pointers.  The library never takes ownership of a
 *    caller buffer and, outside bigcn_plan_create, never allocates or frees device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *    enqueued asynchronously on it; the function returns without synchronising unless
 *    stated otherwise.
 *  - Return value: BIGCN_OK (0) or a negative bigcn_status.  Argument errors are detected
 *    on the host before anything is launched, so on error no output is touched.  The
 *    library never aborts, throws or prints.
 *  - Packed layout: a +-1 vector of length K occupies ceil(K/64) uint64 words; bit l
 *    (LSB = bit 0) of word w is 1 iff element 64*w + l is +1; bits past K are 0.
 *  - sign(0) = +1: an element is +1 iff value >= threshold.  NaN compares false (-1) and
 *    poisons the scale of its row; inputs are not screened for NaN.
 */
#ifndef BIGCN_H
#define BIGCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BIGCN_OK = 0,
    BIGCN_EINVAL = -1,     /* a size, stride or flag is out of range                    */
    BIGCN_ENULL = -2,      /* a required pointer is NULL                               */
    BIGCN_ESHAPE = -3,     /* the shape is valid but exceeds a documented limit        */
    BIGCN_EWORKSPACE = -4, /* workspace missing, too small or misaligned               */
    BIGCN_EGRAPH = -5,     /* the CSR pattern failed validation                        */
    BIGCN_EHIP = -6        /* a HIP runtime call or kernel launch failed               */
} bigcn_status;

/* Static, NUL-terminated description of a status code (never NULL). */
const char *bigcn_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int bigcn_version(void);

/* Largest supported inner dimension (bits) of bigcn_binary_gemm / a layer's d_in, and
 * largest d_out of a layer of bigcn_forward. */
#define BIGCN_MAX_K_BITS 8192
#define BIGCN_MAX_GEMM_N 4194240 /* 65535 * 64: one launch covers the columns in at most 65535 blocks of 64 */
#define BIGCN_MAX_FORWARD_D_OUT 512
#define BIGCN_MAX_LAYERS 64
/* Size of the per-GPU workspace that bigcn_forward_static uses instead of a caller buffer. */
#define BIGCN_STATIC_WORKSPACE_BYTES (32u << 20)

/*
 * Kernel 1 - binarise and pack the rows of a strided fp32 matrix
 * (Sec. 4.1: V_B = sign(V), alpha = ||V||_1 / t; Sec. 4.2.2 for node features with
 * t = d_in; Sec. 4.2.1 for the columns of a weight matrix, by passing its transpose view;
 * Sec. 4.4 step 1 for the optional standardisation of the input).
 *
 *   element (r, c) is read at x[r*row_stride + c*col_stride]              (DEVICE, fp32)
 *   x' = (x - shift[c]) * mul[c]      shift == NULL -> 0, mul == NULL -> 1  (DEVICE, cols)
 *   bits[r*ld_words + w]  packed signs, +1 iff x >= shift[c]               (DEVICE, out)
 *   scale[r] = (1/cols) * sum_c |x'|                                        (DEVICE, out)
 *
 * Packing W^T (d_out rows of length d_in) from a row-major W (d_in, d_out):
 *   bigcn_pack(W, d_out, d_in, 1, d_out, NULL, NULL, bits, ld_words, alpha, stream).
 * Only the first ceil(cols/64) words of each output row are written.
 * Errors: ENULL (x, bits or scale NULL), EINVAL (rows < 0, cols <= 0, strides <= 0,
 * ld_words < ceil(cols/64)).  rows == 0 is a no-op.
 */
int bigcn_pack(const float *x, int64_t rows, int64_t cols, int64_t row_stride,
               int64_t col_stride, const float *shift, const float *mul, uint64_t *bits,
               int64_t ld_words, float *scale, void *stream);

/*
 * Kernel 2 - binary matrix product with fused rescale (Sec. 4.2.3,
 * zeta_ij = beta_i alpha_j F_i (*) B_j with (*) = XNOR + bit count).
 *
 *   a_bits: m rows of packed signs, row stride lda_words        (DEVICE)
 *   b_bits: n rows of packed signs (row j = column j of B), row stride ldb_words (DEVICE)
 *   acc[i*ld_acc + j] = k_bits - 2*popcount(a_i xor b_j)  (int32, exact)  (DEVICE, nullable)
 *   out[i*ld_out + j] = a_scale[i] * b_scale[j] * acc_ij  (fp32)          (DEVICE, nullable)
 * At least one of acc / out must be given; a_scale and b_scale are required iff out is.
 * Pad bits (positions >= k_bits) must be equal in both operands (bigcn_pack writes 0).
 * Errors: ENULL, EINVAL (negative sizes, k_bits <= 0, leading dimensions too small),
 * ESHAPE (k_bits > BIGCN_MAX_K_BITS or n > BIGCN_MAX_GEMM_N).  m == 0 or n == 0 is a no-op.
 */
int bigcn_binary_gemm(const uint64_t *a_bits, const float *a_scale, int64_t m,
                      int64_t lda_words, const uint64_t *b_bits, const float *b_scale,
                      int64_t n, int64_t ldb_words, int64_t k_bits, int32_t *acc,
                      int64_t ld_acc, float *out, int64_t ld_out, void *stream);

/*
 * The same product with the evaluation path chosen by the caller (benchmarking and tests):
 * BIGCN_GEMM_AUTO picks per shape (what bigcn_binary_gemm does), BIGCN_GEMM_VALU evaluates
 * XOR + bit count on the vector ALU, BIGCN_GEMM_MFMA expands the bits to +-1 bytes and uses
 * the int8 matrix cores, BIGCN_GEMM_FP4 expands them to FP4 codes of +-1 and uses the
 * block-scaled matrix cores with unit scales (exact: the partial sums are integers below 2^24).
 * All paths give bit-identical acc and identical out.
 * Errors: as bigcn_binary_gemm, plus EINVAL for an unknown variant.
 */
enum { BIGCN_GEMM_AUTO = 0, BIGCN_GEMM_VALU = 1, BIGCN_GEMM_MFMA = 2, BIGCN_GEMM_FP4 = 3 };
int bigcn_binary_gemm_variant(const uint64_t *a_bits, const float *a_scale, int64_t m,
                              int64_t lda_words, const uint64_t *b_bits, const float *b_scale,
                              int64_t n, int64_t ldb_words, int64_t k_bits, int32_t *acc,
                              int64_t ld_acc, float *out, int64_t ld_out, int variant,
                              void *stream);

/*
 * Normalisation coefficients of A~ = D^-1/2 (A+I) D^-1/2 (Sec. 3.1 Notations, Eq. (1)).
 * The CSR arrays describe the pattern of A + I: symmetric, one self-loop per node,
 * columns strictly increasing inside a row; D_ii is the number of stored entries of row i.
 *
 *   row_ptr int64[n+1], col_idx int32[nnz]                      (DEVICE)
 *   dinv_sqrt[i] = D_ii^-1/2                                    (DEVICE, out, n)
 *   vals[p] = dinv_sqrt[i] * dinv_sqrt[col_idx[p]]              (DEVICE, out, nnz, nullable)
 * Errors: ENULL, EINVAL (n < 0).
 */
int bigcn_gcn_norm(const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                   float *dinv_sqrt, float *vals, void *stream);

/*
 * Aggregation schedule for one graph: rows ordered by decreasing length so that long
 * rows start first and the waves of a workgroup carry similar work.  The plan owns a
 * small amount of device memory (4 bytes per row), is immutable after creation and may
 * be used from any stream of the device it was created on.
 *
 * bigcn_plan_create copies row_ptr to the host and therefore SYNCHRONISES `stream`.
 * With validate = BIGCN_VALIDATE_GCN it also checks on the device that every column index
 * lies in [0, n), columns increase strictly inside each row, every row holds its self-loop
 * and the pattern is symmetric; BIGCN_VALIDATE_NEIGHBOURS checks the first two only (rows
 * that list N_i for the mean aggregator of Sec. 4.4.2 hold no self-loop and may be empty).
 * A violation returns BIGCN_EGRAPH and creates nothing.
 * Errors: ENULL, EINVAL (n < 0 or n >= 2^31, row_ptr not non-decreasing from 0, unknown
 * validate value),
 * EGRAPH, EHIP.  *out is set only on success.  bigcn_plan_destroy(NULL) is a no-op.
 */
typedef struct bigcn_plan bigcn_plan;
enum {
    BIGCN_VALIDATE_NONE = 0,
    BIGCN_VALIDATE_GCN = 1,        /* pattern of A + I: all four checks above            */
    BIGCN_VALIDATE_NEIGHBOURS = 2  /* neighbour lists: index range and strict order only */
};
int bigcn_plan_create(const int64_t *row_ptr, const int32_t *col_idx, int64_t n, int validate,
                      bigcn_plan **out, void *stream);
void bigcn_plan_destroy(bigcn_plan *plan);
/* Number of rows / stored entries the plan was built for. */
int64_t bigcn_plan_rows(const bigcn_plan *plan);
int64_t bigcn_plan_nnz(const bigcn_plan *plan);

/*
 * Kernel 3 - aggregation H = A~ Z as a CSR sparse-dense product (Sec. 4.2.3,
 * H_b^(l+1) = A~ zeta^(l); the aggregation itself stays in floating point, Sec. 4):
 *
 *   out[i*ld_out + j] = sum_{p in row i} vals[p] * z[col_idx[p]*ld_z + j],  j < d
 *
 * vals == NULL means all ones.  z (n rows, d columns, fp32) and out must not overlap.
 * Each output element is a sum in a fixed order, so results are run-to-run identical.
 * `plan` must have been created from the same row_ptr / col_idx.
 * Errors: ENULL, EINVAL (n differs from the plan's, d <= 0, ld_z < d or ld_z >= 2^29, ld_out < d).
 */
int bigcn_spmm(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
               const float *vals, int64_t n, const float *z, int64_t d, int64_t ld_z,
               float *out, int64_t ld_out, void *stream);

/*
 * One binarised graph-convolution layer (Sec. 4.2): packed weights and scales as produced
 * by bigcn_pack on the transposed weight matrix, and the optional frozen standardisation
 * (Sec. 4.4 step 1) applied to the layer's *input* before it is binarised.
 */
typedef struct {
    const uint64_t *w_bits; /* DEVICE: d_out rows of packed signs of W[:, j], stride ld_words */
    const float *alpha;     /* DEVICE: d_out scales alpha_j = ||W[:, j]||_1 / d_in           */
    int64_t d_in;
    int64_t d_out;
    int64_t ld_words;       /* >= ceil(d_in/64)                                             */
    const float *bn_shift;  /* DEVICE, d_in, nullable: threshold / mean of each input column */
    const float *bn_mul;    /* DEVICE, d_in, nullable: 1/sqrt(var + eps) of each column      */
} bigcn_layer;

/*
 * Fused L-layer forward (Eq. (1) with H^(0) = X; per layer Sec. 4.2.3):
 *   for l = 0..L-1:  (F, beta) = binarise(standardise_l(H^(l)));  C = F (*) B_l;
 *                    H^(l+1) = A~ (beta_i alpha_j C_ij)
 * and logits = H^(L) (no bias, no ReLU, no softmax).  Hidden activations are never stored
 * in fp32: the aggregation of layer l emits the packed signs and scales of layer l+1.
 *
 *   plan, row_ptr, col_idx : the graph (pattern of A + I)                 (DEVICE arrays)
 *   dinv_sqrt              : output of bigcn_gcn_norm for the same graph   (DEVICE, n)
 *   x                      : fp32 node features, n rows of layers[0].d_in, row stride ld_x (DEVICE)
 *   layers                 : HOST array of n_layers descriptors; layers[l+1].d_in must equal
 *                            layers[l].d_out
 *   logits                 : n rows of layers[L-1].d_out fp32, row stride ld_logits (DEVICE, out)
 *   workspace              : DEVICE scratch of at least bigcn_forward_workspace_bytes(...)
 *                            bytes, 256-byte aligned; contents are undefined afterwards
 * Errors: ENULL, EINVAL (also n_layers > BIGCN_MAX_LAYERS), ESHAPE (d_in > BIGCN_MAX_K_BITS or
 * d_out > BIGCN_MAX_FORWARD_D_OUT), EWORKSPACE.  bigcn_forward_workspace_bytes returns 0 for
 * invalid arguments.
 */
size_t bigcn_forward_workspace_bytes(int64_t n, const bigcn_layer *layers, int n_layers);
/* Bytes of the compact row of integer products (Sec. 4.2.3, F_i (*) B_j for all j) that the
 * fused forward keeps per node for a layer with d_in input bits and d_out columns, and
 * whether the node's source scale is stored inside that row (*scale_embedded, HOST,
 * nullable).  Used to size the aggregation's gather traffic; 0 for unsupported shapes. */
int64_t bigcn_forward_row_bytes(int64_t d_in, int64_t d_out, int *scale_embedded);
/*
 * Inspection of the intermediate integer products (Sec. 4.2.3, F_i (*) B_j) that bigcn_forward leaves
 * in its workspace, for tests and tools that check them against a reference.
 *
 * bigcn_forward_row_layout: fields[0..7] (HOST, int32) = {groups G, values per lane V, kind, K',
 * fold_last, scale_place, escape, alt_kind} of the compact row of a layer with d_in input bits and
 * d_out columns:
 *   - a row has G*V stored positions; position g*V + v holds output column g + G*v (columns >= d_out
 *     hold no product);
 *   - kind 0: one byte, q = floor(K'/2) - popcount over the first K' input bits, so the product over
 *     those bits is 2q + (K' mod 2); kind 1 / 2: the product itself as fp16 / fp32;
 *   - fold_last 1: K' = d_in - 1; the last input bit's term f_{i,K-1} b_{K-1,j} is added by the
 *     aggregation (the sign f_{i,K-1} rides on the sign of the node's stored scale);
 *   - scale_place 0: no scale in the row; 1: its last 4 bytes hold the node's fp32 scale; 2: the
 *     values use 7 bits (two's complement in bits 0..6) and bit 7 of byte 8i (rows of 32 or 64 lanes,
 *     i < 32) or of bytes 8i and 8i + 4 (rows of 16 lanes: scale bits i and 16 + i) carries a bit
 *     of the scale; 3: the last byte of lanes 4..7 of an 8-lane row holds byte 0..3 of the scale;
 *   - escape 1: a row whose values do not all fit carries a NaN as its scale and its values live at
 *     the same positions of the alternate array, as bytes (alt_kind 0) or fp16 (alt_kind 1), with
 *     its scale in the per-node scale array.  With scale_place 2 "fit" means 7 bits; with
 *     scale_place 3 (more than 256 input bits, at most 60 columns: 8-bit values) it means
 *     [-127, 126], the range in which a byte cannot be a saturated conversion.
 * bigcn_forward_workspace_map: offsets[0..5] (HOST) = byte offsets inside the workspace of
 * {packed signs of the hidden layers, scale array 0, scale array 1, product rows, alternate rows,
 * total size}; row i of the product array starts at rows + i * (row bytes of the layer that ran
 * last).  Layer l uses scale array l mod 2.
 * Errors: ENULL, EINVAL (shapes the forward does not take).
 */
int bigcn_forward_row_layout(int64_t d_in, int64_t d_out, int32_t *fields);
int bigcn_forward_workspace_map(int64_t n, const bigcn_layer *layers, int n_layers, size_t *offsets);
/* Which evaluation of the binary product (Sec. 4.2.3) the fused forward uses for a layer of a graph
 * of n nodes: BIGCN_GEMM_FP4 (matrix cores) or BIGCN_GEMM_VALU (XOR + bit count); both are exact.
 * For reports: the arithmetic peak a layer's bit-GEMM is compared with.  EINVAL for shapes the
 * forward does not take. */
int bigcn_forward_gemm_path(int64_t n, int64_t d_in, int64_t d_out);
int bigcn_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                  const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                  const bigcn_layer *layers, int n_layers, float *logits, int64_t ld_logits,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * bigcn_forward for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments,
 * kernels and results as bigcn_forward, with the workspace taken from a device array of
 * BIGCN_STATIC_WORKSPACE_BYTES that is part of the library's code object (one copy per GPU
 * that loads the library, held until the process ends).  The call allocates and frees nothing
 * and clears nothing with a memset: every workspace region is written by a kernel of the call
 * before a kernel of the same call reads it, so stale contents of an earlier call are harmless.
 *
 *  - Problems whose bigcn_forward_workspace_bytes(n, layers, n_layers) exceeds
 *    BIGCN_STATIC_WORKSPACE_BYTES are rejected with BIGCN_ESHAPE before anything is launched
 *    (the three citation-network workloads need 0.9, 2.4 and 9.0 MB).
 *  - All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different
 *    streams, or graph replays that run concurrently) race.  Calls on one stream are ordered.
 *  - The first call on each device looks the array's address up (hipGetSymbolAddress); make it
 *    outside stream capture.  The plan still comes from bigcn_plan_create, at set-up.
 * Errors: as bigcn_forward without EWORKSPACE; ESHAPE also for the size limit above; EHIP if the
 * address lookup fails.
 */
int bigcn_forward_static(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                         const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                         const bigcn_layer *layers, int n_layers, float *logits, int64_t ld_logits,
                         void *stream);

/*
 * The same forward from an input that is already binarised (Sec. 5.2: the loaded features can
 * be kept as N*d bits plus N scales, which is what makes the data-size reduction of that
 * section usable at run time): (x_bits, x_beta) are the outputs of bigcn_pack on X, with the
 * first layer's standardisation, if any, applied in that call.
 *
 *   x_bits : n rows of packed signs, row stride ld_x_words >= ceil(layers[0].d_in/64)  (DEVICE)
 *   x_beta : n row scales                                                            (DEVICE)
 * layers[0].bn_shift and bn_mul must be NULL (EINVAL otherwise).  The result is bit-identical
 * to bigcn_forward on the fp32 X those bits came from.  Other arguments and errors as
 * bigcn_forward; the same workspace size applies.
 */
int bigcn_forward_packed(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                         const float *dinv_sqrt, int64_t n, const uint64_t *x_bits,
                         int64_t ld_x_words, const float *x_beta, const bigcn_layer *layers,
                         int n_layers, float *logits, int64_t ld_logits, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Frozen standardisation parameters from data (Sec. 4.4, first step of the binarisation
 * recipe: the input of a binarised layer is brought to zero mean and unit variance; Sec. 7.2):
 * per column c of an fp32 matrix (rows x cols, row stride ld),
 *
 *   shift[c] = mean_r x[r, c],    mul[c] = 1 / sqrt(var_r x[r, c] + eps)   (biased variance)
 *
 * accumulated in fp64 in a fixed order (run-to-run identical) and rounded to fp32: the two
 * vectors are what bigcn_pack and the layer descriptors take as bn_shift / bn_mul.
 *   x DEVICE; shift, mul DEVICE out (cols floats each); workspace DEVICE scratch of at least
 *   bigcn_column_stats_workspace_bytes(rows, cols) bytes, 8-byte aligned.
 * Errors: ENULL, EINVAL (rows <= 0, cols <= 0, ld < cols, eps negative or NaN), ESHAPE
 * (cols > 2^24), EWORKSPACE.  The size query returns 0 for invalid arguments.
 */
size_t bigcn_column_stats_workspace_bytes(int64_t rows, int64_t cols);
int bigcn_column_stats(const float *x, int64_t rows, int64_t cols, int64_t ld, double eps,
                       float *shift, float *mul, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * Prediction from the last layer's output (Sec. 3.2: Y~ = softmax(H^(L)); the predicted class
 * of a node is the largest entry of its row):
 *
 *   labels[i] = argmax_c logits[i*ld + c]   (lowest c among equal maxima)   (DEVICE, int32, nullable)
 *   probs[i*ld_probs + c] = softmax_c(logits[i, :])                          (DEVICE, fp32, nullable)
 *
 * At least one output must be given.  Rows containing NaN give unspecified results.
 * Errors: ENULL, EINVAL (n < 0, d <= 0, ld < d, ld_probs < d with probs), ESHAPE (d > 2^20 or
 * n > 2^38).
 */
int bigcn_predict(const float *logits, int64_t n, int64_t d, int64_t ld, int32_t *labels,
                  float *probs, int64_t ld_probs, void *stream);

/*
 * Back propagation through one binarised graph-convolution layer (Sec. 4.3, Algorithm 1 and the
 * two gradient rules of that section).  With g_out = dL/dH^(l+1):
 *
 *   g_zeta = A~^T g_out
 *   g_wt   = H~^T g_zeta            H~ = beta_i F_i   (the layer input as bigcn_pack produced it)
 *   g_ht   = g_zeta W~^T            W~ = alpha_j B_j  (from the fp32 weights w)
 *   g_in   = g_ht * 1[|g_ht| < 1] * bn_mul[t]         (clipped straight-through rule; bn_mul, if
 *                                                     given, is the frozen standardisation factor
 *                                                     of the layer input)
 *   g_w[t,j] = sign(w[t,j]) (sum_k g_wt[k,j] sign(w[k,j])) / d_in
 *              + alpha_j g_wt[t,j] 1[|w[t,j]| < 1]
 *
 *   plan, row_ptr, col_idx, vals : the graph and the coefficients of A~ (bigcn_gcn_norm); vals
 *                                  must be symmetric, as those are, so that A~^T = A~   (DEVICE)
 *   g_out  : n rows of d_out fp32, row stride ld_g                                    (DEVICE)
 *   f_bits : n rows of packed input signs, row stride ld_f_words; beta: n scales      (DEVICE)
 *   w      : fp32 weights, d_in rows of d_out, row stride ld_w                        (DEVICE)
 *   g_w    : d_in rows of d_out fp32, row stride ld_gw                                (DEVICE, out)
 *   g_in   : n rows of d_in fp32, row stride ld_gin; NULL skips it (first layer)      (DEVICE, out)
 *   workspace : at least bigcn_layer_backward_workspace_bytes(n, d_in, d_out) bytes, 256-byte
 *               aligned (holds g_zeta, both packings of w and the partial sums over node chunks)
 * Sums over the nodes are taken in a fixed order: results are run-to-run identical.
 * Without g_in and with d_in <= d_out (the first layer of a model) g_wt is evaluated as
 * (A~ H~)^T g_out, the same value since A~ is symmetric: the aggregation then gathers packed sign
 * rows instead of fp32 gradient rows.  Its rounding differs from the other order's in the last
 * bits, so g_w with and without g_in need not be bit-identical for such shapes.
 * Errors: ENULL, EINVAL (n differs from the plan's, sizes <= 0, leading dimensions too small),
 * ESHAPE (d_in or d_out > BIGCN_MAX_K_BITS), EWORKSPACE.  The size query returns 0 for invalid
 * arguments.
 */
size_t bigcn_layer_backward_workspace_bytes(int64_t n, int64_t d_in, int64_t d_out);
int bigcn_layer_backward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                         const float *vals, int64_t n, const float *g_out, int64_t ld_g,
                         const uint64_t *f_bits, int64_t ld_f_words, const float *beta,
                         const float *w, int64_t ld_w, int64_t d_in, int64_t d_out,
                         const float *bn_mul, float *g_w, int64_t ld_gw, float *g_in,
                         int64_t ld_gin, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One Bi-GAT layer (Sec. 4.4.1): z_j = W~ (*) h~_j (binarise+pack of x with the optional
 * standardisation, then the binary product of Sec. 4.2.3) and, for each of `heads` blocks of
 * d_out / heads columns,
 *
 *   e_ij = LeakyReLU(a_src . z_i + a_dst . z_j)     (a^T (z_i || z_j); a is not binarised)
 *   a_ij = softmax over j in N_i of e_ij            (row i of the CSR lists N_i as given)
 *   out_i = sum_{j in N_i} a_ij z_j                 (no further non-linearity)
 *
 *   plan, row_ptr, col_idx : the graph (any validated pattern)                       (DEVICE)
 *   x : n rows of d_in fp32, row stride ld_x; bn_shift / bn_mul: d_in, nullable       (DEVICE)
 *   w_bits, alpha, ld_words : packed weights as in bigcn_layer (d_out rows)           (DEVICE)
 *   a_src, a_dst : d_out floats each, head-major (head h owns entries h*d_out/heads ..) (DEVICE)
 *   out : n rows of d_out fp32, row stride ld_out; a node with an empty row gets zeros (DEVICE)
 *   workspace : at least bigcn_gat_layer_workspace_bytes(...) bytes, 256-byte aligned
 * Sums are taken in a fixed order: results are run-to-run identical.
 * Errors: ENULL, EINVAL (sizes, strides, d_out not a multiple of heads), ESHAPE (heads not in
 * {1, 2, 4, 8}, d_out > 512, d_in > BIGCN_MAX_K_BITS), EWORKSPACE.  The size query returns 0
 * for invalid arguments.
 */
size_t bigcn_gat_layer_workspace_bytes(int64_t n, int64_t d_in, int64_t d_out, int heads);
int bigcn_gat_layer(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx, int64_t n,
                    const float *x, int64_t ld_x, const float *bn_shift, const float *bn_mul,
                    const uint64_t *w_bits, const float *alpha, int64_t ld_words, int64_t d_in,
                    int64_t d_out, int heads, const float *a_src, const float *a_dst,
                    float negative_slope, float *out, int64_t ld_out, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * Entropy estimate of a hidden layer by binning (Sec. 6.2), used by the paper to choose the width
 * of a binarised layer: neuron c (a column of h, one row per node) is discretised into `bins`
 * equal-width intervals over its own [min, max],
 *
 *   per_neuron[c] = - sum_m p_m log2 p_m,  p_m = count_m / rows;     *total = sum_c per_neuron[c]
 *
 * The bin of a value is decided in fp32 as min(bins - 1, floor((x - lo) * (bins / (hi - lo)))),
 * each operation rounded; a constant neuron falls into bin 0.  Counting is exact.
 *   h DEVICE fp32 (rows x cols, row stride ld); per_neuron DEVICE out, cols doubles, nullable;
 *   total DEVICE out, one double; counts DEVICE out, cols * bins uint32 (row c = neuron c),
 *   nullable; workspace DEVICE, at least bigcn_entropy_workspace_bytes(cols, bins) bytes,
 *   256-byte aligned.
 * Errors: ENULL, EINVAL (rows <= 0, cols <= 0, ld < cols, bins < 1), ESHAPE (bins > 1024,
 * cols > BIGCN_MAX_K_BITS, rows >= 2^32), EWORKSPACE.  The size query returns 0 for invalid arguments.
 */
size_t bigcn_entropy_workspace_bytes(int64_t cols, int bins);
int bigcn_entropy(const float *h, int64_t rows, int64_t cols, int64_t ld, int bins,
                  double *per_neuron, double *total, uint32_t *counts, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * Bi-GraphSAGE with the mean aggregator (Sec. 4.4.2, the binarised layer):
 *
 *   h_i^(l+1) = W~_theta (*) h~_i  +  (1/|N_i|) sum_{j in N_i} W~_n (*) h~_j
 *
 * with (*) the binarised product of Sec. 4.2 (beta_i alpha_j c_ij), no non-linearity, and
 * the same optional standardisation of each layer's input.  Row i of the CSR lists N_i as
 * given (pass the graph without self-loops for the usual aggregator); a node with an empty
 * row keeps only its own term.
 *
 * bigcn_mean_norm: inv_deg[i] = 1/|N_i| (0 for an empty row).   row_ptr DEVICE int64[n+1],
 * inv_deg DEVICE out, n floats.  Errors: ENULL, EINVAL (n < 0).
 *
 * bigcn_sage_forward: arguments as bigcn_forward, with inv_deg in place of dinv_sqrt, a plan
 * created from the neighbour-list CSR, and `out` = h^(L) (n rows of layers[L-1].d_out fp32).
 * Per layer two bit-GEMMs run (one per weight matrix) and one aggregation; the workspace
 * holds two product arrays.  Errors as bigcn_forward.  Profiled variant: slot 1 + 2l covers
 * both bit-GEMMs of layer l.
 */
typedef struct {
    const uint64_t *w_self_bits; /* DEVICE: packed signs of W_theta[:, j], d_out rows        */
    const float *alpha_self;     /* DEVICE: d_out scales of W_theta                          */
    const uint64_t *w_nbr_bits;  /* DEVICE: packed signs of W_n[:, j], d_out rows            */
    const float *alpha_nbr;      /* DEVICE: d_out scales of W_n                              */
    int64_t d_in;
    int64_t d_out;
    int64_t ld_words;            /* row stride of both packed matrices, >= ceil(d_in/64)     */
    const float *bn_shift;       /* DEVICE, d_in, nullable                                   */
    const float *bn_mul;         /* DEVICE, d_in, nullable                                   */
} bigcn_sage_layer;
int bigcn_mean_norm(const int64_t *row_ptr, int64_t n, float *inv_deg, void *stream);
size_t bigcn_sage_forward_workspace_bytes(int64_t n, const bigcn_sage_layer *layers, int n_layers);
int bigcn_sage_forward(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                       const float *inv_deg, int64_t n, const float *x, int64_t ld_x,
                       const bigcn_sage_layer *layers, int n_layers, float *out, int64_t ld_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Per-launch timing of the fused forward (measurement aid; HIP events on the caller's
 * stream).  One forward issues 1 + 2L launches: slot 0 is the binarise+pack of X
 * (Sec. 4.2.2), slot 1 + 2l the bit-GEMM of layer l and slot 2 + 2l its aggregation
 * (Sec. 4.2.3).  A profile holds the events of up to max_calls (<= 4096) calls.
 *
 * bigcn_forward_profiled is bigcn_forward plus one event record before / after every
 * launch; it fails with BIGCN_ESHAPE once max_calls calls are pending and BIGCN_EINVAL if
 * the profile was created for another layer count.
 * bigcn_profile_read waits for the recorded calls to finish (it SYNCHRONISES with them),
 * writes the mean duration of every slot in milliseconds to launch_ms (HOST, 1 + 2L
 * floats) and the number of calls averaged to *calls (HOST, nullable), and resets the
 * profile (also when it returns an error).  A forward that fails after some of its launches is not
 * counted.  A profile must not be used from two threads at once.
 */
typedef struct bigcn_profile bigcn_profile;
int bigcn_profile_create(int n_layers, int max_calls, bigcn_profile **out);
void bigcn_profile_destroy(bigcn_profile *profile);
int bigcn_forward_profiled(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                           const float *dinv_sqrt, int64_t n, const float *x, int64_t ld_x,
                           const bigcn_layer *layers, int n_layers, float *logits,
                           int64_t ld_logits, void *workspace, size_t workspace_bytes,
                           void *stream, bigcn_profile *profile);
int bigcn_sage_forward_profiled(const bigcn_plan *plan, const int64_t *row_ptr, const int32_t *col_idx,
                                const float *inv_deg, int64_t n, const float *x, int64_t ld_x,
                                const bigcn_sage_layer *layers, int n_layers, float *out,
                                int64_t ld_out, void *workspace, size_t workspace_bytes,
                                void *stream, bigcn_profile *profile);
int bigcn_profile_read(bigcn_profile *profile, float *launch_ms, int *calls);

/*
 * Measurement aid for the matrix-core evaluation of the binary product (Sec. 4.2.3): a launch of
 * nothing but independent 32 x 32 x 64 FP4 multiplies on pseudo-random +-1 codes, one wavefront
 * per SIMD with sixteen accumulator tiles, `iterations` x 16 multiplies per wavefront.  Timed by
 * the caller (events on `stream`), it gives the multiply rate this device sustains when loads,
 * code expansion and stores cost nothing: the ceiling the FP4 path of bigcn_binary_gemm is
 * compared with beside the published peak.
 *   sink: DEVICE, at least 256 floats per compute unit (sink_floats says how many there are);
 *   *multiply_accumulates: HOST out, +-1 multiply-accumulates the launch performs.
 * Errors: ENULL, EINVAL (iterations outside 1 .. 2^20), EWORKSPACE (sink too small), EHIP.
 */
int bigcn_probe_fp4_multiply_rate(int iterations, float *sink, int64_t sink_floats,
                                  int64_t *multiply_accumulates, void *stream);
/*
 * The same launch with the one step that a bit-packed input (Sec. 4.2.2) cannot avoid put back:
 * the eight operands of every sixteen multiplies are expanded from 32 packed bits each to FP4
 * codes with the instructions the FP4 path of bigcn_binary_gemm uses (28 vector instructions for
 * four row and four column operands, plus one rotate each to vary the bits), issued three at a
 * time between the multiplies of the step before.  Loads and stores still cost nothing, so this is
 * the rate a kernel fed with packed bits is compared with.  Arguments and errors as above.
 */
int bigcn_probe_fp4_expand_multiply_rate(int iterations, float *sink, int64_t sink_floats,
                                         int64_t *multiply_accumulates, void *stream);

/*
 * Measurement aid for the steps bound by reading their input once (binarise + pack of Sec. 4.2.2,
 * the column statistics of Sec. 4.4): a launch that only reads `bytes` bytes (a multiple of 16 is
 * read; src DEVICE, 16-byte aligned), every workgroup one contiguous piece, a thread eight
 * 16-byte loads at a time.  Timed by the caller, it gives the read rate such a step is compared
 * with beside the published HBM peak.
 *   sink: DEVICE, at least 8192 floats per compute unit (sink_floats says how many there are).
 * Errors: ENULL, EINVAL (fewer than 16 bytes, misaligned src), EWORKSPACE (sink too small), EHIP.
 */
int bigcn_probe_stream_read(const void *src, int64_t bytes, float *sink, int64_t sink_floats, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BIGCN_H */
