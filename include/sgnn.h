/*
 * sgnn - the single-GPU hot path of mini-batch GCN training with uniform vertex sampling
 * (ScaleGNN, arXiv 2604.02651), as a C library of hand-written HIP kernels for gfx950.
 *
 * One training step (Algorithm 1 of the paper, without the parameter update) is
 *     sgnn_sample_uniform   S ~ Uniform(B-subsets of V)                        (Eq. 20)
 *     sgnn_induced_csr      A~[S,S]: induced edges, normalised, rescaled by 1/p (Eqs. 21-24)
 *     sgnn_gather_rows      X_S = X[S], Y_S = Y[S]                              (Eq. 26)
 *     sgnn_gcn_fwd  x L     T = A~ H (SpMM), Y = act(T W + b) (GEMM)            (Eqs. 5-6, 8)
 *     sgnn_softmax_xent     mean cross-entropy and its gradient                 (Sec. III-B)
 *     sgnn_gcn_bwd  x L     dW = T^T dZ, dT = dZ W^T, dH = A~^T dT              (Sec. III-C)
 *
 * Conventions
 *  - Every array pointer is a DEVICE pointer owned by the caller unless a parameter says "host".
 *    The library neither allocates nor frees caller-visible memory.  Its own scratch lives in
 *    the context and grows only inside sgnn_ctx_reserve().
 *  - Every call is asynchronous on the HIP stream passed last (a hipStream_t, passed as void*;
 *    NULL is the default stream) and does not synchronise unless a host out-pointer is given.
 *  - A context must be used from one stream at a time: calls that share a context and overlap
 *    on different streams race on its scratch.  Use one context per concurrent stream.
 *  - Matrices are dense row-major with a leading dimension in elements.
 *  - Return value: SGNN_OK or a negative error code; sgnn_last_error() gives the message of the
 *    last failing call on that context.  No call throws.
 */
#ifndef SGNN_H
#define SGNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SGNN_OK = 0,
    SGNN_ERR_INVALID_ARG = -1, /* null pointer, B == 0, B > N, shape mismatch ...                  */
    SGNN_ERR_CAPACITY = -2,    /* an output buffer or the reserved scratch is too small             */
    SGNN_ERR_UNSUPPORTED = -3, /* a valid request this build does not implement                     */
    SGNN_ERR_HIP = -4,         /* a HIP runtime call failed; the message names it                   */
    SGNN_ERR_INTERNAL = -5     /* a device-side consistency check failed (see sgnn_ctx_status)      */
};

enum { SGNN_F32 = 0, SGNN_BF16 = 1 };

/* layer flags */
enum {
    SGNN_RELU = 1,      /* Y = max(Z, 0) (Eq. 8); backward masks dY where Y <= 0                    */
    SGNN_BF16_MFMA = 2, /* round both GEMM operands to bfloat16 (nearest even), accumulate in fp32  */
    SGNN_DY_MASKED = 8, /* backward only: dY already carries the ReLU mask of this layer's output (the
                           layer above was given H_in), so it is not applied again                   */
    SGNN_FUSE_TAIL = 16, /* sgnn_gemm_tail_fwd only: run the tail in the epilogue of the product (see there)  */
    SGNN_XFORM_FIRST = 4 /* evaluate A (H W) instead of (A H) W: the same result up to rounding, with
                            the sparse product at width d_out; worth it when d_out < d_in           */
};

typedef struct sgnn_ctx sgnn_ctx;
typedef void *sgnn_stream; /* hipStream_t */

/* Context: binds a device, owns scratch.  `device` is a HIP device ordinal. */
int sgnn_ctx_create(sgnn_ctx **out, int device);
int sgnn_ctx_destroy(sgnn_ctx *ctx);

/*
 * Size the scratch for graphs of up to N vertices and E stored entries, samples of up to B
 * vertices, layers of width up to d_max and mini-batch matrices with room for up to max_entries
 * entries (their sgnn_csr.capacity).  The only call that allocates device memory
 * (hipMalloc); it synchronises the device when it has to grow.  Later calls that need more
 * scratch than reserved fail with SGNN_ERR_CAPACITY.
 */
int sgnn_ctx_reserve(sgnn_ctx *ctx, uint64_t N, uint64_t E, uint32_t B, uint32_t d_max,
                     uint64_t max_entries);

/* Message of the last error on this context ("" if none).  Host string owned by the context. */
const char *sgnn_last_error(const sgnn_ctx *ctx);

/*
 * Synchronises `stream` and reads the device-side status word that kernels set when a
 * check on the device fails, and clears the word.  Returns SGNN_OK; SGNN_ERR_CAPACITY if the
 * only finding is that an asynchronous sgnn_induced_csr (nnz_host == NULL) produced more entries
 * than out->capacity (the surplus was dropped, so whatever was computed from that matrix is
 * invalid); SGNN_ERR_INTERNAL for a failed consistency check (sampler candidate buffer overflow,
 * an entry count of 2^31 or more).
 */
int sgnn_ctx_status(sgnn_ctx *ctx, sgnn_stream stream);

/*
 * Per-kernel timing for benchmarks.  With enable != 0 every kernel launch made through this
 * context is bracketed by two HIP events recorded on the launch's own stream (this costs a few
 * microseconds per launch, so throughput is measured with profiling off); enabling also discards
 * earlier records.  sgnn_ctx_profile_read synchronises the device and writes one line per
 * (kernel, shape tag) into the host buffer: "name<TAB>tag<TAB>launches<TAB>total milliseconds".
 */
int sgnn_ctx_profile(sgnn_ctx *ctx, int enable);
int sgnn_ctx_profile_read(sgnn_ctx *ctx, char *buf /* host */, uint64_t buf_len);

/*
 * Eq. 20: uniform sample of B of the N vertices without replacement.
 * The sample is the B vertices with the smallest (key(v), v), key(v) = 64 bits of
 * Philox4x32-10 with key words (seed lo, seed hi) and counter (v/2 lo, v/2 hi, step lo, step hi);
 * vertex 2j takes output words (1,0), vertex 2j+1 words (3,2), high word first.  It depends on
 * (N, B, seed, step) only, so every process that passes the same four values gets the same S.
 *   S       out int32[B], ascending
 *   bitmap  out uint64[ceil(N/64)], bit v%64 of word v/64 set iff v in S; the unused high bits of
 *           the last word are zero
 *   rank    out uint32[ceil(N/64)], rank[w] = number of sampled vertices below 64*w, so the
 *           position of a sampled v in S is rank[v/64] + popcount(bitmap[v/64] & ((1<<v%64)-1))
 * Errors: B == 0, B > N, N >= 2^31, null pointers -> SGNN_ERR_INVALID_ARG; scratch -> CAPACITY.
 * Debugging switch: the environment variable SGNN_SAMPLER_WINDOW_SHIFT (an integer, read at every call) moves
 * the window of histogram bins in which a sparse sample of a large graph looks for its threshold, so that the
 * passes taken when the window misses can be tested; the result does not depend on it.
 */
int sgnn_sample_uniform(sgnn_ctx *ctx, uint64_t N, uint32_t B, uint64_t seed, uint64_t step,
                        int32_t *S, uint64_t *bitmap, uint32_t *rank, sgnn_stream stream);

/*
 * The same sample for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It takes no context (creating one allocates) and runs on
 * the CURRENT device; the kernels are those of sgnn_sample_uniform, and so are S, bitmap and rank, bit for bit.
 * The sampler's scratch (histogram, selection state, candidate list, workgroup counts: 1.7 MB) is a
 * file-scope device array inside the library, of which every GPU the library runs on holds one copy until
 * the process ends; its address is looked up once per device (by sgnn_ctx_create on that device, else by the
 * first call here) and the call itself makes no hipMalloc / hipFree and no allocating library call.
 *   N           at most SGNN_STATIC_SAMPLER_MAX_N (what the array is sized for); beyond it SGNN_ERR_CAPACITY
 *   status_dev  device uint32[1] or NULL: sticky error bits OR-ed in by the kernels (bit 0: the selection was
 *               inconsistent - candidate list overflow, probability below 1e-15 for Philox keys); with NULL the
 *               bits go to a word inside the array that nothing reads
 * All calls on one GPU share that GPU's array, whichever stream they use: two calls that overlap in time on
 * one GPU race.  What has to start at zero is cleared by a kernel at the start of every call (no memset node,
 * so the call can be captured into a HIP graph).
 * Errors as sgnn_sample_uniform; the message of a failure is returned by sgnn_last_error(NULL) on the
 * calling thread.
 */
#define SGNN_STATIC_SAMPLER_MAX_N (1ull << 27)
int sgnn_sample_uniform_static(uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S, uint64_t *bitmap,
                               uint32_t *rank, uint32_t *status_dev, sgnn_stream stream);

/*
 * The full graph: canonical CSR of A + I (Eq. 3) - ascending unique columns in every row and
 * exactly one self-loop per row.  rowptr has N+1 entries of int32 or int64.
 * val == NULL: a_vu = 1/sqrt(deg(v) deg(u)), deg = row length (self-loop included);
 * val != NULL: fp32[E] weights taken verbatim (Algorithm 2 lists them as an input).
 */
typedef struct {
    uint64_t N;
    uint64_t E; /* number of stored entries = rowptr[N] */
    const void *rowptr;
    int rowptr_is_i64;
    const int32_t *colidx;
    const float *val;
} sgnn_graph;

/*
 * A mini-batch matrix in CSR: rows x cols, int32 rowptr[rows+1], colidx/val with room for
 * `capacity` entries.  nnz_dev (device uint32[1], may be NULL) receives the number of entries.
 * plan (may be NULL) is a device buffer of sgnn_csr_plan_bytes(rows, capacity) bytes that holds
 * the split of the long rows into chunks used by the sparse products.  sgnn_induced_csr fills it
 * for the matrix it writes; sgnn_csr_plan fills it for any other matrix.  It stays valid while
 * rows, capacity and the contents of rowptr do not change.  Without a plan every sparse product
 * builds a temporary one in the context scratch (two more small kernel launches per product).
 */
typedef struct {
    uint32_t rows, cols;
    int32_t *rowptr;
    int32_t *colidx;
    float *val;
    uint64_t capacity;
    uint32_t *nnz_dev;
    void *plan;
    int rowptr_is_i64; /* 0: rowptr is int32 (every matrix the library writes); 1: rowptr points at int64
                        * offsets - a full graph with 2^31 entries or more as the matrix of a sparse product
                        * (sgnn_spmm, sgnn_gcn_fwd, sgnn_csr_plan); other calls refuse such a matrix */
} sgnn_csr;

uint64_t sgnn_csr_plan_bytes(uint32_t rows, uint64_t capacity);
int sgnn_csr_plan(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_stream stream);

/*
 * Eqs. 21-24 / Algorithm 2 with the full row and column range: for i in [0,B), v = S[i], keep
 * every u in row v of the graph with u in S; column = position of u in S (ascending within the
 * row); value = a_vu / p for u != v and a_vv for u == v, p = (B-1)/(N-1).
 *   S, bitmap, rank   as written by sgnn_sample_uniform for the same N and B
 *   norm_mode 0       a_vu inherited from the full graph (the paper's definition)
 *   norm_mode 1       a_vu recomputed from the degrees of the induced subgraph (val ignored)
 *   rescale   1       divide off-diagonal entries by p;  0: leave them
 *   out               rows/cols are set to B; rowptr[B+1] always complete; colidx/val are written
 *                     up to out->capacity entries
 *   nnz_host          NULL: fully asynchronous; an entry count above out->capacity then sets a sticky
 *                     bit in the device status word, which the next sgnn_ctx_status reports as
 *                     SGNN_ERR_CAPACITY.  Otherwise the stream is synchronised, the entry
 *                     count is stored there, and SGNN_ERR_CAPACITY is returned if it exceeds
 *                     out->capacity (the required count is still reported).
 * The entry count must stay below 2^31 (checked on the device, reported by sgnn_ctx_status).
 */
int sgnn_induced_csr(sgnn_ctx *ctx, const sgnn_graph *graph, const int32_t *S, uint32_t B,
                     const uint64_t *bitmap, const uint32_t *rank, int norm_mode, int rescale,
                     sgnn_csr *out, uint64_t *nnz_host, sgnn_stream stream);

/*
 * One shard of the mini-batch matrix (Algorithm 2 as stated there, "per GPU"): the same B x B matrix
 * restricted to the rows of S inside the row range [R0, R1) and the columns of S inside the column
 * range [C0, C1), both in global vertex ids.  Row and column numbers stay in the [0, B) namespace of the
 * whole sample (the shards of a grid tile the full matrix); rows outside the row range are empty.
 * Weights from the full-graph degrees (or g->val), as with norm_mode 0.  Everything else as
 * sgnn_induced_csr.  S depends on (seed, step, N) only, so every owner of a shard derives it alone.
 */
int sgnn_induced_csr_range(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B,
                           const uint64_t *bitmap, const uint32_t *rank, int rescale, int64_t R0, int64_t R1,
                           int64_t C0, int64_t C1, sgnn_csr *out, uint64_t *nnz_host, sgnn_stream stream);

/*
 * out = A^T as CSR with ascending columns (Algorithm 2's last phase assembles the matrix and its
 * transpose; Sec. III-C multiplies by the transpose).  Needed for shards with different row and column
 * ranges and for directed graphs; the full matrix of an undirected graph is its own transpose.
 *   out   cols x rows (set out->rows / out->cols accordingly), capacity >= A's, plan optional (filled)
 * The result does not depend on timing (bit-reproducible).
 */
int sgnn_csr_transpose(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_csr *out, sgnn_stream stream);


/*
 * Dense row-major matrix.  row_index (may be NULL) makes logical row i the physical row
 * row_index[i] of ptr; it is honoured only where a parameter says so.
 */
typedef struct {
    void *ptr;
    int dtype; /* SGNN_F32; SGNN_BF16 (bfloat16 storage, round to nearest even, ld in elements) only where a call
                * says so: the operand and the result of a sparse product (X and out of sgnn_spmm) and, with
                * SGNN_BF16_MFMA, the activations of a layer (H, T, Y of sgnn_gcn_fwd; T, Y, H_in of sgnn_gcn_bwd) and the
                * gradient handed from one layer to the one below (dH, dY of sgnn_gcn_bwd).  Weights, their gradients,
                * the logits handed to the loss and the loss gradient are always fp32. */
    int64_t rows, cols, ld;
    const int32_t *row_index;
} sgnn_mat;

/*
 * Eq. 26: out[i, :] = X[S[i], :] for i < B (fp32, d columns), and labels_out[i] = labels[S[i]]
 * when labels != NULL.  X == NULL slices the labels only (the feature slice can instead be fused
 * into the first layer through sgnn_mat.row_index).
 */
int sgnn_gather_rows(sgnn_ctx *ctx, const float *X, int64_t d, int64_t ldx, const int32_t *S,
                     uint32_t B, float *out, int64_t ldo, const int32_t *labels,
                     int32_t *labels_out, sgnn_stream stream);

/*
 * One GCN layer forward (Eqs. 5-6, 8): T = A H, Y = act(T W + bias).
 *   A     B x B mini-batch CSR (entries beyond A->capacity are never read)
 *   H     B x d_in fp32 or bfloat16; H->row_index is honoured (fuses the slice of Eq. 26 into layer 1:
 *         pass the full feature matrix with row_index = S)
 *   W     d_in x d_out fp32;  bias fp32[d_out] or NULL
 *   flags SGNN_RELU, SGNN_BF16_MFMA
 *   Y     out B x d_out fp32 or bfloat16
 *   T     out B x d_in fp32 or bfloat16, the aggregate, kept by the caller for the backward pass; unused
 *         (may be NULL) with SGNN_XFORM_FIRST, where the backward pass needs the layer input H instead
 * bfloat16 storage of T, of Y, or of the input of a transform-first layer needs SGNN_BF16_MFMA (else
 * SGNN_ERR_UNSUPPORTED): the dense product rounds its operands to bfloat16 anyway, so a bfloat16 T holds
 * exactly what the product would have read, and only Y - rounded once, after the activation - carries a
 * new rounding.  A transform-first layer whose input is bfloat16 keeps its intermediate product H W in
 * bfloat16 as well.  The tall-operand kernel (B >= 4096, widths up to 256) reads and writes the 16-bit
 * storage itself; other shapes go through fp32 copies in the context scratch.
 */
int sgnn_gcn_fwd(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *H, const sgnn_mat *W,
                 const float *bias, int flags, sgnn_mat *Y, sgnn_mat *T, sgnn_stream stream);

/*
 * One GCN layer backward (Sec. III-C): dZ = dY where Y > 0 (all of dY without SGNN_RELU or with SGNN_DY_MASKED),
 * dbias = column sums of dZ, dW = T^T dZ, dT = dZ W^T, dH = A_T dT.
 *   A_T   the transpose of the forward matrix as CSR (the same object when it is symmetric)
 *   T, W, Y   as in the forward call (T and Y in the storage they were written in; with T stored as bfloat16
 *             the internal dT - and dP below - is stored as bfloat16 too, rounded to nearest even once);
 *             dY  B x d_out fp32, or
 *             bfloat16 when it already carries the layer's mask (SGNN_DY_MASKED, or no SGNN_RELU); dbias is then
 *             available along with the dW of an aggregate-first layer only (the sum of the stored, rounded
 *             values); anything else with a bfloat16 dY is SGNN_ERR_UNSUPPORTED
 *             with SGNN_XFORM_FIRST (same flag as in the forward call) T is the layer INPUT H
 *             (B x d_in, row_index honoured) and the products are dP = A_T dZ, dW = H^T dP,
 *             dH = dP W^T
 *   dH    out B x d_in fp32 or bfloat16 (rounded to nearest even when stored: what the dense products of the
 *         layer below would round it to anyway), or NULL to skip it (first layer)
 *   H_in  optional (NULL = none; needs dH): the layer's input activations, B x d_in fp32 or bfloat16, the
 *         output of the ReLU of the layer below.  dH is then returned already multiplied by [H_in > 0],
 *         i.e. with that layer's ReLU backward fused into the product that writes dH; call that
 *         layer's backward with SGNN_DY_MASKED so that it skips its own masking pass.
 *   dW    out fp32[d_in x d_out] row-major, overwritten, or NULL to skip it (a caller that computes
 *         T^T dZ itself, e.g. on another stream: with SGNN_DY_MASKED or without SGNN_RELU dZ is dY);
 *         dbias out fp32[d_out] or NULL
 * The reduction over the B rows in dW and dbias uses a fixed split and a fixed summation order:
 * results are bit-reproducible from run to run.
 */
int sgnn_gcn_bwd(sgnn_ctx *ctx, const sgnn_csr *A_T, const sgnn_mat *T, const sgnn_mat *W,
                 const sgnn_mat *Y, const sgnn_mat *dY, int flags, sgnn_mat *dH, const sgnn_mat *H_in,
                 float *dW, float *dbias, sgnn_stream stream);

/*
 * The full graph as a sparse matrix for the full-graph evaluation forward (the paper's evaluation
 * rounds run the model on all N vertices): int32 row offsets and the weights of Eq. 3,
 * a_vu = 1 / sqrt(deg(v) deg(u)) (g->val verbatim when given), no 1/p rescale.
 *   rowptr32  out device int32[N + 1], or NULL: the offsets are not copied and the caller uses the
 *             graph's own (sgnn_csr.rowptr_is_i64 = g->rowptr_is_i64) - the only way with 2^31 - 1 or more
 *             stored entries, where a non-NULL rowptr32 is SGNN_ERR_UNSUPPORTED
 *   val       out device fp32[E]
 * Together with g->colidx they form an sgnn_csr {rows = cols = N, capacity = E} for sgnn_gcn_fwd /
 * sgnn_spmm.
 */
int sgnn_graph_normalized_csr(sgnn_ctx *ctx, const sgnn_graph *g, int32_t *rowptr32, float *val,
                              sgnn_stream stream);

/*
 * The element-wise tail of the paper's GNN layer as one kernel (Sec. III-B Eqs. 7-10; the fusion of
 * Sec. V "Kernel Fusion"):   Y = dropout(relu(rmsnorm(Z))) + R
 *   rmsnorm(z)_j = gamma_j z_j / sqrt(mean_j z_j^2 + eps)        (Eq. 7; the paper's RMS has no eps: eps = 0)
 *   dropout: element e = i * d + j of layer `layer` at step `step` is kept iff word e % 4 of
 *            Philox4x32-10 with key = (drop_seed lo, hi), counter = (e / 4 lo, e / 4 hi, step mod 2^32,
 *            2^31 + layer) is >= floor(drop_q * 2^32); kept values are multiplied by 1 / (1 - drop_q)
 *   Z       B x d fp32, the convolution output X_conv;  gamma fp32[d] or NULL (ones)
 *   R       optional B x d fp32 residual input X_{h,l-1} (Eq. 10), NULL = none
 *   drop_q  drop probability, 0 <= q < 1 (0 = no dropout)
 *   Y       out B x d fp32 (must not alias Z);  inv_rms out fp32[B] = 1 / sqrt(mean z^2 + eps), kept
 *           by the caller for sgnn_tail_bwd (NULL to skip)
 * Rows of up to 2048 values (512 when d, the leading dimensions or the pointers are not multiples of 4 /
 * 16 bytes); wider rows are SGNN_ERR_UNSUPPORTED.
 */
int sgnn_tail_fwd(sgnn_ctx *ctx, const sgnn_mat *Z, const float *gamma, float eps, const sgnn_mat *R,
                  float drop_q, uint64_t drop_seed, uint32_t layer, uint64_t step, sgnn_mat *Y,
                  float *inv_rms, sgnn_stream stream);

/*
 * The dense transform and the tail in one call: Z = T W (Eq. 6), Y = dropout(relu(rmsnorm(Z))) + R
 * (Eqs. 7-10).  By default the product and sgnn_tail_fwd run one after the other.  With SGNN_FUSE_TAIL,
 * SGNN_BF16_MFMA and a tall T (at least 4096 rows, at most 256 columns in T and W, W's width a multiple
 * of 4, T's rows 16-byte aligned) both run in ONE kernel - the tail in the epilogue of the product, whose
 * wavefronts own whole rows - so Z is written for the backward pass but never read back.  Same result up
 * to the summation order of the mean square.  On MI355X the fused form is the slower one (its epilogue
 * has no registers left to hide the loads of R): it is kept as an option, not as the default.
 *   T  B x d_in fp32;  W  d_in x d fp32;  flags  SGNN_BF16_MFMA, SGNN_FUSE_TAIL;  the rest as in sgnn_tail_fwd
 *   Z  out B x d fp32 (kept for sgnn_tail_bwd);  Y  out B x d fp32
 */
int sgnn_gemm_tail_fwd(sgnn_ctx *ctx, const sgnn_mat *T, const sgnn_mat *W, const float *gamma, float eps,
                       const sgnn_mat *R, float drop_q, uint64_t drop_seed, uint32_t layer, uint64_t step,
                       int flags, sgnn_mat *Z, sgnn_mat *Y, float *inv_rms, sgnn_stream stream);

/*
 * Backward of the main branch of that tail (Sec. III-C: dropout mask, ReLU mask, RMSNorm backward).
 * The dropout mask is recomputed from (drop_seed, layer, step), never stored.
 *   Z, inv_rms, gamma   as in / from the forward call;  dY  B x d fp32, the gradient of Y
 *   dZ      out B x d fp32, the gradient of X_conv (must not alias dY)
 *   dgamma  out fp32[d] or NULL;  dbias out fp32[d] or NULL: column sums of dZ (the gradient of a
 *           bias added in front of the tail).  Fixed summation order: bit-reproducible.
 * The gradient of the skip path of Eq. 10 is dY itself and is not formed here.
 */
int sgnn_tail_bwd(sgnn_ctx *ctx, const sgnn_mat *Z, const float *inv_rms, const float *gamma, float drop_q,
                  uint64_t drop_seed, uint32_t layer, uint64_t step, const sgnn_mat *dY, sgnn_mat *dZ,
                  float *dgamma, float *dbias, sgnn_stream stream);

/*
 * Mean softmax cross-entropy over B rows of C logits (Sec. III-B, single-label loss) and its
 * gradient dO = (softmax(O) - onehot(label)) / B.  loss_dev: device float[1] or NULL.
 * dO: device B x C with leading dimension lddo (elements), fp32 (dO_dtype = SGNN_F32) or bfloat16 (SGNN_BF16:
 * every entry rounded to nearest even as it is stored, and dO_colsum adds the stored values), or NULL.
 * dO_colsum: device float[C] or NULL (needs dO): the column sums of dO, i.e. the bias gradient of a
 * last layer without activation (Sec. III-C), from the same pass and in a fixed summation order.
 */
int sgnn_softmax_xent(sgnn_ctx *ctx, const float *O, int64_t ldo, const int32_t *labels, uint32_t B,
                      uint32_t C, float *loss_dev, void *dO, int dO_dtype, int64_t lddo, float *dO_colsum,
                      sgnn_stream stream);

/*
 * The last layer of a transform-first stack and its loss in one pass (Sec. V "Kernel Fusion": the logits are
 * not read back from memory): O = A X + bias (Eq. 5 with the layer's H W as X, Sec. III-B), the mean softmax
 * cross-entropy of O's rows against `labels` and its gradient dO = (softmax(O) - onehot(label)) / A.rows, as
 * sgnn_spmm followed by sgnn_softmax_xent would give them (same arithmetic per row; the sums over the rows are
 * taken in another, equally fixed order: bit-reproducible from run to run).
 *   X       A.cols x C, fp32 or bfloat16, no row_index;  bias  device fp32[C] or NULL;  labels  device int32[A.rows]
 *   O       out A.rows x C fp32, or NULL when the caller does not keep the logits
 *   loss_dev, dO, dO_dtype, lddo, dO_colsum   as in sgnn_softmax_xent (dO may be NULL)
 * Up to 512 classes run in one kernel; wider or oddly aligned operands take the two kernels one after the other
 * (with the logits in the context scratch when O is NULL).
 */
int sgnn_spmm_xent(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *X, const float *bias, const int32_t *labels,
                   sgnn_mat *O, float *loss_dev, void *dO, int dO_dtype, int64_t lddo, float *dO_colsum,
                   sgnn_stream stream);

/*
 * Mean binary cross-entropy on logits over the B x C entries, the paper's loss for multi-label tasks
 * (Sec. III-B), and its gradient dO = (logistic(O) - Y) / (B C).  Y: fp32 targets in [0, 1], B x C.
 * loss_dev: device float[1] or NULL; dO may be NULL.  Fixed summation order.
 */
int sgnn_sigmoid_bce(sgnn_ctx *ctx, const float *O, int64_t ldo, const float *Y, int64_t ldy, uint32_t B,
                     uint32_t C, float *loss_dev, float *dO, int64_t lddo, sgnn_stream stream);

/*
 * out[j] = sum over the rows of X[:, j] (fixed summation order): the bias gradient of Sec. III-C as an
 * operator of its own, for callers that take it off the main stream.  X rows x cols fp32, out fp32[cols].
 */
int sgnn_colsum(sgnn_ctx *ctx, const sgnn_mat *X, float *out, sgnn_stream stream);

/*
 * Parameter update ("update parameters", Alg. 1 line 7; the paper names no optimizer).
 * sgnn_sgd_step:  w <- w - lr * (g + weight_decay * w)
 * sgnn_adam_step: Adam (Kingma & Ba, ICLR 2015, Algorithm 1) with bias correction:
 *     m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2;
 *     w <- w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = 1, 2, ... the step number
 * w, g, m, v: device fp32[n], updated in place (g is read only).  The scalars are host doubles; the factors
 * derived from them (1 - b1, 1 / (1 - b1^t), ...) are evaluated in double precision and rounded to fp32 once.
 */
int sgnn_sgd_step(sgnn_ctx *ctx, float *w, const float *g, int64_t n, double lr, double weight_decay,
                  sgnn_stream stream);
int sgnn_adam_step(sgnn_ctx *ctx, float *w, const float *g, float *m, float *v, int64_t n, double lr,
                   double beta1, double beta2, double eps, int64_t t, sgnn_stream stream);

/* Plain operators, exported for tests and for callers that build their own layer. */

/*
 * out = A X (+ add): A rows x cols CSR, X cols x d fp32 or bfloat16 (X->row_index honoured), out rows x d fp32
 * or bfloat16 (accumulated in fp32, rounded to nearest even when stored);
 * add: optional rows x d fp32 matrix added to the product (NULL = none; must not be `out`) - the skip path of a residual layer merged into the transposed product of Sec. III-C.
 */
int sgnn_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *X, const sgnn_mat *add, sgnn_mat *out,
              sgnn_stream stream);

/*
 * C = act(op(A) op(B) + bias): row-major, M x N result, reduction length K.  bias is fp32; A, B, C and the
 * mask are fp32 (SGNN_F32) or - with SGNN_BF16_MFMA - stored as bfloat16 (SGNN_BF16, leading dimension in elements).
 *   trans_a 0: A is M x K;  1: A is K x M (used as its transpose)
 *   trans_b 0: B is K x N;  1: B is N x K (used as its transpose)
 *   flags   SGNN_RELU, SGNN_BF16_MFMA;  bias fp32[N] or NULL
 *   mask    optional M x N matrix (leading dimension ldm), read only: C is set to zero wherever
 *           mask <= 0 - the ReLU backward of the layer below (Sec. III-C) applied to an input
 *           gradient as it is written, with that layer's output as the mask.  NULL = none.
 *   b_colsum  optional, with trans_a = 1 and trans_b = 0 only: out fp32[N], the column sums of B over its
 *             K rows - the bias gradient next to the weight gradient T^T dZ (Sec. III-C), taken from
 *             the operand the product reads anyway.  NULL = not wanted.
 */
int sgnn_gemm(sgnn_ctx *ctx, int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
              const void *A, int a_dtype, int64_t lda, const void *B, int b_dtype, int64_t ldb,
              const float *bias, int flags, void *C, int c_dtype, int64_t ldc, const void *mask, int mask_dtype,
              int64_t ldm, float *b_colsum, sgnn_stream stream);

/*
 * dst[0..n) = src[0..n) (fp32, 16-byte aligned, n a multiple of 4): a plain streaming copy of known
 * size, the reference point against which hardware traffic counters of the other kernels are
 * scaled in the benchmark.
 */
int sgnn_copy_f32(sgnn_ctx *ctx, const float *src, float *dst, int64_t n, sgnn_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SGNN_H */
