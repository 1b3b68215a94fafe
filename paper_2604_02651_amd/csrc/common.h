// Internal declarations shared by the HIP translation units of libsgnn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "sgnn.h"

#define SGNN_WAVE 64

// One timed kernel launch of the optional profiling mode (sgnn_ctx_profile).
struct sgnn_prof_rec {
    const char *name;   // kernel name (string literal)
    char tag[56];       // shape of the launch, e.g. "NN 32768x256x256 f32"
    hipEvent_t e0, e1;
};

struct sgnn_ctx {
    int device;
    int prof_on;                 // bracket every launch with HIP events on its stream
    sgnn_prof_rec *prof;         // event pool, grown on demand, reused
    size_t prof_n, prof_cap;
    const char *cur_tag;         // tag attached to the launches that follow
    char err[512];
    uint8_t *ws;        // device scratch, carved afresh by every call
    uint8_t *persist;   // small device area that keeps its contents between calls
    size_t ws_bytes;
    uint32_t *status;   // device uint32[4]: [0] sticky error bits set by kernels
    uint64_t res_N, res_E;
    uint32_t res_B, res_d;
};

// Offset in the persistent area of the SpMM chunk counter (uint32, zero between calls).
#define SGNN_PERSIST_BYTES 32768
#define SGNN_PERSIST_SPMM_OFF 12288

// status bits
#define SGNN_ST_CAND_OVERFLOW 1u
#define SGNN_ST_NNZ_OVERFLOW 2u
#define SGNN_ST_CAPACITY_OVERFLOW 4u

int sgnn_fail(sgnn_ctx *ctx, int code, const char *fmt, ...);

#define SGNN_HIP(ctx, call)                                                                     \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return sgnn_fail((ctx), SGNN_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

#define SGNN_LAUNCH_CHECK(ctx, name)                                                            \
    do {                                                                                        \
        hipError_t e_ = hipGetLastError();                                                      \
        if (e_ != hipSuccess)                                                                   \
            return sgnn_fail((ctx), SGNN_ERR_HIP, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

void sgnn_prof_begin(sgnn_ctx *ctx, hipStream_t st, const char *name, const char *tag);
void sgnn_prof_end(sgnn_ctx *ctx, hipStream_t st);

// Launch + error check; in profiling mode the launch is bracketed by two events on its stream.
#define SGNN_TAG (ctx->cur_tag ? ctx->cur_tag : "")
#define SGNN_LAUNCH(ctx, st, name, tag, ...)                                                    \
    do {                                                                                        \
        if ((ctx)->prof_on) sgnn_prof_begin((ctx), (st), name, tag);                            \
        hipLaunchKernelGGL(__VA_ARGS__);                                                        \
        if ((ctx)->prof_on) sgnn_prof_end((ctx), (st));                                         \
        SGNN_LAUNCH_CHECK(ctx, name);                                                           \
    } while (0)

// Bump allocator over the context scratch, reset at the start of every API call.
struct ws_alloc {
    uint8_t *base;
    size_t cap, off;
    bool ok;
    explicit ws_alloc(sgnn_ctx *c) : base(c->ws), cap(c->ws_bytes), off(0), ok(true) {}
    template <class T> T *get(size_t n) {
        size_t bytes = (n * sizeof(T) + 255) & ~size_t(255);
        if (!base || off + bytes > cap) { ok = false; off += bytes; return nullptr; }
        T *p = reinterpret_cast<T *>(base + off);
        off += bytes;
        return p;
    }
};

static inline unsigned cdiv(uint64_t a, uint64_t b) { return (unsigned)((a + b - 1) / b); }

// ---- scan.hip ---------------------------------------------------------------------------------
// Exclusive prefix sum of n uint32 (n known on the host), 64-bit result: out[i] = sum_{k<i} in[k]
// for i <= n (out has n+1 entries).  tmp: ceil(n/2048)+1 uint64.
size_t sgnn_scan_tmp_elems(uint64_t n);
int sgnn_scan_u32_to_u64(sgnn_ctx *ctx, const uint32_t *in, uint64_t *out, uint64_t n, uint64_t *tmp,
                         hipStream_t st);
// Same with a 32-bit result and the element count read from device memory (*n_dev <= n_max).
int sgnn_scan_u32_devn(sgnn_ctx *ctx, const uint32_t *in, uint32_t *out, const uint64_t *n_dev,
                       uint64_t n_max, uint32_t *tmp, hipStream_t st);

// ---- launchers ----------------------------------------------------------------------------------
int sgnn_launch_sampler(sgnn_ctx *ctx, uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S,
                        uint64_t *bitmap, uint32_t *rank, hipStream_t st);
int sgnn_launch_induced(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B,
                        const uint64_t *bitmap, const uint32_t *rank, int norm_mode, int rescale, int64_t R0,
                        int64_t R1, int64_t C0, int64_t C1, sgnn_csr *out, int sticky_capacity, hipStream_t st);
int sgnn_launch_csr_transpose(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_csr *out, ws_alloc *ws, hipStream_t st);
size_t sgnn_transpose_ws_bytes(uint64_t max_entries, uint32_t B);
int sgnn_launch_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, const int32_t *row_index,
                     int64_t d, float *out, int64_t ldo, const float *bias, int relu, const float *mask, int64_t ldm,
                     const float *add, int64_t ldadd, ws_alloc *ws, hipStream_t st);
int sgnn_launch_spmm_x(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, const int32_t *row_index, int64_t d,
                       void *out, int out_bf16, int64_t ldo, const float *bias, int relu, const void *mask, int mask_bf16,
                       int64_t ldm, const float *add, int64_t ldadd, ws_alloc *ws, hipStream_t st);
int sgnn_launch_spmm_plan(sgnn_ctx *ctx, const sgnn_csr *A, hipStream_t st);   // fills A->plan when it is attached
// a_row_index (may be NULL): physical row of A for every logical row (M x K operand: rows of the
// result; K x M operand used transposed: reduction index)
int sgnn_launch_gemm(sgnn_ctx *ctx, int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A,
                     int64_t lda, const int32_t *a_row_index, const float *B, int64_t ldb, const float *bias,
                     int flags, float *C, int64_t ldc, const float *mask, int64_t ldm, float *b_colsum, ws_alloc *ws,
                     hipStream_t st);
// The same with A, B, C and the mask optionally stored as bfloat16 (a_bf16 / b_bf16 / c_bf16 / m_bf16; leading dimensions in
// elements; needs SGNN_BF16_MFMA): read and written as stored by the kernels that can, converted through scratch for the others.
int sgnn_launch_gemm_x(sgnn_ctx *ctx, int ta, int tb, int64_t M, int64_t N, int64_t K, const void *A, int a_bf16, int64_t lda,
                       const int32_t *a_row_index, const void *B, int b_bf16, int64_t ldb, const float *bias, int flags, void *C,
                       int c_bf16, int64_t ldc, const void *mask, int m_bf16, int64_t ldm, float *b_colsum, ws_alloc *ws,
                       hipStream_t st);
int sgnn_launch_splitk_reduce(sgnn_ctx *ctx, const float *partial, int splits, int64_t M, int64_t N, float *C, int64_t ldc,
                              const float *cs_partial, float *cs_out, hipStream_t st);
// A^T B, both operands bfloat16, result up to 256 x 256, long reduction: SGNN_ERR_UNSUPPORTED (nothing launched) outside its range
int sgnn_launch_gemm_tn_stream(sgnn_ctx *ctx, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               float *C, int64_t ldc, float *b_colsum, ws_alloc *ws, hipStream_t st);
int sgnn_launch_gemm_tail(sgnn_ctx *ctx, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *W,
                          int64_t ldw, const float *gamma, float eps, const float *R, int64_t ldr, float q, uint64_t seed,
                          uint32_t layer, uint64_t step, float *Z, int64_t ldz, float *Y, int64_t ldy, float *inv_rms,
                          hipStream_t st);
int sgnn_launch_relu_bwd_bias(sgnn_ctx *ctx, const void *Y, int y_bf16, int64_t ldy, const float *dY, int64_t lddy,
                              int relu, int64_t rows, int64_t cols, float *dZ, int64_t lddz, float *dbias,
                              ws_alloc *ws, hipStream_t st);
int sgnn_launch_gather(sgnn_ctx *ctx, const float *X, int64_t d, int64_t ldx, const int32_t *S, uint32_t B,
                       float *out, int64_t ldo, const int32_t *labels, int32_t *labels_out, hipStream_t st);
int sgnn_launch_tail_fwd(sgnn_ctx *ctx, int64_t rows, int64_t d, const float *Z, int64_t ldz, const float *gamma, float eps,
                         const float *R, int64_t ldr, float q, uint64_t seed, uint32_t layer, uint64_t step, float *Y,
                         int64_t ldy, float *inv_rms, hipStream_t st);
int sgnn_launch_tail_bwd(sgnn_ctx *ctx, int64_t rows, int64_t d, const float *Z, int64_t ldz, const float *inv_rms,
                         const float *gamma, float q, uint64_t seed, uint32_t layer, uint64_t step, const float *dY,
                         int64_t lddy, float *dZ, int64_t lddz, float *dgamma, float *dbias, ws_alloc *ws, hipStream_t st);
int sgnn_launch_bce(sgnn_ctx *ctx, const float *O, int64_t ldo, const float *Y, int64_t ldy, int64_t B, int64_t C, float *loss,
                    float *dO, int64_t lddo, ws_alloc *ws, hipStream_t st);
int sgnn_launch_sgd(sgnn_ctx *ctx, float *w, const float *g, int64_t n, double lr, double wd, hipStream_t st);
int sgnn_launch_adam(sgnn_ctx *ctx, float *w, const float *g, float *m, float *v, int64_t n, double lr, double b1, double b2,
                     double eps, int64_t t, hipStream_t st);
int sgnn_launch_graph_normalize(sgnn_ctx *ctx, const sgnn_graph *g, int32_t *rowptr32, float *val, hipStream_t st);
int sgnn_launch_copy(sgnn_ctx *ctx, const float *src, float *dst, int64_t n, hipStream_t st);
// mean loss and column sums from the per-workgroup partial sums of a loss kernel (n rows of partial sums)
// fix (may be null): fix_slots rows of cols + 1 fixed-point sums (64-bit integers; column `cols` holds loss terms) that are
// added in as well, scaled by cs_unit / loss_unit
int sgnn_launch_xent_final(sgnn_ctx *ctx, const float *partial, int n, float inv_rows, float *loss, const float *cs_partial, int cols,
                           float *colsum, const unsigned long long *fix, int fix_slots, double cs_unit, double loss_unit, hipStream_t st);
// O = A X + bias, mean softmax cross-entropy of O against labels and its gradient, in one kernel (SGNN_ERR_UNSUPPORTED,
// nothing launched, for shapes the fused kernels do not take); out may be null (logits not kept)
int sgnn_launch_spmm_xent(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, int64_t d, const float *bias,
                          const int32_t *labels, float *out, int64_t ldo, float *loss, void *dO, int dO_bf16, int64_t lddo,
                          float *dO_colsum, ws_alloc *ws, hipStream_t st);
int sgnn_launch_xent(sgnn_ctx *ctx, const float *O, int64_t ldo, const int32_t *labels, uint32_t B, uint32_t C,
                     float *loss, void *dO, int do_bf16, int64_t lddo, float *dO_colsum, ws_alloc *ws, hipStream_t st);
