// C ABI of libsgnn: argument validation, context and scratch management, and the composition of the
// kernels into the calls declared in sgnn.h.
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "common.h"

size_t sgnn_sampler_persist_bytes();
int sgnn_static_scratch_init(int device);
size_t sgnn_sampler_ws_bytes(uint64_t N);
size_t sgnn_induced_ws_bytes(uint64_t N, uint64_t E, uint32_t B);
size_t sgnn_gemm_ws_bytes(uint32_t d_max);
size_t sgnn_spmm_ws_bytes(uint64_t max_entries, uint32_t B, uint32_t d_max);

// message of the last failing call that had no context (the allocation-free entry point), per thread
static thread_local char g_err_no_ctx[512] = "";

int sgnn_fail(sgnn_ctx *ctx, int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    if (ctx) vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    else vsnprintf(g_err_no_ctx, sizeof(g_err_no_ctx), fmt, ap);
    va_end(ap);
    return code;
}

void sgnn_prof_begin(sgnn_ctx *ctx, hipStream_t st, const char *name, const char *tag)
{
    if (ctx->prof_n == ctx->prof_cap) {
        const size_t cap = ctx->prof_cap ? 2 * ctx->prof_cap : 1024;
        sgnn_prof_rec *p = static_cast<sgnn_prof_rec *>(realloc(ctx->prof, cap * sizeof(sgnn_prof_rec)));
        if (!p) { ctx->prof_on = 0; return; }
        for (size_t i = ctx->prof_cap; i < cap; ++i) {
            if (hipEventCreate(&p[i].e0) != hipSuccess || hipEventCreate(&p[i].e1) != hipSuccess) {
                ctx->prof = p; ctx->prof_cap = i; ctx->prof_on = 0;
                return;
            }
        }
        ctx->prof = p;
        ctx->prof_cap = cap;
    }
    sgnn_prof_rec &r = ctx->prof[ctx->prof_n];
    r.name = name;
    snprintf(r.tag, sizeof(r.tag), "%s", tag ? tag : "");
    hipEventRecord(r.e0, st);
}

void sgnn_prof_end(sgnn_ctx *ctx, hipStream_t st)
{
    if (!ctx->prof_on || ctx->prof_n >= ctx->prof_cap) return;
    hipEventRecord(ctx->prof[ctx->prof_n].e1, st);
    ++ctx->prof_n;
}

namespace {

constexpr size_t PERSIST_BYTES = SGNN_PERSIST_BYTES;

int bind_device(sgnn_ctx *ctx)
{
    SGNN_HIP(ctx, hipSetDevice(ctx->device));
    return SGNN_OK;
}

bool mat_ok(const sgnn_mat *m) { return m && m->ptr && m->dtype == SGNN_F32 && m->rows >= 0 && m->cols >= 0 && m->ld >= m->cols; }
// the operand of a sparse product may also be stored as bfloat16
bool mat_ok_in(const sgnn_mat *m) { return m && m->ptr && (m->dtype == SGNN_F32 || m->dtype == SGNN_BF16) && m->rows >= 0 && m->cols >= 0 && m->ld >= m->cols; }

bool csr_ok(const sgnn_csr *c) { return c && c->rowptr && (c->capacity == 0 || (c->colidx && c->val)) && (c->rowptr_is_i64 == 0 || c->rowptr_is_i64 == 1); }

} // namespace

static inline int64_t pad4(int64_t d) { return (d + 3) & ~int64_t(3); }
// leading dimension of a scratch matrix: rows start on 64-byte boundaries (16 fp32 or 32 bfloat16 elements)
static inline int64_t pad_ld(int64_t d, bool is16) { return is16 ? ((d + 31) & ~int64_t(31)) : ((d + 15) & ~int64_t(15)); }

extern "C" {

int sgnn_ctx_create(sgnn_ctx **out, int device)
{
    if (!out) return SGNN_ERR_INVALID_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return SGNN_ERR_HIP;
    sgnn_ctx *ctx = new (std::nothrow) sgnn_ctx();
    if (!ctx) return SGNN_ERR_HIP;
    memset(ctx, 0, sizeof(*ctx));
    ctx->device = device;
    if (hipSetDevice(device) != hipSuccess || hipMalloc(&ctx->persist, PERSIST_BYTES) != hipSuccess) {
        delete ctx;
        return SGNN_ERR_HIP;
    }
    if (hipMemset(ctx->persist, 0, PERSIST_BYTES) != hipSuccess) {
        hipFree(ctx->persist);
        delete ctx;
        return SGNN_ERR_HIP;
    }
    ctx->status = reinterpret_cast<uint32_t *>(ctx->persist + PERSIST_BYTES - 256);
    sgnn_static_scratch_init(device);     // address of the allocation-free sampler's scratch on this device (failure is
                                          // reported by that entry point itself)
    *out = ctx;
    return SGNN_OK;
}

int sgnn_ctx_destroy(sgnn_ctx *ctx)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    hipSetDevice(ctx->device);
    hipDeviceSynchronize();
    if (ctx->ws) hipFree(ctx->ws);
    if (ctx->persist) hipFree(ctx->persist);
    for (size_t i = 0; i < ctx->prof_cap; ++i) {
        hipEventDestroy(ctx->prof[i].e0);
        hipEventDestroy(ctx->prof[i].e1);
    }
    free(ctx->prof);
    delete ctx;
    return SGNN_OK;
}

const char *sgnn_last_error(const sgnn_ctx *ctx) { return ctx ? ctx->err : g_err_no_ctx; }

int sgnn_ctx_reserve(sgnn_ctx *ctx, uint64_t N, uint64_t E, uint32_t B, uint32_t d_max, uint64_t max_entries)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    int rc = bind_device(ctx);
    if (rc) return rc;
    size_t need = sgnn_sampler_ws_bytes(N);
    need = std::max(need, sgnn_induced_ws_bytes(N, E, B));
    // backward: dZ and dT (B x d_max each), split-K partials, column-sum partials
    // Products whose kernel does not handle bfloat16 storage itself (fewer than 4096 rows, or wider than 256) go through
    // widened / narrowed fp32 copies: three more B x d_max matrices for those shapes.
    const size_t copies = (B < 4096 || d_max > 256) ? 5 : 2;
    size_t layer = copies * B * (((size_t)d_max + 15) & ~size_t(15)) * 4 + 5 * 256 + sgnn_gemm_ws_bytes(d_max) + (size_t)1100 * d_max * 4 +
                   sgnn_spmm_ws_bytes(max_entries, B, d_max) + 16 * 256;
    need = std::max(need, layer);
    need = std::max(need, sgnn_transpose_ws_bytes(max_entries, B));
    need = std::max(need, (size_t)B / 64 * 4 + 4096);
    need += 4096;
    if (need > ctx->ws_bytes) {
        SGNN_HIP(ctx, hipDeviceSynchronize());
        if (ctx->ws) SGNN_HIP(ctx, hipFree(ctx->ws));
        ctx->ws = nullptr;
        ctx->ws_bytes = 0;
        SGNN_HIP(ctx, hipMalloc(&ctx->ws, need));
        ctx->ws_bytes = need;
    }
    ctx->res_N = N; ctx->res_E = E; ctx->res_B = B; ctx->res_d = d_max;
    return SGNN_OK;
}

int sgnn_ctx_status(sgnn_ctx *ctx, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t word = 0;
    SGNN_HIP(ctx, hipMemcpyAsync(&word, ctx->status, sizeof(word), hipMemcpyDeviceToHost, st));
    SGNN_HIP(ctx, hipStreamSynchronize(st));
    if (word) {
        SGNN_HIP(ctx, hipMemsetAsync(ctx->status, 0, sizeof(word), st));
        SGNN_HIP(ctx, hipStreamSynchronize(st));
        return sgnn_fail(ctx, (word & ~SGNN_ST_CAPACITY_OVERFLOW) ? SGNN_ERR_INTERNAL : SGNN_ERR_CAPACITY,
                         "device status 0x%x:%s%s%s", word,
                         (word & SGNN_ST_CAND_OVERFLOW) ? " sampler selection inconsistent" : "",
                         (word & SGNN_ST_NNZ_OVERFLOW) ? " induced entry count exceeds int32" : "",
                         (word & SGNN_ST_CAPACITY_OVERFLOW) ? " a mini-batch matrix had more entries than its capacity "
                                                              "(entries were dropped: the results of that step are invalid)" : "");
    }
    return SGNN_OK;
}

int sgnn_ctx_profile(sgnn_ctx *ctx, int enable)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    ctx->prof_on = enable ? 1 : 0;
    if (enable) ctx->prof_n = 0;
    return SGNN_OK;
}

int sgnn_ctx_profile_read(sgnn_ctx *ctx, char *buf, uint64_t buf_len)
{
    if (!ctx || !buf || buf_len == 0) return SGNN_ERR_INVALID_ARG;
    int rc = bind_device(ctx);
    if (rc) return rc;
    SGNN_HIP(ctx, hipDeviceSynchronize());
    // aggregate by (name, tag) in order of first appearance
    struct agg { const char *name; const char *tag; uint64_t calls; double ms; };
    agg *a = static_cast<agg *>(calloc(ctx->prof_n ? ctx->prof_n : 1, sizeof(agg)));
    if (!a) return sgnn_fail(ctx, SGNN_ERR_HIP, "sgnn_ctx_profile_read: out of host memory");
    size_t na = 0;
    for (size_t i = 0; i < ctx->prof_n; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->prof[i].e0, ctx->prof[i].e1) != hipSuccess) ms = 0.f;
        size_t j = 0;
        for (; j < na; ++j)
            if (a[j].name == ctx->prof[i].name && strcmp(a[j].tag, ctx->prof[i].tag) == 0) break;
        if (j == na) { a[na].name = ctx->prof[i].name; a[na].tag = ctx->prof[i].tag; ++na; }
        a[j].calls += 1;
        a[j].ms += ms;
    }
    uint64_t off = 0;
    buf[0] = 0;
    for (size_t j = 0; j < na; ++j) {
        int w = snprintf(buf + off, buf_len - off, "%s\t%s\t%llu\t%.6f\n", a[j].name, a[j].tag,
                         (unsigned long long)a[j].calls, a[j].ms);
        if (w < 0 || (uint64_t)w >= buf_len - off) { free(a); return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_ctx_profile_read: buffer too small"); }
        off += (uint64_t)w;
    }
    free(a);
    return SGNN_OK;
}

int sgnn_sample_uniform(sgnn_ctx *ctx, uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S,
                        uint64_t *bitmap, uint32_t *rank, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!S || !bitmap || !rank) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_sample_uniform: null output pointer");
    if (B == 0 || B > N) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_sample_uniform: need 1 <= B <= N (B=%u, N=%llu)", B, (unsigned long long)N);
    if (N >= (1ull << 31)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_sample_uniform: N must be below 2^31");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_sampler(ctx, N, B, seed, step, S, bitmap, rank, static_cast<hipStream_t>(stream));
}

static int induced_impl(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                        const uint32_t *rank, int norm_mode, int rescale, int64_t R0, int64_t R1, int64_t C0, int64_t C1,
                        sgnn_csr *out, uint64_t *nnz_host, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!g || !g->rowptr || !g->colidx || !S || !bitmap || !rank || !out || !out->rowptr)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: null pointer");
    if (out->capacity > 0 && (!out->colidx || !out->val))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: capacity > 0 but colidx/val is null");
    if (B == 0 || B > g->N) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: need 1 <= B <= N");
    if (g->N >= (1ull << 31)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: N must be below 2^31");
    if (!g->rowptr_is_i64 && g->E >= (1ull << 31))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: E >= 2^31 needs an int64 rowptr");
    if (norm_mode != 0 && norm_mode != 1) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: norm_mode must be 0 or 1");
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t *nnz_dev = out->nnz_dev;
    if (out->rowptr_is_i64) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: a mini-batch matrix has int32 row offsets");
    sgnn_csr o = *out;
    o.rows = o.cols = B;
    if (nnz_host && !nnz_dev) o.nnz_dev = ctx->status + 2;
    // with a host read-back the overflow is reported right here; without one through the sticky status word
    rc = sgnn_launch_induced(ctx, g, S, B, bitmap, rank, norm_mode, rescale, R0, R1, C0, C1, &o, nnz_host ? 0 : 1, st);
    if (rc) return rc;
    rc = sgnn_launch_spmm_plan(ctx, &o, st);
    if (rc) return rc;
    out->rows = out->cols = B;
    if (nnz_host) {
        uint32_t n = 0;
        SGNN_HIP(ctx, hipMemcpyAsync(&n, o.nnz_dev, sizeof(n), hipMemcpyDeviceToHost, st));
        SGNN_HIP(ctx, hipStreamSynchronize(st));
        *nnz_host = n;
        if (n > out->capacity)
            return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_induced_csr: %u entries do not fit capacity %llu", n,
                             (unsigned long long)out->capacity);
    }
    return SGNN_OK;
}

int sgnn_induced_csr(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                     const uint32_t *rank, int norm_mode, int rescale, sgnn_csr *out, uint64_t *nnz_host,
                     sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!g) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr: null pointer");
    return induced_impl(ctx, g, S, B, bitmap, rank, norm_mode, rescale, 0, (int64_t)g->N, 0, (int64_t)g->N, out, nnz_host, stream);
}

int sgnn_induced_csr_range(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                           const uint32_t *rank, int rescale, int64_t R0, int64_t R1, int64_t C0, int64_t C1, sgnn_csr *out,
                           uint64_t *nnz_host, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!g) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr_range: null pointer");
    if (R0 < 0 || R1 < R0 || (uint64_t)R1 > g->N || C0 < 0 || C1 < C0 || (uint64_t)C1 > g->N)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_induced_csr_range: need 0 <= R0 <= R1 <= N and 0 <= C0 <= C1 <= N");
    return induced_impl(ctx, g, S, B, bitmap, rank, 0, rescale, R0, R1, C0, C1, out, nnz_host, stream);
}

int sgnn_csr_transpose(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_csr *out, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!csr_ok(A) || !out || !out->rowptr || (out->capacity > 0 && (!out->colidx || !out->val)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_csr_transpose: bad argument");
    if (A->rowptr_is_i64 || out->rowptr_is_i64)
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_csr_transpose: int32 row offsets only");
    if (out->rows != A->cols || out->cols != A->rows || out->capacity < A->capacity)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_csr_transpose: out must be cols x rows with at least A's capacity");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    rc = sgnn_launch_csr_transpose(ctx, A, out, &ws, static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return sgnn_launch_spmm_plan(ctx, out, static_cast<hipStream_t>(stream));
}

int sgnn_csr_plan(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!A || !A->rowptr || !A->plan) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_csr_plan: null pointer");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_spmm_plan(ctx, A, static_cast<hipStream_t>(stream));
}

int sgnn_gather_rows(sgnn_ctx *ctx, const float *X, int64_t d, int64_t ldx, const int32_t *S, uint32_t B, float *out,
                     int64_t ldo, const int32_t *labels, int32_t *labels_out, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!S || (labels && !labels_out) || (!X && !labels))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gather_rows: bad argument");
    if (X && (!out || d <= 0 || ldx < d || ldo < d))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gather_rows: bad matrix argument");
    if (B == 0) return SGNN_OK;
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_gather(ctx, X, d, ldx, S, B, out, ldo, labels, labels_out, static_cast<hipStream_t>(stream));
}

int sgnn_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *X, const sgnn_mat *add, sgnn_mat *out, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!csr_ok(A) || !mat_ok_in(X) || !mat_ok_in(out)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_spmm: bad argument");
    if (out->rows != A->rows || out->cols != X->cols || (!X->row_index && X->rows != A->cols) ||
        (add && (!mat_ok(add) || add->row_index || add->rows != out->rows || add->cols != out->cols)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_spmm: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_spmm_x(ctx, A, X->ptr, X->dtype == SGNN_BF16, X->ld, X->row_index, X->cols, out->ptr,
                              out->dtype == SGNN_BF16, out->ld, nullptr, 0, nullptr, 0, 0,
                              add ? static_cast<const float *>(add->ptr) : nullptr, add ? add->ld : 0, &ws,
                              static_cast<hipStream_t>(stream));
}

int sgnn_spmm_xent(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *X, const float *bias, const int32_t *labels, sgnn_mat *O,
                   float *loss_dev, void *dO, int dO_dtype, int64_t lddo, float *dO_colsum, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!csr_ok(A) || !mat_ok_in(X) || X->row_index || !labels || (O && (!mat_ok(O) || O->row_index)) ||
        (dO && dO_dtype != SGNN_F32 && dO_dtype != SGNN_BF16) || (dO_colsum && !dO))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_spmm_xent: bad argument");
    const int64_t d = X->cols;
    if (X->rows != A->cols || (O && (O->rows != A->rows || O->cols != d)) || (dO && lddo < d) || A->rows == 0 || d == 0)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_spmm_xent: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ws_alloc ws(ctx);
    rc = sgnn_launch_spmm_xent(ctx, A, X->ptr, X->dtype == SGNN_BF16, X->ld, d, bias, labels, O ? static_cast<float *>(O->ptr) : nullptr,
                               O ? O->ld : 0, loss_dev, dO, dO_dtype == SGNN_BF16, lddo, dO_colsum, &ws, st);
    if (rc != SGNN_ERR_UNSUPPORTED) return rc;
    // a shape the fused kernels do not take: the product, then the loss kernel (logits in scratch if the caller keeps none)
    ws_alloc ws2(ctx);
    float *logits = O ? static_cast<float *>(O->ptr) : nullptr;
    int64_t ldl = O ? O->ld : pad_ld(d, false);
    if (!logits) {
        logits = ws2.get<float>((size_t)A->rows * ldl);
        if (!ws2.ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_spmm_xent: scratch too small: call sgnn_ctx_reserve");
    }
    rc = sgnn_launch_spmm_x(ctx, A, X->ptr, X->dtype == SGNN_BF16, X->ld, nullptr, d, logits, 0, ldl, bias, 0, nullptr, 0, 0, nullptr, 0,
                            &ws2, st);
    if (rc) return rc;
    return sgnn_launch_xent(ctx, logits, ldl, labels, A->rows, (uint32_t)d, loss_dev, dO, dO_dtype == SGNN_BF16 ? 1 : 0, lddo, dO_colsum,
                            &ws2, st);
}

int sgnn_gemm(sgnn_ctx *ctx, int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const void *A, int a_dtype, int64_t lda,
              const void *B, int b_dtype, int64_t ldb, const float *bias, int flags, void *C, int c_dtype, int64_t ldc,
              const void *mask, int mask_dtype, int64_t ldm, float *b_colsum, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!A || !B || !C || M < 0 || N < 0 || K < 0) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: bad argument");
    if ((a_dtype != SGNN_F32 && a_dtype != SGNN_BF16) || (b_dtype != SGNN_F32 && b_dtype != SGNN_BF16) ||
        (c_dtype != SGNN_F32 && c_dtype != SGNN_BF16) ||
        (mask && mask_dtype != SGNN_F32 && mask_dtype != SGNN_BF16))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: unknown storage type");
    if ((a_dtype == SGNN_BF16 || b_dtype == SGNN_BF16 || c_dtype == SGNN_BF16) && !(flags & SGNN_BF16_MFMA))
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gemm: bfloat16 storage of A, B or C goes with SGNN_BF16_MFMA only");
    if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N || (mask && ldm < N))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: leading dimension too small");
    if (M == 0 || N == 0) return SGNN_OK;
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_gemm_x(ctx, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, a_dtype == SGNN_BF16, lda, nullptr, B,
                              b_dtype == SGNN_BF16, ldb, bias, flags, C, c_dtype == SGNN_BF16, ldc, mask, mask && mask_dtype == SGNN_BF16, mask ? ldm : 0, b_colsum, &ws,
                              static_cast<hipStream_t>(stream));
}

int sgnn_gcn_fwd(sgnn_ctx *ctx, const sgnn_csr *A, const sgnn_mat *H, const sgnn_mat *W, const float *bias, int flags,
                 sgnn_mat *Y, sgnn_mat *T, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    const bool xform_first = (flags & SGNN_XFORM_FIRST) != 0;
    if (!csr_ok(A) || !mat_ok_in(H) || !mat_ok(W) || !mat_ok_in(Y) || (!xform_first && !mat_ok_in(T)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_fwd: bad argument");
    const bool h16 = H->dtype == SGNN_BF16, y16 = Y->dtype == SGNN_BF16, t16 = !xform_first && T->dtype == SGNN_BF16;
    if ((y16 || t16 || (xform_first && h16)) && !(flags & SGNN_BF16_MFMA))
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gcn_fwd: bfloat16 storage of T, Y or of the input of a transform-first "
                                                    "layer goes with SGNN_BF16_MFMA only (the dense product rounds to it anyway)");
    const int64_t Bn = A->rows, d_in = W->rows, d_out = W->cols;
    if (H->cols != d_in || Y->rows != Bn || Y->cols != d_out || (!H->row_index && H->rows != A->cols) ||
        (H->row_index && H->rows != A->cols) || W->row_index || Y->row_index ||
        (!xform_first && (T->rows != Bn || T->cols != d_in || T->row_index)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_fwd: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ws_alloc ws(ctx);
    const int gflags = flags & (SGNN_RELU | SGNN_BF16_MFMA);
    if (!xform_first) {
        // Eqs. 5-6 in the paper's order: aggregate, then transform with bias and activation fused
        rc = sgnn_launch_spmm_x(ctx, A, H->ptr, h16, H->ld, H->row_index, d_in, T->ptr, t16, T->ld, nullptr, 0, nullptr, 0, 0, nullptr,
                                0, &ws, st);
        if (rc) return rc;
        return sgnn_launch_gemm_x(ctx, 0, 0, Bn, d_out, d_in, T->ptr, t16, T->ld, nullptr, W->ptr, 0, W->ld, bias, gflags, Y->ptr, y16,
                                  Y->ld, nullptr, 0, 0, nullptr, &ws, st);
    }
    // A (H W): transform first (the aggregation then runs at width d_out), bias and activation
    // fused into the sparse product
    // The product H W lives in scratch; with the layer's input stored as bfloat16 it is stored as bfloat16 too (the
    // activations of such a stack are 16-bit between all of its kernels).
    const bool p16 = h16;
    const int64_t ldp = pad_ld(d_out, p16);
    float *P = ws.get<float>(p16 ? ((size_t)A->cols * ldp + 1) / 2 : (size_t)A->cols * ldp);
    if (!ws.ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gcn_fwd: scratch too small: call sgnn_ctx_reserve");
    rc = sgnn_launch_gemm_x(ctx, 0, 0, A->cols, d_out, d_in, H->ptr, h16, H->ld, H->row_index, W->ptr, 0, W->ld, nullptr,
                            flags & SGNN_BF16_MFMA, P, p16, ldp, nullptr, 0, 0, nullptr, &ws, st);
    if (rc) return rc;
    return sgnn_launch_spmm_x(ctx, A, P, p16, ldp, nullptr, d_out, Y->ptr, y16, Y->ld, bias, (flags & SGNN_RELU) ? 1 : 0, nullptr, 0, 0,
                              nullptr, 0, &ws, st);
}

int sgnn_gcn_bwd(sgnn_ctx *ctx, const sgnn_csr *A_T, const sgnn_mat *T, const sgnn_mat *W, const sgnn_mat *Y,
                 const sgnn_mat *dY, int flags, sgnn_mat *dH, const sgnn_mat *H_in, float *dW, float *dbias,
                 sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!csr_ok(A_T) || !mat_ok_in(T) || !mat_ok(W) || !mat_ok_in(dY) || (dH && !mat_ok_in(dH)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_bwd: bad argument");
    const bool t16 = T->dtype == SGNN_BF16, dy16 = dY->dtype == SGNN_BF16, dh16 = dH && dH->dtype == SGNN_BF16;
    if ((t16 || dy16 || dh16) && !(flags & SGNN_BF16_MFMA))
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gcn_bwd: bfloat16 storage of T, dY or dH goes with SGNN_BF16_MFMA only");
    const int relu = (flags & SGNN_RELU) ? 1 : 0;
    const bool xform_first = (flags & SGNN_XFORM_FIRST) != 0;
    const bool dy_masked = (flags & SGNN_DY_MASKED) != 0;   // the caller's dY already carries this layer's ReLU mask
    if (relu && !dy_masked && !mat_ok_in(Y)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_bwd: SGNN_RELU needs Y");
    if (H_in && (!dH || !mat_ok_in(H_in) || H_in->row_index))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_bwd: H_in needs dH and must be a plain matrix");
    const int64_t Bn = T->rows, d_in = W->rows, d_out = W->cols;
    if (T->cols != d_in || dY->rows != Bn || dY->cols != d_out ||
        (relu && !dy_masked && (Y->rows != Bn || Y->cols != d_out)) ||
        (H_in && (H_in->rows != dH->rows || H_in->cols != d_in)) ||
        (dH && (dH->rows != A_T->rows || dH->cols != d_in || A_T->cols != Bn)) || (!xform_first && T->row_index) ||
        (xform_first && (A_T->rows != Bn || A_T->cols != Bn)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gcn_bwd: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ws_alloc ws(ctx);
    const int mfma = flags & SGNN_BF16_MFMA;
    // dT = dZ W^T of an aggregate-first layer is written by a dense product and read by the transposed sparse product
    // only: with the layer's aggregate stored as bfloat16 it is stored as bfloat16 as well (the mirror image of the
    // forward pass, whose sparse product reads 16-bit activations), which halves the bytes of both kernels
    const bool dt16 = t16 && !xform_first;
    const int64_t ld_in = pad_ld(d_in, dt16);         // dT
    const int64_t ld_out = pad_ld(d_out, t16 && xform_first);     // dZ (fp32), or dP of a transform-first layer (16-bit with a 16-bit input)

    // element-wise backward: ReLU mask and bias gradient
    const void *dZ = dY->ptr;
    int dz16 = dy16 ? 1 : 0;
    int64_t lddz = dY->ld;
    const int mask_here = relu && !dy_masked;
    if (dy16 && (mask_here || (dbias && (!dW || xform_first))))
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gcn_bwd: a bfloat16 dY must carry the layer's ReLU mask already "
                                                    "(SGNN_DY_MASKED, or no SGNN_RELU), and dbias then comes with the dW of an "
                                                    "aggregate-first layer only");
    const void *hmask = H_in ? H_in->ptr : nullptr;
    const int64_t ldhm = H_in ? H_in->ld : 0;
    const int hm16 = (H_in && H_in->dtype == SGNN_BF16) ? 1 : 0;
    // the bias gradient rides on the weight-gradient product when both read the same dZ = dY
    const bool db_in_gemm = dbias && dW && !mask_here && !xform_first;
    if (mask_here || (dbias && !db_in_gemm)) {
        float *dZbuf = nullptr;
        if (mask_here) {
            dZbuf = ws.get<float>((size_t)Bn * ld_out);
            if (!ws.ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gcn_bwd: scratch too small: call sgnn_ctx_reserve");
        }
        rc = sgnn_launch_relu_bwd_bias(ctx, mask_here ? Y->ptr : nullptr, (mask_here && Y->dtype == SGNN_BF16) ? 1 : 0,
                                       mask_here ? Y->ld : 0, static_cast<const float *>(dY->ptr), dY->ld, mask_here, Bn, d_out, dZbuf,
                                       ld_out, dbias, &ws, st);
        if (rc) return rc;
        if (mask_here) { dZ = dZbuf; lddz = ld_out; dz16 = 0; }
    }
    if (!xform_first) {
        // dW = T^T dZ
        if (dW) {
            rc = sgnn_launch_gemm_x(ctx, 1, 0, d_in, d_out, Bn, T->ptr, t16, T->ld, nullptr, dZ, dz16, lddz, nullptr, mfma, dW, 0, d_out,
                                    nullptr, 0, 0, db_in_gemm ? dbias : nullptr, &ws, st);
            if (rc) return rc;
        }
        if (dH) {
            // dT = dZ W^T, dH = A^T dT
            float *dT = ws.get<float>(dt16 ? ((size_t)Bn * ld_in + 1) / 2 : (size_t)Bn * ld_in);
            if (!ws.ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gcn_bwd: scratch too small: call sgnn_ctx_reserve");
            rc = sgnn_launch_gemm_x(ctx, 0, 1, Bn, d_in, d_out, dZ, dz16, lddz, nullptr, W->ptr, 0, W->ld, nullptr, mfma, dT, dt16, ld_in,
                                    nullptr, 0, 0, nullptr, &ws, st);
            if (rc) return rc;
            rc = sgnn_launch_spmm_x(ctx, A_T, dT, dt16, ld_in, nullptr, d_in, dH->ptr, dh16, dH->ld, nullptr, 0, hmask, hm16, ldhm,
                                    nullptr, 0, &ws, st);
            if (rc) return rc;
        }
        return SGNN_OK;
    }
    // transform-first layer: dP = A^T dZ (width d_out), dW = H^T dP, dH = dP W^T; T is the layer input H.
    // dP is read by those two dense products only: with the layer's input stored as bfloat16 it is stored as bfloat16 as
    // well (the value the products would round it to), which halves its traffic and lets dW take the streaming kernel.
    const bool p16 = t16;
    float *dP = ws.get<float>(p16 ? ((size_t)Bn * ld_out + 1) / 2 : (size_t)Bn * ld_out);
    if (!ws.ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gcn_bwd: scratch too small: call sgnn_ctx_reserve");
    rc = sgnn_launch_spmm_x(ctx, A_T, dZ, dz16, lddz, nullptr, d_out, dP, p16, ld_out, nullptr, 0, nullptr, 0, 0, nullptr, 0, &ws, st);
    if (rc) return rc;
    if (dW) {
        rc = sgnn_launch_gemm_x(ctx, 1, 0, d_in, d_out, Bn, T->ptr, t16, T->ld, T->row_index, dP, p16, ld_out, nullptr, mfma, dW, 0, d_out,
                                nullptr, 0, 0, nullptr, &ws, st);
        if (rc) return rc;
    }
    if (dH)
        rc = sgnn_launch_gemm_x(ctx, 0, 1, Bn, d_in, d_out, dP, p16, ld_out, nullptr, W->ptr, 0, W->ld, nullptr, mfma, dH->ptr, dh16, dH->ld,
                                hmask, hm16, ldhm, nullptr, &ws, st);
    return rc;
}

int sgnn_tail_fwd(sgnn_ctx *ctx, const sgnn_mat *Z, const float *gamma, float eps, const sgnn_mat *R, float drop_q,
                  uint64_t drop_seed, uint32_t layer, uint64_t step, sgnn_mat *Y, float *inv_rms, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!mat_ok(Z) || !mat_ok(Y) || (R && !mat_ok(R)) || Z->row_index || Y->row_index || (R && R->row_index) || !(eps >= 0.f))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_fwd: bad argument");
    if (Y->rows != Z->rows || Y->cols != Z->cols || (R && (R->rows != Z->rows || R->cols != Z->cols)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_fwd: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_tail_fwd(ctx, Z->rows, Z->cols, static_cast<const float *>(Z->ptr), Z->ld, gamma, eps,
                                R ? static_cast<const float *>(R->ptr) : nullptr, R ? R->ld : 0, drop_q, drop_seed, layer, step,
                                static_cast<float *>(Y->ptr), Y->ld, inv_rms, static_cast<hipStream_t>(stream));
}

int sgnn_gemm_tail_fwd(sgnn_ctx *ctx, const sgnn_mat *T, const sgnn_mat *W, const float *gamma, float eps, const sgnn_mat *R,
                       float drop_q, uint64_t drop_seed, uint32_t layer, uint64_t step, int flags, sgnn_mat *Z, sgnn_mat *Y,
                       float *inv_rms, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!mat_ok(T) || !mat_ok(W) || !mat_ok(Z) || !mat_ok(Y) || (R && !mat_ok(R)) || T->row_index || W->row_index ||
        Z->row_index || Y->row_index || (R && R->row_index) || !(eps >= 0.f))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm_tail_fwd: bad argument");
    const int64_t M = T->rows, K = T->cols, N = W->cols;
    if (W->rows != K || Z->rows != M || Z->cols != N || Y->rows != M || Y->cols != N || (R && (R->rows != M || R->cols != N)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm_tail_fwd: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float *Rp = R ? static_cast<const float *>(R->ptr) : nullptr;
    const int64_t ldr = R ? R->ld : 0;
    if ((flags & SGNN_BF16_MFMA) && (flags & SGNN_FUSE_TAIL)) {
        rc = sgnn_launch_gemm_tail(ctx, M, N, K, static_cast<const float *>(T->ptr), T->ld, static_cast<const float *>(W->ptr),
                                   W->ld, gamma, eps, Rp, ldr, drop_q, drop_seed, layer, step, static_cast<float *>(Z->ptr),
                                   Z->ld, static_cast<float *>(Y->ptr), Y->ld, inv_rms, st);
        if (rc != SGNN_ERR_UNSUPPORTED) return rc;     // done, or a real error
    }
    // shapes outside the fused kernel: the product, then the tail
    ws_alloc ws(ctx);
    rc = sgnn_launch_gemm(ctx, 0, 0, M, N, K, static_cast<const float *>(T->ptr), T->ld, nullptr, static_cast<const float *>(W->ptr),
                          W->ld, nullptr, flags & SGNN_BF16_MFMA, static_cast<float *>(Z->ptr), Z->ld, nullptr, 0, nullptr, &ws, st);
    if (rc) return rc;
    return sgnn_launch_tail_fwd(ctx, M, N, static_cast<const float *>(Z->ptr), Z->ld, gamma, eps, Rp, ldr, drop_q, drop_seed, layer,
                                step, static_cast<float *>(Y->ptr), Y->ld, inv_rms, st);
}

int sgnn_tail_bwd(sgnn_ctx *ctx, const sgnn_mat *Z, const float *inv_rms, const float *gamma, float drop_q,
                  uint64_t drop_seed, uint32_t layer, uint64_t step, const sgnn_mat *dY, sgnn_mat *dZ, float *dgamma,
                  float *dbias, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!mat_ok(Z) || !mat_ok(dY) || !mat_ok(dZ) || !inv_rms || Z->row_index || dY->row_index || dZ->row_index)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_bwd: bad argument");
    if (dY->rows != Z->rows || dY->cols != Z->cols || dZ->rows != Z->rows || dZ->cols != Z->cols)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_bwd: shape mismatch");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_tail_bwd(ctx, Z->rows, Z->cols, static_cast<const float *>(Z->ptr), Z->ld, inv_rms, gamma, drop_q,
                                drop_seed, layer, step, static_cast<const float *>(dY->ptr), dY->ld,
                                static_cast<float *>(dZ->ptr), dZ->ld, dgamma, dbias, &ws, static_cast<hipStream_t>(stream));
}

int sgnn_sigmoid_bce(sgnn_ctx *ctx, const float *O, int64_t ldo, const float *Y, int64_t ldy, uint32_t B, uint32_t C,
                     float *loss_dev, float *dO, int64_t lddo, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!O || !Y || B == 0 || C == 0 || ldo < C || ldy < C || (dO && lddo < C))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_sigmoid_bce: bad argument");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_bce(ctx, O, ldo, Y, ldy, B, C, loss_dev, dO, lddo, &ws, static_cast<hipStream_t>(stream));
}

int sgnn_colsum(sgnn_ctx *ctx, const sgnn_mat *X, float *out, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!mat_ok(X) || X->row_index || !out) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_colsum: bad argument");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_relu_bwd_bias(ctx, nullptr, 0, 0, static_cast<const float *>(X->ptr), X->ld, 0, X->rows, X->cols, nullptr, 0,
                                     out, &ws, static_cast<hipStream_t>(stream));
}

int sgnn_sgd_step(sgnn_ctx *ctx, float *w, const float *g, int64_t n, double lr, double weight_decay, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (n < 0 || (n > 0 && (!w || !g))) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_sgd_step: bad argument");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_sgd(ctx, w, g, n, lr, weight_decay, static_cast<hipStream_t>(stream));
}

int sgnn_adam_step(sgnn_ctx *ctx, float *w, const float *g, float *m, float *v, int64_t n, double lr, double beta1,
                   double beta2, double eps, int64_t t, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (n < 0 || t < 1 || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || (n > 0 && (!w || !g || !m || !v)))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_adam_step: bad argument");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_adam(ctx, w, g, m, v, n, lr, beta1, beta2, eps, t, static_cast<hipStream_t>(stream));
}

int sgnn_graph_normalized_csr(sgnn_ctx *ctx, const sgnn_graph *g, int32_t *rowptr32, float *val, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!g || !g->rowptr || !g->colidx || !val)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_graph_normalized_csr: bad argument");
    if (g->N >= 0x7fffffffull) return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_graph_normalized_csr: N must be below 2^31");
    if (rowptr32 && g->E >= 0x7fffffffull)
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_graph_normalized_csr: %llu entries do not fit 32-bit row offsets: pass "
                                                    "rowptr32 = NULL and use the graph's own int64 offsets in the sgnn_csr",
                         (unsigned long long)g->E);
    if (!g->rowptr_is_i64 && g->E >= 0x7fffffffull)
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_graph_normalized_csr: E >= 2^31 needs an int64 rowptr");
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_graph_normalize(ctx, g, rowptr32, val, static_cast<hipStream_t>(stream));
}

int sgnn_copy_f32(sgnn_ctx *ctx, const float *src, float *dst, int64_t n, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!src || !dst || n < 0 || n % 4 != 0 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_copy_f32: need 16-byte aligned pointers and n a multiple of 4");
    if (n == 0) return SGNN_OK;
    int rc = bind_device(ctx);
    if (rc) return rc;
    return sgnn_launch_copy(ctx, src, dst, n, static_cast<hipStream_t>(stream));
}

int sgnn_softmax_xent(sgnn_ctx *ctx, const float *O, int64_t ldo, const int32_t *labels, uint32_t B, uint32_t C,
                      float *loss_dev, void *dO, int dO_dtype, int64_t lddo, float *dO_colsum, sgnn_stream stream)
{
    if (!ctx) return SGNN_ERR_INVALID_ARG;
    if (!O || !labels || B == 0 || C == 0 || ldo < C || (dO && lddo < C) || (dO_colsum && !dO) ||
        (dO && dO_dtype != SGNN_F32 && dO_dtype != SGNN_BF16))
        return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_softmax_xent: bad argument");
    int rc = bind_device(ctx);
    if (rc) return rc;
    ws_alloc ws(ctx);
    return sgnn_launch_xent(ctx, O, ldo, labels, B, C, loss_dev, dO, dO_dtype == SGNN_BF16 ? 1 : 0, lddo, dO_colsum, &ws,
                            static_cast<hipStream_t>(stream));
}

} // extern "C"
