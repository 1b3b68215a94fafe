// Sparse aggregation of the GCN layer (Sec. III-B Eq. 5 and the transposed SpMM of Sec. III-C):
// out = A X with A in CSR.
//
// Row-split with a side path for long rows.  A group of LPR lanes (a power of two up to a whole
// wavefront) owns one output row and walks its entries; each lane keeps VEC*CH columns of the row
// in registers, so every gathered feature row is read with full-width coalesced vector loads and
// the output row is written once.  Rows much longer than the mean (power-law graphs have them)
// would leave one wavefront walking alone long after the others are done, so a plan built once
// per matrix cuts them into chunks of 256 entries:
//   spmm_plan_kernel    (once per matrix) chunk descriptors of the long rows
//   spmm_main_kernel    workgroups [0, n_chunk_wgs) take chunks (entries staged in LDS, partial row
//                       per chunk), the others take rows; both kinds run side by side
//   spmm_fixup_kernel   adds the partial rows of every long row up, in chunk order
// No atomics touch floating-point data: results are bit-reproducible.
#include <stdlib.h>

#include <algorithm>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int VEC> struct vec_t;
template <> struct vec_t<1> { typedef float type; };
template <> struct vec_t<2> { typedef f32x2 type; };
template <> struct vec_t<4> { typedef f32x4 type; };

template <int VEC> __device__ __forceinline__ void vload(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 1) dst[0] = *p;
    else {
        typename vec_t<VEC>::type v = *reinterpret_cast<const typename vec_t<VEC>::type *>(p);
#pragma unroll
        for (int i = 0; i < VEC; ++i) dst[i] = v[i];
    }
}

template <int VEC> __device__ __forceinline__ void vstore(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 1) *p = src[0];
    else {
        typename vec_t<VEC>::type v;
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = src[i];
        *reinterpret_cast<typename vec_t<VEC>::type *>(p) = v;
    }
}

constexpr int SPMM_NT = 1024;      // threads of a workgroup
constexpr int SPMM_SHORT = 32;     // smallest length from which a row counts as long
constexpr int SPMM_CHUNK = 256;    // entries per chunk of a long row
constexpr unsigned SPMM_CHUNK_WGS = 256;

// Plan of a matrix (device memory): header, first chunk number per row, chunk descriptors.
struct spmm_plan_view {
    uint32_t *n_chunks;     // header word 0
    uint32_t *part_base;    // [rows], defined for long rows only
    uint2 *desc;            // [max_chunks] (row, chunk index inside the row)
};

// Rows longer than this count as long: four times the mean row length of the matrix.  Evaluated
// on the device from the true entry count when the plan is built (header word 1 of the plan).
__host__ __device__ inline int spmm_long_len(uint32_t rows, uint64_t entries)
{
    const uint64_t mean = rows ? entries / rows : 0;
    uint64_t t = 4 * mean;
    if (t < SPMM_SHORT) t = SPMM_SHORT;
    if (t > (1u << 20)) t = 1u << 20;
    return (int)t;
}

inline uint32_t spmm_max_chunks(uint32_t rows, uint64_t capacity)
{
    // a long row has more than SPMM_SHORT entries whatever the mean is: at most capacity / SPMM_SHORT
    // of them, each with at most one partly filled chunk, plus the full chunks
    (void)rows;
    const uint64_t n = capacity / SPMM_SHORT + capacity / SPMM_CHUNK + 2;
    return (uint32_t)std::min<uint64_t>(n, 0x7fffffffu);
}

inline spmm_plan_view plan_view(void *plan, uint32_t rows)
{
    uint8_t *p = static_cast<uint8_t *>(plan);
    spmm_plan_view v;
    v.n_chunks = reinterpret_cast<uint32_t *>(p);
    v.part_base = reinterpret_cast<uint32_t *>(p + 256);
    v.desc = reinterpret_cast<uint2 *>(p + 256 + (((size_t)rows * 4 + 255) & ~size_t(255)));
    return v;
}

__global__ void spmm_plan_clear_kernel(uint32_t *n_chunks) { *n_chunks = 0; }

// One thread per row: a long row reserves its chunk numbers with one atomic add, records the
// first of them in part_base[row] and writes one (row, chunk) descriptor per chunk.  The chunk
// numbering depends on timing; the values computed from it do not.
__global__ __launch_bounds__(256) void spmm_plan_kernel(uint32_t rows, const int32_t *__restrict__ rowptr, uint64_t capacity,
                                                        uint32_t *__restrict__ n_chunks,
                                                        uint32_t max_chunks, uint32_t *__restrict__ part_base,
                                                        uint2 *__restrict__ desc)
{
    const uint32_t row = blockIdx.x * 256 + threadIdx.x;
    const int long_len = spmm_long_len(rows, min((uint64_t)rowptr[rows], capacity));
    if (row == 0) n_chunks[1] = (uint32_t)long_len;
    if (row >= rows) return;
    const int64_t len = min((int64_t)rowptr[row + 1], (int64_t)capacity) - min((int64_t)rowptr[row], (int64_t)capacity);
    if (len <= long_len) return;
    const uint32_t nch = (uint32_t)((len + SPMM_CHUNK - 1) / SPMM_CHUNK);
    const uint32_t base = atomicAdd(n_chunks, nch);
    part_base[row] = base;
    for (uint32_t c = 0; c < nch && base + c < max_chunks; ++c) desc[base + c] = make_uint2(row, c);
}

// U entries e, e+1, ... fetched together: acc[m][:] += a_e * X[src_e, cols of chunk m].
// Entries at or past `re` are redirected to entry e and masked out.
template <int VEC, int CH, int U>
__device__ __forceinline__ void spmm_batch(float (&acc)[CH][VEC], const int32_t *__restrict__ colidx,
                                           const float *__restrict__ val, int64_t e, int64_t re,
                                           const float *__restrict__ X, int64_t ldx, const int32_t *__restrict__ row_index,
                                           int d, int lpr, int g)
{
    float a[U];
    bool ok[U];
    const float *x[U];
#pragma unroll
    for (int t = 0; t < U; ++t) {
        ok[t] = e + t < re;
        const int64_t ec = ok[t] ? e + t : e;
        const int32_t c = colidx[ec];
        a[t] = val[ec];
        x[t] = X + (int64_t)(row_index ? row_index[c] : c) * ldx;
    }
    float v[U][CH][VEC];
#pragma unroll
    for (int t = 0; t < U; ++t)
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) vload<VEC>(v[t][m], x[t] + col);
        }
#pragma unroll
    for (int t = 0; t < U; ++t)
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d && ok[t]) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[m][i] = fmaf(a[t], v[t][m][i], acc[m][i]);
            }
        }
}

// acc += sum over the entries [e, re) of a row.  Entries are fetched four at a time while three or
// more are left, so a short row costs one round trip to memory without redundant loads.
template <int VEC, int CH>
__device__ __forceinline__ void spmm_accumulate(float (&acc)[CH][VEC], const int32_t *__restrict__ colidx,
                                                const float *__restrict__ val, int64_t e, int64_t re,
                                                const float *__restrict__ X, int64_t ldx,
                                                const int32_t *__restrict__ row_index, int d, int lpr, int g)
{
    for (; e + 2 < re; e += 4) spmm_batch<VEC, CH, 4>(acc, colidx, val, e, re, X, ldx, row_index, d, lpr, g);
    if (e + 1 < re) spmm_batch<VEC, CH, 2>(acc, colidx, val, e, re, X, ldx, row_index, d, lpr, g);
    else if (e < re) spmm_batch<VEC, CH, 1>(acc, colidx, val, e, re, X, ldx, row_index, d, lpr, g);
}

// The same over entries already staged in LDS (source row and weight), eight in flight.
template <int VEC, int CH>
__device__ __forceinline__ void spmm_accumulate_staged(float (&acc)[CH][VEC], const int32_t *s_src, const float *s_val, int i0,
                                                       int i1, const float *__restrict__ X, int64_t ldx, int d, int lpr, int g)
{
    constexpr int U = 8;
    for (int i = i0; i < i1; i += U) {
        float v[U][CH][VEC];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const float *x = X + (int64_t)s_src[min(i + t, i1 - 1)] * ldx;
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * lpr + g) * VEC;
                if (col < d) vload<VEC>(v[t][m], x + col);
            }
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const float a = s_val[min(i + t, i1 - 1)];
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * lpr + g) * VEC;
                if (col < d && i + t < i1) {
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[m][k] = fmaf(a, v[t][m][k], acc[m][k]);
                }
            }
        }
    }
}

// Sum of the per-group partial rows of a workgroup through LDS, in group order; group 0 stores.
template <int VEC, int CH>
__device__ __forceinline__ void spmm_reduce_store(const float (&acc)[CH][VEC], float *red, float *__restrict__ o, int d,
                                                  int lpr, int G, int q, int g)
{
#pragma unroll
    for (int m = 0; m < CH; ++m) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[(q * lpr + g) * VEC + i] = acc[m][i];
        __syncthreads();
        if (q == 0) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) {
                float sum[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) sum[i] = 0.f;
                for (int w = 0; w < G; ++w)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) sum[i] += red[(w * lpr + g) * VEC + i];
                vstore<VEC>(o + col, sum);
            }
        }
        __syncthreads();
    }
}

// out = act(acc + bias) on the VEC columns starting at col
template <int VEC> __device__ __forceinline__ void spmm_epilogue(float (&v)[VEC], const float *__restrict__ bias, int relu, int col)
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if (bias) v[i] += bias[col + i];
        if (relu) v[i] = fmaxf(v[i], 0.f);
    }
}

// Workgroups [0, n_chunk_wgs): chunks of long rows.  The chunk's entries are staged in LDS with
// one coalesced load, every group of lanes takes a contiguous share, and the partial rows of the
// groups are summed through LDS in a fixed order into part[chunk number].
// The other workgroups own G = 1024 / lpr consecutive rows each, a group of lpr lanes per row; a
// row of up to long_len entries is walked by its group alone, a longer one is left to the fix-up.
template <int VEC, int CH>
__global__ __launch_bounds__(SPMM_NT) void spmm_main_kernel(uint32_t rows, const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const float *__restrict__ val, uint64_t capacity,
                                                            const float *__restrict__ X, int64_t ldx,
                                                            const int32_t *__restrict__ row_index, int d,
                                                            unsigned n_chunk_wgs, const uint32_t *__restrict__ n_chunks,
                                                            uint32_t max_chunks, const uint2 *__restrict__ desc,
                                                            float *__restrict__ part, float *__restrict__ out, int64_t ldo,
                                                            const float *__restrict__ bias, int relu, int lpr_log2)
{
    __shared__ float red[SPMM_NT * VEC];
    __shared__ int32_t s_src[SPMM_CHUNK];
    __shared__ float s_val[SPMM_CHUNK];
    const int lpr = 1 << lpr_log2;
    const int G = SPMM_NT >> lpr_log2;
    const int q = threadIdx.x >> lpr_log2;
    const int g = threadIdx.x & (lpr - 1);
    if (blockIdx.x < n_chunk_wgs) {
        const uint32_t total = min(*n_chunks, max_chunks);
        for (uint32_t pc = blockIdx.x; pc < total; pc += n_chunk_wgs) {
            const uint2 rc = desc[pc];
            const int64_t rs = rowptr[rc.x], re = min((int64_t)rowptr[rc.x + 1], (int64_t)capacity);
            const int64_t c0 = rs + (int64_t)rc.y * SPMM_CHUNK, c1 = min(re, c0 + SPMM_CHUNK);
            if (c0 + threadIdx.x < c1) {
                const int32_t cc = colidx[c0 + threadIdx.x];
                s_src[threadIdx.x] = row_index ? row_index[cc] : cc;
                s_val[threadIdx.x] = val[c0 + threadIdx.x];
            }
            __syncthreads();
            float acc[CH][VEC];
#pragma unroll
            for (int m = 0; m < CH; ++m)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
            const int nent = (int)(c1 - c0), per = (SPMM_CHUNK + G - 1) / G;
            spmm_accumulate_staged<VEC, CH>(acc, s_src, s_val, min(nent, q * per), min(nent, (q + 1) * per), X, ldx, d, lpr, g);
            spmm_reduce_store<VEC, CH>(acc, red, part + (int64_t)pc * d, d, lpr, G, q, g);   // ends with a barrier
        }
        return;
    }
    const uint32_t row = (blockIdx.x - n_chunk_wgs) * (uint32_t)G + q;
    if (row >= rows) return;
    const int64_t re = min((int64_t)rowptr[row + 1], (int64_t)capacity);
    const int64_t rs = min((int64_t)rowptr[row], re);
    if (n_chunks && re - rs > (int64_t)n_chunks[1]) return;   // a long row: its chunks and the fix-up write it
    float acc[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
    spmm_accumulate<VEC, CH>(acc, colidx, val, rs, re, X, ldx, row_index, d, lpr, g);
    float *o = out + (int64_t)row * ldo;
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * lpr + g) * VEC;
        if (col < d) {
            spmm_epilogue<VEC>(acc[m], bias, relu, col);
            vstore<VEC>(o + col, acc[m]);
        }
    }
}

// Long rows: a group of lpr lanes per row adds its partial rows up in chunk order.
template <int VEC, int CH>
__global__ __launch_bounds__(256) void spmm_fixup_kernel(const int32_t *__restrict__ rowptr, uint64_t capacity, int d,
                                                         const uint32_t *__restrict__ n_chunks, uint32_t max_chunks,
                                                         const uint2 *__restrict__ desc, const float *__restrict__ part,
                                                         float *__restrict__ out, int64_t ldo,
                                                         const float *__restrict__ bias, int relu, int lpr_log2)
{
    const int lpr = 1 << lpr_log2;
    const int G = 256 >> lpr_log2;
    const int q = threadIdx.x >> lpr_log2;
    const int g = threadIdx.x & (lpr - 1);
    const uint32_t total = min(*n_chunks, max_chunks);
    for (uint32_t pc = blockIdx.x * (uint32_t)G + q; pc < total; pc += gridDim.x * (uint32_t)G) {
        const uint2 rc = desc[pc];
        if (rc.y != 0) continue;      // only the first chunk of a row starts a sum
        const int64_t len = min((int64_t)rowptr[rc.x + 1], (int64_t)capacity) - (int64_t)rowptr[rc.x];
        const uint32_t nch = min((uint32_t)((len + SPMM_CHUNK - 1) / SPMM_CHUNK), total - pc);
        float acc[CH][VEC];
#pragma unroll
        for (int m = 0; m < CH; ++m)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
        uint32_t c = 0;
        for (; c + 4 <= nch; c += 4) {
            float v[4][CH][VEC];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int m = 0; m < CH; ++m) {
                    const int col = (m * lpr + g) * VEC;
                    if (col < d) vload<VEC>(v[t][m], part + (int64_t)(pc + c + t) * d + col);
                }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int m = 0; m < CH; ++m) {
                    const int col = (m * lpr + g) * VEC;
                    if (col < d) {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[m][i] += v[t][m][i];
                    }
                }
        }
        for (; c < nch; ++c) {
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * lpr + g) * VEC;
                if (col < d) {
                    float v[VEC];
                    vload<VEC>(v, part + (int64_t)(pc + c) * d + col);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[m][i] += v[i];
                }
            }
        }
        float *o = out + (int64_t)rc.x * ldo;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) {
                spmm_epilogue<VEC>(acc[m], bias, relu, col);
                vstore<VEC>(o + col, acc[m]);
            }
        }
    }
}

int build_plan(sgnn_ctx *ctx, const sgnn_csr *A, void *plan, hipStream_t st)
{
    const spmm_plan_view pv = plan_view(plan, A->rows);
    const uint32_t max_chunks = spmm_max_chunks(A->rows, A->capacity);
    SGNN_LAUNCH(ctx, st, "spmm_plan_clear_kernel", SGNN_TAG, spmm_plan_clear_kernel, dim3(1), dim3(1), 0, st, pv.n_chunks);
    SGNN_LAUNCH(ctx, st, "spmm_plan_kernel", SGNN_TAG, spmm_plan_kernel, dim3(cdiv(A->rows, 256)), dim3(256), 0, st, A->rows,
                A->rowptr, A->capacity, pv.n_chunks, max_chunks, pv.part_base, pv.desc);
    return SGNN_OK;
}

template <int VEC, int CH>
int launch_vc(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int d, float *out,
              int64_t ldo, const float *bias, int relu, int lpr_log2, ws_alloc *ws, hipStream_t st)
{
    const unsigned rows_per_block = (unsigned)SPMM_NT >> lpr_log2;
    char tag[56];
    snprintf(tag, sizeof(tag), "%ux%u d=%d", A->rows, A->cols, d);
    const bool may_have_long = A->capacity > (uint64_t)SPMM_SHORT;
    spmm_plan_view pv = {nullptr, nullptr, nullptr};
    float *part = nullptr;
    uint32_t max_chunks = 0;
    unsigned n_chunk_wgs = 0;
    if (may_have_long) {
        max_chunks = spmm_max_chunks(A->rows, A->capacity);
        void *plan = A->plan;
        if (!plan) {   // no plan attached to the matrix: build one for this call
            plan = ws->get<uint8_t>(sgnn_csr_plan_bytes(A->rows, A->capacity));
            if (!ws->ok)
                return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_spmm: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                                 ws->off);
            int rc = build_plan(ctx, A, plan, st);
            if (rc) return rc;
        }
        pv = plan_view(plan, A->rows);
        part = ws->get<float>((size_t)max_chunks * d);
        if (!ws->ok)
            return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_spmm: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                             ws->off);
        n_chunk_wgs = std::min<unsigned>(max_chunks, SPMM_CHUNK_WGS);
    }
    SGNN_LAUNCH(ctx, st, "spmm_main_kernel", tag, (spmm_main_kernel<VEC, CH>), dim3(n_chunk_wgs + cdiv(A->rows, rows_per_block)),
                dim3(SPMM_NT), 0, st, A->rows, A->rowptr, A->colidx, A->val, A->capacity, X, ldx, row_index, d,
                n_chunk_wgs, pv.n_chunks, max_chunks, pv.desc, part, out, ldo, bias, relu, lpr_log2);
    if (may_have_long) {
        const unsigned groups = 256u >> lpr_log2;
        SGNN_LAUNCH(ctx, st, "spmm_fixup_kernel", tag, (spmm_fixup_kernel<VEC, CH>),
                    dim3(std::min<unsigned>(cdiv(max_chunks, groups), 1024)), dim3(256), 0, st, A->rowptr, A->capacity, d,
                    pv.n_chunks, max_chunks, pv.desc, part, out, ldo, bias, relu, lpr_log2);
    }
    return SGNN_OK;
}

template <int VEC>
int launch_v(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int d, float *out,
             int64_t ldo, const float *bias, int relu, ws_alloc *ws, hipStream_t st)
{
    const int per = (d + VEC - 1) / VEC;   // lanes needed for one pass over the row
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < per && lpr_log2 < 6) ++lpr_log2;
    const int ch = (per + (1 << lpr_log2) - 1) >> lpr_log2;
    switch (ch) {
    case 1: return launch_vc<VEC, 1>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 2: return launch_vc<VEC, 2>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 3: return launch_vc<VEC, 3>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 4: return launch_vc<VEC, 4>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 5: return launch_vc<VEC, 5>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 6: return launch_vc<VEC, 6>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 7: return launch_vc<VEC, 7>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    case 8: return launch_vc<VEC, 8>(ctx, A, X, ldx, row_index, d, out, ldo, bias, relu, lpr_log2, ws, st);
    default: break;
    }
    return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_spmm: feature width %d is beyond %d columns", d, 64 * 8 * VEC);
}

} // namespace

size_t sgnn_spmm_ws_bytes(uint64_t max_entries, uint32_t B, uint32_t d_max)
{
    // a plan built on the fly plus the partial rows, for the smallest long-row threshold
    const size_t max_chunks = (size_t)(max_entries / SPMM_SHORT + max_entries / SPMM_CHUNK + 2);
    return max_chunks * ((size_t)d_max * sizeof(float) + 8) + (size_t)B * 4 + 4 * 256;
}

extern "C" uint64_t sgnn_csr_plan_bytes(uint32_t rows, uint64_t capacity)
{
    return 256 + (((uint64_t)rows * 4 + 255) & ~uint64_t(255)) + (uint64_t)spmm_max_chunks(rows, capacity) * 8 + 256;
}

int sgnn_launch_spmm_plan(sgnn_ctx *ctx, const sgnn_csr *A, hipStream_t st)
{
    if (!A->plan || A->rows == 0) return SGNN_OK;
    return build_plan(ctx, A, A->plan, st);
}

int sgnn_launch_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int64_t d,
                     float *out, int64_t ldo, const float *bias, int relu, ws_alloc *ws, hipStream_t st)
{
    if (A->rows == 0 || d == 0) return SGNN_OK;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(out);
    if (d % 4 == 0 && ldx % 4 == 0 && ldo % 4 == 0 && (bits & 15) == 0)
        return launch_v<4>(ctx, A, X, ldx, row_index, (int)d, out, ldo, bias, relu, ws, st);
    if (d % 2 == 0 && ldx % 2 == 0 && ldo % 2 == 0 && (bits & 7) == 0)
        return launch_v<2>(ctx, A, X, ldx, row_index, (int)d, out, ldo, bias, relu, ws, st);
    return launch_v<1>(ctx, A, X, ldx, row_index, (int)d, out, ldo, bias, relu, ws, st);
}
