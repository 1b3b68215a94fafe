// Sparse aggregation of the GCN layer (Sec. III-B Eq. 5 and the transposed SpMM of Sec. III-C):
// out = A X with A in CSR.  Row-split: a group of LPR lanes (a power of two up to a whole
// wavefront) owns one output row and walks its entries; each lane keeps VEC*CH consecutive-strided
// columns of the row in registers, so every gathered feature row is read with full-width
// coalesced vector loads and the output row is written once.
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
constexpr int SPMM_LONG = 96;      // rows with more entries than this are shared by the whole workgroup

// acc[m][:] += a * x[cols of chunk m]
template <int VEC, int CH>
__device__ __forceinline__ void spmm_accumulate(float (&acc)[CH][VEC], const int32_t *__restrict__ colidx,
                                                const float *__restrict__ val, int64_t e, int64_t re, int64_t stride,
                                                const float *__restrict__ X, int64_t ldx,
                                                const int32_t *__restrict__ row_index, int d, int lpr, int g)
{
    // two entries in flight per iteration
    for (; e + stride < re; e += 2 * stride) {
        const int32_t c0 = colidx[e], c1 = colidx[e + stride];
        const float a0 = val[e], a1 = val[e + stride];
        const int64_t s0 = row_index ? row_index[c0] : c0;
        const int64_t s1 = row_index ? row_index[c1] : c1;
        const float *x0 = X + s0 * ldx, *x1 = X + s1 * ldx;
        float v0[CH][VEC], v1[CH][VEC];
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) { vload<VEC>(v0[m], x0 + col); vload<VEC>(v1[m], x1 + col); }
        }
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) { acc[m][i] = fmaf(a0, v0[m][i], acc[m][i]); acc[m][i] = fmaf(a1, v1[m][i], acc[m][i]); }
            }
        }
    }
    if (e < re) {
        const int32_t c0 = colidx[e];
        const float a0 = val[e];
        const int64_t s0 = row_index ? row_index[c0] : c0;
        const float *x0 = X + s0 * ldx;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * lpr + g) * VEC;
            if (col < d) {
                float v0[VEC];
                vload<VEC>(v0, x0 + col);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[m][i] = fmaf(a0, v0[i], acc[m][i]);
            }
        }
    }
}

// Phase 1: every group of lpr lanes takes one row and walks it alone if it is short.
// Phase 2: the rows that are long are taken one after the other by the whole workgroup: the
// groups share the entries (group q takes entries q, q+G, ...), and the partial rows are summed
// through LDS in a fixed order, so the result does not depend on timing.
template <int VEC, int CH>
__global__ __launch_bounds__(SPMM_NT) void spmm_rowsplit_kernel(uint32_t rows, const int32_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ colidx,
                                                                const float *__restrict__ val, uint64_t capacity,
                                                                const float *__restrict__ X, int64_t ldx,
                                                                const int32_t *__restrict__ row_index, int d,
                                                                float *__restrict__ out, int64_t ldo, int lpr_log2)
{
    __shared__ float red[SPMM_NT * VEC];
    __shared__ uint32_t long_rows[SPMM_NT];
    __shared__ uint32_t n_long;
    const int lpr = 1 << lpr_log2;
    const int G = SPMM_NT >> lpr_log2;
    const int q = threadIdx.x >> lpr_log2;
    const int g = threadIdx.x & (lpr - 1);
    const uint32_t row = blockIdx.x * (uint32_t)G + q;
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();
    if (row < rows) {
        const int64_t rs = rowptr[row];
        const int64_t re = min((int64_t)rowptr[row + 1], (int64_t)capacity);
        if (re - rs > SPMM_LONG) {
            if (g == 0) long_rows[atomicAdd(&n_long, 1u)] = row;
        } else {
            float acc[CH][VEC];
#pragma unroll
            for (int m = 0; m < CH; ++m)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
            spmm_accumulate<VEC, CH>(acc, colidx, val, rs, re, 1, X, ldx, row_index, d, lpr, g);
            float *o = out + (int64_t)row * ldo;
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * lpr + g) * VEC;
                if (col < d) vstore<VEC>(o + col, acc[m]);
            }
        }
    }
    __syncthreads();
    const uint32_t nl = n_long;
    for (uint32_t k = 0; k < nl; ++k) {
        // the list order depends on timing, the value written for each row does not
        const uint32_t lrow = long_rows[k];
        const int64_t rs = rowptr[lrow];
        const int64_t re = min((int64_t)rowptr[lrow + 1], (int64_t)capacity);
        float acc[CH][VEC];
#pragma unroll
        for (int m = 0; m < CH; ++m)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
        spmm_accumulate<VEC, CH>(acc, colidx, val, rs + q, re, G, X, ldx, row_index, d, lpr, g);
        float *o = out + (int64_t)lrow * ldo;
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
}

template <int VEC, int CH>
int launch_vc(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int d, float *out,
              int64_t ldo, int lpr_log2, hipStream_t st)
{
    const unsigned rows_per_block = (unsigned)SPMM_NT >> lpr_log2;
    char tag[56];
    snprintf(tag, sizeof(tag), "%ux%u d=%d", A->rows, A->cols, d);
    SGNN_LAUNCH(ctx, st, "spmm_rowsplit_kernel", tag, (spmm_rowsplit_kernel<VEC, CH>), dim3(cdiv(A->rows, rows_per_block)), dim3(SPMM_NT), 0, st, A->rows,
                       A->rowptr, A->colidx, A->val, A->capacity, X, ldx, row_index, d, out, ldo, lpr_log2);
    return SGNN_OK;
}

template <int VEC>
int launch_v(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int d, float *out,
             int64_t ldo, hipStream_t st)
{
    const int per = (d + VEC - 1) / VEC;   // lanes needed for one pass over the row
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < per && lpr_log2 < 6) ++lpr_log2;
    const int ch = (per + (1 << lpr_log2) - 1) >> lpr_log2;
    switch (ch) {
    case 1: return launch_vc<VEC, 1>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 2: return launch_vc<VEC, 2>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 3: return launch_vc<VEC, 3>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 4: return launch_vc<VEC, 4>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 5: return launch_vc<VEC, 5>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 6: return launch_vc<VEC, 6>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 7: return launch_vc<VEC, 7>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    case 8: return launch_vc<VEC, 8>(ctx, A, X, ldx, row_index, d, out, ldo, lpr_log2, st);
    default: break;
    }
    return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_spmm: feature width %d is beyond %d columns", d, 64 * 8 * VEC);
}

} // namespace

int sgnn_launch_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int64_t d,
                     float *out, int64_t ldo, hipStream_t st)
{
    if (A->rows == 0 || d == 0) return SGNN_OK;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(out);
    if (d % 4 == 0 && ldx % 4 == 0 && ldo % 4 == 0 && (bits & 15) == 0)
        return launch_v<4>(ctx, A, X, ldx, row_index, (int)d, out, ldo, st);
    if (d % 2 == 0 && ldx % 2 == 0 && ldo % 2 == 0 && (bits & 7) == 0)
        return launch_v<2>(ctx, A, X, ldx, row_index, (int)d, out, ldo, st);
    return launch_v<1>(ctx, A, X, ldx, row_index, (int)d, out, ldo, st);
}
