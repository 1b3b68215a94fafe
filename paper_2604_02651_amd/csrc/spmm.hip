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

template <int VEC, int CH>
__global__ __launch_bounds__(256) void spmm_rowsplit_kernel(uint32_t rows, const int32_t *__restrict__ rowptr,
                                                            const int32_t *__restrict__ colidx,
                                                            const float *__restrict__ val, uint64_t capacity,
                                                            const float *__restrict__ X, int64_t ldx,
                                                            const int32_t *__restrict__ row_index, int d,
                                                            float *__restrict__ out, int64_t ldo, int lpr_log2)
{
    const int lpr = 1 << lpr_log2;
    const uint32_t row = blockIdx.x * (256u >> lpr_log2) + (threadIdx.x >> lpr_log2);
    const int g = threadIdx.x & (lpr - 1);
    if (row >= rows) return;
    int64_t e = rowptr[row];
    const int64_t re = min((int64_t)rowptr[row + 1], (int64_t)capacity);
    float acc[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;

    for (; e + 1 < re; e += 2) {
        const int32_t c0 = colidx[e], c1 = colidx[e + 1];
        const float a0 = val[e], a1 = val[e + 1];
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
    float *o = out + (int64_t)row * ldo;
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * lpr + g) * VEC;
        if (col < d) vstore<VEC>(o + col, acc[m]);
    }
}

template <int VEC, int CH>
int launch_vc(sgnn_ctx *ctx, const sgnn_csr *A, const float *X, int64_t ldx, const int32_t *row_index, int d, float *out,
              int64_t ldo, int lpr_log2, hipStream_t st)
{
    const unsigned rows_per_block = 256u >> lpr_log2;
    char tag[56];
    snprintf(tag, sizeof(tag), "%ux%u d=%d", A->rows, A->cols, d);
    SGNN_LAUNCH(ctx, st, "spmm_rowsplit_kernel", tag, (spmm_rowsplit_kernel<VEC, CH>), dim3(cdiv(A->rows, rows_per_block)), dim3(256), 0, st, A->rows,
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
