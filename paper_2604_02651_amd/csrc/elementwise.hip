// Memory-bound helpers around the two big operators: the feature / label slice (Eq. 26), the
// element-wise part of the layer backward (ReLU mask and bias gradient), and the harness loss.
#include <algorithm>

#include "block_prims.h"
#include <math.h>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int VEC> __device__ __forceinline__ void vload(float (&dst)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(p);
        dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
    } else dst[0] = *p;
}

template <int VEC> __device__ __forceinline__ void vstore(float *p, const float (&src)[VEC])
{
    if constexpr (VEC == 4) {
        f32x4 v = {src[0], src[1], src[2], src[3]};
        *reinterpret_cast<f32x4 *>(p) = v;
    } else *p = src[0];
}

// out[i, :] = X[S[i], :];  VEC = 4 when everything is 16-byte aligned, else 1.
template <int VEC>
__global__ __launch_bounds__(256) void gather_rows_kernel(const float *__restrict__ X, int64_t dv, int64_t ldx,
                                                          const int32_t *__restrict__ S, uint32_t B,
                                                          float *__restrict__ out, int64_t ldo,
                                                          const int32_t *__restrict__ labels,
                                                          int32_t *__restrict__ labels_out)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t i = idx / dv, c = idx % dv;
    if (i >= B) return;
    const int64_t v = S[i];
    if (X) {
        if (VEC == 4)
            *reinterpret_cast<f32x4 *>(out + i * ldo + 4 * c) = *reinterpret_cast<const f32x4 *>(X + v * ldx + 4 * c);
        else
            out[i * ldo + c] = X[v * ldx + c];
    }
    if (c == 0 && labels) labels_out[i] = labels[v];
}

// dZ = dY where Y > 0 (or all of dY), and per-workgroup column sums of dZ.
// A thread owns VEC consecutive columns; tx < cwp walks the column chunks, ty the rows of the
// workgroup's slab, four rows in flight.
template <int VEC>
__global__ __launch_bounds__(256) void relu_bwd_colsum_kernel(const float *__restrict__ Y, int y_bf16, int64_t ldy,
                                                              const float *__restrict__ dY, int64_t lddy, int relu,
                                                              int64_t rows, int cols, int64_t rows_per_wg, int cwp_log2,
                                                              float *__restrict__ dZ, int64_t lddz,
                                                              float *__restrict__ partial)
{
    __shared__ float red[256 * VEC];
    const int cwp = 1 << cwp_log2, ry = 256 >> cwp_log2;
    const int tx = threadIdx.x & (cwp - 1), ty = threadIdx.x >> cwp_log2;
    const int cw = cols / VEC;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg, r1 = min(rows, r0 + rows_per_wg);
    for (int c0 = 0; c0 < cw; c0 += cwp) {
        const int ch = c0 + tx;
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
        if (ch < cw) {
            const int col = ch * VEC;
#pragma unroll 4
            for (int64_t r = r0 + ty; r < r1; r += ry) {
                float g[VEC], y[VEC];
                vload<VEC>(g, dY + r * lddy + col);
                if (relu) {
                    if (y_bf16) {      // Y stored as bfloat16: positive iff the 16-bit pattern is a positive integer
                        const uint16_t *y16 = reinterpret_cast<const uint16_t *>(Y) + r * ldy + col;
#pragma unroll
                        for (int i = 0; i < VEC; ++i) y[i] = (int16_t)y16[i] > 0 ? 1.f : 0.f;
                    } else vload<VEC>(y, Y + r * ldy + col);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) if (!(y[i] > 0.f)) g[i] = 0.f;
                }
                if (dZ) vstore<VEC>(dZ + r * lddz + col, g);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += g[i];
            }
        }
        if (partial) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) red[threadIdx.x * VEC + i] = acc[i];
            __syncthreads();
            if (ty == 0 && ch < cw) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    float s = 0.f;
                    for (int w = 0; w < ry; ++w) s += red[(w * cwp + tx) * VEC + i];
                    partial[(int64_t)blockIdx.x * cols + ch * VEC + i] = s;
                }
            }
            __syncthreads();
        }
    }
}

// out[col] = sum over workgroups of partial[w][col], in a fixed order: 16 interleaved chains a
// column, then the 16 chain sums in order.
__global__ __launch_bounds__(1024) void colsum_final_kernel(const float *__restrict__ partial, int nwg, int cols,
                                                            float *__restrict__ out)
{
    __shared__ float red[1024];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + tx;
    float s = 0.f;
    if (col < cols) {
#pragma unroll 8
        for (int w = ty; w < nwg; w += 16) s += partial[(int64_t)w * cols + col];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (ty == 0 && col < cols) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w * 64 + tx];
        out[col] = t;
    }
}

// A group of lpr lanes (a power of two >= C, at most 64) owns a row and keeps it in registers
// (NX values a lane: C <= 64 * NX); a block of XENT_PASSES * 256 / lpr rows is one round of a workgroup, which walks the
// blocks grid-stride (a fixed assignment, so every sum below is taken in the same order whenever it runs) and
// writes one partial loss and, if asked, its column sums of dO (the bias gradient of a last layer without
// activation): cs_partial[workgroup][C].  The number of workgroups is bounded by the launcher: what the final
// kernel has to add up does not grow with the batch.
#ifndef XENT_PASSES
#define XENT_PASSES 4
#endif
template <int NX>
__global__ __launch_bounds__(256) void xent_kernel(const float *__restrict__ O, int64_t ldo,
                                                   const int32_t *__restrict__ labels, uint32_t B, uint32_t C,
                                                   int lpr_log2, uint32_t n_blocks, void *__restrict__ dOv, int do_bf16,
                                                   int64_t lddo, float *__restrict__ partial, float *__restrict__ cs_partial)
{
    float *dO = static_cast<float *>(dOv);
    unsigned short *dO16 = static_cast<unsigned short *>(dOv);
    __shared__ float lds[4];
    __shared__ float cs_lds[4][64 * NX];
    float csum[NX];
#pragma unroll
    for (int t = 0; t < NX; ++t) csum[t] = 0.f;
    const int lpr = 1 << lpr_log2;
    const uint32_t rows_per_pass = 256u >> lpr_log2;
    const uint32_t gq = threadIdx.x >> lpr_log2, g = threadIdx.x & (lpr - 1);
    float loss = 0.f;
    const float invB = 1.f / (float)B;
    for (uint32_t blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
#pragma unroll
    for (int q = 0; q < XENT_PASSES; ++q) {       // unrolled: the loads of all passes go out together
        const uint32_t row = (blk * XENT_PASSES + q) * rows_per_pass + gq;
        const bool live = row < B;
        const float *o = O + (int64_t)(live ? row : 0) * ldo;
        const int32_t y = labels[live ? row : 0];      // requested along with the row: nothing below waits for a second round trip
        float x[NX];
        float m = -INFINITY;
#pragma unroll
        for (int t = 0; t < NX; ++t) {
            const uint32_t j = g + t * lpr;
            x[t] = (live && j < C) ? o[j] : -INFINITY;
            m = fmaxf(m, x[t]);
        }
        for (int s = lpr >> 1; s > 0; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
        // e = exp(x - max), kept: the probabilities are e / sum (one exponential per entry, and no rounding of
        // the log-sum-exp in between: with logits in the hundreds that rounding alone is 1e-4 of a probability)
        float sum = 0.f, oy = 0.f;      // oy: (logit of the label) - max, in the lane that holds that column
        bool mine = false;
#pragma unroll
        for (int t = 0; t < NX; ++t) {
            if ((int32_t)(g + t * lpr) == y && x[t] != -INFINITY) { oy = x[t] - m; mine = true; }
            x[t] = (x[t] == -INFINITY) ? 0.f : exp_neg(x[t] - m);
            sum += x[t];
        }
        for (int s = lpr >> 1; s > 0; s >>= 1) sum += __shfl_xor(sum, s, 64);
        if (live) {
            // - log p_y = log(sum) - (o_y - max): added by the lane that holds column y (a label outside [0, C) adds the
            // log-sum-exp alone, through lane 0 of the row)
            if (mine) loss += log_ge1(sum) - oy;
            else if (g == 0 && (uint32_t)y >= C) loss += m + log_ge1(sum);
            if (dO) {
                const float inv_sum = __builtin_amdgcn_rcpf(sum);      // 1 ulp
#pragma unroll
                for (int t = 0; t < NX; ++t) {
                    const uint32_t j = g + t * lpr;
                    if (j < C) {
                        float dv = (x[t] * inv_sum - ((int32_t)j == y ? 1.f : 0.f)) * invB;
                        if (do_bf16) {
                            // stored rounded to nearest even; the column sums add what is stored
                            const __bf16 h = (__bf16)dv;
                            dO16[(int64_t)row * lddo + j] = __builtin_bit_cast(unsigned short, h);
                            dv = (float)h;
                        } else dO[(int64_t)row * lddo + j] = dv;
                        csum[t] += dv;
                    }
                }
            }
        }
    }
    }
    loss = wave_sum(loss);
    if (lane_id() == 0) lds[threadIdx.x >> 6] = loss;
    if (cs_partial) {
        // lanes of a wavefront with the same position in their group hold the same columns
#pragma unroll
        for (int t = 0; t < NX; ++t) {
            for (int sft = lpr; sft < 64; sft <<= 1) csum[t] += __shfl_xor(csum[t], sft, 64);
            if ((int)lane_id() < lpr) cs_lds[threadIdx.x >> 6][t * lpr + g] = csum[t];
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (lds[0] + lds[1]) + (lds[2] + lds[3]);
    if (cs_partial) {
        for (int i = threadIdx.x; i < NX * lpr; i += 256) {
            const uint32_t j = (uint32_t)i;           // slot t * lpr + g holds column g + t * lpr
            if (j < C) cs_partial[(int64_t)blockIdx.x * C + j] = (cs_lds[0][i] + cs_lds[1][i]) + (cs_lds[2][i] + cs_lds[3][i]);
        }
    }
}

// Workgroup 0: the mean loss from the partial losses.  Workgroups 1 ..: 16 columns each of the column sums of
// dO, from the partial sums of the loss kernel's workgroups, added as colsum_final_kernel adds its partial sums.
// fix: optional fixed-point sums (64-bit integers, fix_slots rows of cols + 1, column `cols` = loss terms) added in
// exactly: integer addition, one conversion at the end.
__global__ __launch_bounds__(1024) void xent_final_kernel(const float *__restrict__ partial, int n, float invB,
                                                          float *__restrict__ loss, const float *__restrict__ cs_partial,
                                                          int cols, float *__restrict__ colsum,
                                                          const unsigned long long *__restrict__ fix, int fix_slots, double cs_unit,
                                                          double loss_unit)
{
    __shared__ float lds[1024];
    __shared__ long long lfix[1024];
    if (blockIdx.x == 0) {
        if (!loss) return;
        float s = 0.f;
        for (int i = threadIdx.x; i < n; i += 1024) s += partial[i];
        s = block_sum<float, 1024>(s, lds);
        long long f = 0;
        if (fix)
            for (int k = threadIdx.x; k < fix_slots; k += 1024) f += (long long)fix[(int64_t)k * (cols + 1) + cols];
        lfix[threadIdx.x] = f;
        __syncthreads();
        if (threadIdx.x == 0) {
            long long ft = 0;
            for (int k = 0; k < 1024; ++k) ft += lfix[k];          // integers: the order does not matter
            *loss = (s + (float)((double)ft * loss_unit)) * invB;
        }
        return;
    }
    // 16 columns x 64 groups of partial rows per workgroup: with 64 columns and 16 groups the three or four workgroups
    // of a 172-class layer each walked 256 rows of 4096 partial sums one after the other (25 us)
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int col = (blockIdx.x - 1) * 16 + tx;
    float s = 0.f;
    if (col < cols) {
#pragma unroll 8
        for (int w = ty; w < n; w += 64) s += cs_partial[(int64_t)w * cols + col];
    }
    lds[threadIdx.x] = s;
    long long f = 0;
    if (fix && col < cols)
        for (int k = ty; k < fix_slots; k += 64) f += (long long)fix[(int64_t)k * (cols + 1) + col];
    lfix[threadIdx.x] = f;
    __syncthreads();
    if (ty == 0 && col < cols) {
        float t = 0.f;
        long long ft = 0;
#pragma unroll
        for (int w = 0; w < 64; ++w) { t += lds[w * 16 + tx]; ft += lfix[w * 16 + tx]; }
        if (fix) t += (float)((double)ft * cs_unit);
        colsum[col] = t;
    }
}

// plain copy, 16 bytes a lane: the reference point for bandwidth counters
__global__ __launch_bounds__(256) void copy_f32_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, int64_t n4)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// Binary cross-entropy on logits: a thread per entry (grid-stride), per-workgroup partial sums of
// max(o, 0) - o y + log(1 + exp(-|o|)); dO = (s(o) - y) * inv, inv = 1 / (B C).
__global__ __launch_bounds__(256) void bce_kernel(const float *__restrict__ O, int64_t ldo, const float *__restrict__ Y, int64_t ldy,
                                                  int64_t B, int64_t C, float inv, float *__restrict__ dO, int64_t lddo,
                                                  float *__restrict__ partial)
{
    __shared__ float lds[256 / 64];
    float s = 0.f;
    const int64_t n = B * C;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / C, c = i % C;
        const float o = O[r * ldo + c], y = Y[r * ldy + c];
        const float e = expf(-fabsf(o));
        s += fmaxf(o, 0.f) - o * y + log1pf(e);
        if (dO) {
            const float sg = o >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
            dO[r * lddo + c] = (sg - y) * inv;
        }
    }
    s = block_sum<float, 256>(s, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// w <- w - lr * (g + wd * w)
__global__ __launch_bounds__(256) void sgd_kernel(float *__restrict__ w, const float *__restrict__ g, int64_t n, float lr,
                                                  float wd)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) w[i] = w[i] - lr * (g[i] + wd * w[i]);
}

// Adam with bias correction; omb = 1 - b, c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t) evaluated on the host in double precision
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ w, const float *__restrict__ g, float *__restrict__ m,
                                                   float *__restrict__ v, int64_t n, float lr, float b1, float b2, float omb1,
                                                   float omb2, float eps, float c1, float c2)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float gi = g[i];
    const float mi = b1 * m[i] + omb1 * gi;
    const float vi = b2 * v[i] + omb2 * gi * gi;
    m[i] = mi;
    v[i] = vi;
    w[i] = w[i] - lr * (mi * c1) / (sqrtf(vi * c2) + eps);
}

} // namespace

int sgnn_launch_copy(sgnn_ctx *ctx, const float *src, float *dst, int64_t n, hipStream_t st)
{
    SGNN_LAUNCH(ctx, st, "copy_f32_kernel", SGNN_TAG, copy_f32_kernel, dim3((unsigned)std::min<int64_t>((n / 4 + 255) / 256, 16384)),
                dim3(256), 0, st, reinterpret_cast<const f32x4 *>(src), reinterpret_cast<f32x4 *>(dst), n / 4);
    return SGNN_OK;
}

int sgnn_launch_gather(sgnn_ctx *ctx, const float *X, int64_t d, int64_t ldx, const int32_t *S, uint32_t B, float *out,
                       int64_t ldo, const int32_t *labels, int32_t *labels_out, hipStream_t st)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(out);
    if (!X) {   // labels only
        SGNN_LAUNCH(ctx, st, "gather_rows_kernel", SGNN_TAG, gather_rows_kernel<1>, dim3(cdiv(B, 256)), dim3(256), 0, st, X, 1, 0, S, B, out, 0, labels,
                           labels_out);
    } else if (d % 4 == 0 && ldx % 4 == 0 && ldo % 4 == 0 && (bits & 15) == 0) {
        SGNN_LAUNCH(ctx, st, "gather_rows_kernel", SGNN_TAG, gather_rows_kernel<4>, dim3(cdiv((uint64_t)B * (d / 4), 256)), dim3(256), 0, st, X, d / 4, ldx,
                           S, B, out, ldo, labels, labels_out);
    } else {
        SGNN_LAUNCH(ctx, st, "gather_rows_kernel", SGNN_TAG, gather_rows_kernel<1>, dim3(cdiv((uint64_t)B * d, 256)), dim3(256), 0, st, X, d, ldx, S, B, out,
                           ldo, labels, labels_out);
    }
    return SGNN_OK;
}

int sgnn_launch_relu_bwd_bias(sgnn_ctx *ctx, const void *Yv, int y_bf16, int64_t ldy, const float *dY, int64_t lddy, int relu,
                              int64_t rows, int64_t cols, float *dZ, int64_t lddz, float *dbias, ws_alloc *ws,
                              hipStream_t st)
{
    const float *Y = static_cast<const float *>(Yv);
    int64_t rows_per_wg = (rows + 1023) / 1024;
    if (rows_per_wg < 64) rows_per_wg = 64;
    const unsigned nwg = cdiv(rows, rows_per_wg);
    float *partial = nullptr;
    if (dbias) {
        partial = ws->get<float>((size_t)nwg * cols);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gcn_bwd: scratch too small: call sgnn_ctx_reserve");
    }
    const uintptr_t bits = reinterpret_cast<uintptr_t>(Y) | reinterpret_cast<uintptr_t>(dY) | reinterpret_cast<uintptr_t>(dZ);
    const bool v4 = cols % 4 == 0 && lddy % 4 == 0 && (!relu || ldy % 4 == 0) && (!dZ || lddz % 4 == 0) && (bits & 15) == 0;
    const int cw = (int)(v4 ? cols / 4 : cols);
    int cwp_log2 = 0;
    while ((1 << cwp_log2) < cw && cwp_log2 < 8) ++cwp_log2;
    if (v4)
        SGNN_LAUNCH(ctx, st, "relu_bwd_colsum_kernel", SGNN_TAG, relu_bwd_colsum_kernel<4>, dim3(nwg), dim3(256), 0, st, Y, y_bf16, ldy,
                    dY, lddy, relu, rows, (int)cols, rows_per_wg, cwp_log2, dZ, lddz, partial);
    else
        SGNN_LAUNCH(ctx, st, "relu_bwd_colsum_kernel", SGNN_TAG, relu_bwd_colsum_kernel<1>, dim3(nwg), dim3(256), 0, st, Y, y_bf16, ldy,
                    dY, lddy, relu, rows, (int)cols, rows_per_wg, cwp_log2, dZ, lddz, partial);
    if (dbias)
        SGNN_LAUNCH(ctx, st, "colsum_final_kernel", SGNN_TAG, colsum_final_kernel, dim3(cdiv(cols, 64)), dim3(1024), 0, st,
                    partial, (int)nwg, (int)cols, dbias);
    return SGNN_OK;
}

int sgnn_launch_xent(sgnn_ctx *ctx, const float *O, int64_t ldo, const int32_t *labels, uint32_t B, uint32_t C, float *loss,
                     void *dO, int do_bf16, int64_t lddo, float *dO_colsum, ws_alloc *ws, hipStream_t st)
{
    // lanes per row: the fewest (a power of two from 4 to 64) with which a lane holds at most eight values of a row.
    // Fewer lanes per row mean shorter reductions and more rows in flight per wavefront (172 classes: 32 lanes x 6).
    int lpr_log2 = 6;
    while (lpr_log2 > 2 && C <= (4u << lpr_log2)) --lpr_log2;
    const unsigned rows_per_block = XENT_PASSES * (256u >> lpr_log2);
    const unsigned n_blocks = cdiv(B, rows_per_block);
    const unsigned nwg = std::min(n_blocks, 4096u);     // 16 workgroups a compute unit walk the row blocks
    float *partial = ws->get<float>(nwg);
    float *cs_partial = dO_colsum ? ws->get<float>((size_t)nwg * C) : nullptr;
    if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_softmax_xent: scratch too small: call sgnn_ctx_reserve");
    const unsigned nx = (C + (1u << lpr_log2) - 1) >> lpr_log2;
#define SGNN_XENT(NX_)                                                                                                       \
    SGNN_LAUNCH(ctx, st, "xent_kernel", SGNN_TAG, xent_kernel<NX_>, dim3(nwg), dim3(256), 0, st, O, ldo, labels, B, C, lpr_log2, \
                n_blocks, dO, do_bf16, lddo, partial, cs_partial)
    if (nx <= 1) SGNN_XENT(1);
    else if (nx <= 2) SGNN_XENT(2);
    else if (nx <= 4) SGNN_XENT(4);
    else if (nx <= 6) SGNN_XENT(6);
    else if (nx <= 8) SGNN_XENT(8);
    else if (nx <= 16) SGNN_XENT(16);
    else return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_softmax_xent: more than 1024 classes are not supported");
#undef SGNN_XENT
    if (loss || dO_colsum) {
        SGNN_LAUNCH(ctx, st, "xent_final_kernel", SGNN_TAG, xent_final_kernel, dim3(1 + (dO_colsum ? cdiv(C, 16) : 0)), dim3(1024), 0, st,
                    partial, (int)nwg, 1.f / (float)B, loss, cs_partial, (int)C, dO_colsum, (const unsigned long long *)nullptr, 0, 0.0, 0.0);
    }
    return SGNN_OK;
}

int sgnn_launch_xent_final(sgnn_ctx *ctx, const float *partial, int n, float inv_rows, float *loss, const float *cs_partial, int cols,
                           float *colsum, const unsigned long long *fix, int fix_slots, double cs_unit, double loss_unit, hipStream_t st)
{
    SGNN_LAUNCH(ctx, st, "xent_final_kernel", SGNN_TAG, xent_final_kernel, dim3(1 + ((colsum && cs_partial) ? cdiv(cols, 16) : 0)), dim3(1024),
                0, st, partial, n, inv_rows, loss, cs_partial, cols, colsum, fix, fix_slots, cs_unit, loss_unit);
    return SGNN_OK;
}

int sgnn_launch_sgd(sgnn_ctx *ctx, float *w, const float *g, int64_t n, double lr, double wd, hipStream_t st)
{
    if (n == 0) return SGNN_OK;
    SGNN_LAUNCH(ctx, st, "sgd_kernel", SGNN_TAG, sgd_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, w, g, n, (float)lr, (float)wd);
    return SGNN_OK;
}

int sgnn_launch_adam(sgnn_ctx *ctx, float *w, const float *g, float *m, float *v, int64_t n, double lr, double b1, double b2,
                     double eps, int64_t t, hipStream_t st)
{
    if (n == 0) return SGNN_OK;
    const float c1 = (float)(1.0 / (1.0 - pow(b1, (double)t))), c2 = (float)(1.0 / (1.0 - pow(b2, (double)t)));
    SGNN_LAUNCH(ctx, st, "adam_kernel", SGNN_TAG, adam_kernel, dim3(cdiv(n, 256)), dim3(256), 0, st, w, g, m, v, n, (float)lr,
                (float)b1, (float)b2, (float)(1.0 - b1), (float)(1.0 - b2), (float)eps, c1, c2);
    return SGNN_OK;
}

int sgnn_launch_bce(sgnn_ctx *ctx, const float *O, int64_t ldo, const float *Y, int64_t ldy, int64_t B, int64_t C, float *loss,
                    float *dO, int64_t lddo, ws_alloc *ws, hipStream_t st)
{
    const unsigned nwg = (unsigned)std::max<int64_t>(1, std::min<int64_t>((B * C + 255) / 256, 1024));
    float *partial = ws->get<float>(nwg);
    if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_sigmoid_bce: scratch too small: call sgnn_ctx_reserve");
    const float inv = (float)(1.0 / ((double)B * (double)C));
    SGNN_LAUNCH(ctx, st, "bce_kernel", SGNN_TAG, bce_kernel, dim3(nwg), dim3(256), 0, st, O, ldo, Y, ldy, B, C, inv, dO, lddo, partial);
    if (loss)
        SGNN_LAUNCH(ctx, st, "xent_final_kernel", SGNN_TAG, xent_final_kernel, dim3(1), dim3(1024), 0, st, partial, (int)nwg, inv, loss,
                    (const float *)nullptr, 0, (float *)nullptr, (const unsigned long long *)nullptr, 0, 0.0, 0.0);
    return SGNN_OK;
}
