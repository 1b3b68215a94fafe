// The element-wise tail of the paper's GNN layer as one kernel each way (Sec. III-B Eqs. 7-10,
// Sec. V "Kernel Fusion"):   Y = dropout(relu(rmsnorm(Z; gamma))) + R
// and the element-wise part of the layer backward (Sec. III-C): dropout mask, ReLU mask, RMSNorm
// backward, plus the column sums that give the gradients of gamma and of the bias.
//
// A wavefront owns a row and keeps it in registers (VEC x CH values per lane), so Z is read once,
// the mean square is a wave reduction, and Y (or dZ) is written once: 3 x B x d x 4 bytes of HBM
// traffic each way, which is what bounds these kernels.
//
// Dropout mask (Eq. 9): element e = row * d + col of layer l at step t is kept iff word e % 4 of
// Philox4x32-10 with key = (seed lo, seed hi) and counter = (e / 4 lo, e / 4 hi, t mod 2^32,
// 2^31 + l) is >= floor(q * 2^32); kept values are scaled by 1 / (1 - q).  The mask is recomputed
// in the backward pass, never stored.  A lane with four consecutive elements (16-byte aligned rows)
// spends one Philox block on them.
#include <math.h>

#include <algorithm>

#include "common.h"
#include "philox.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct tail_drop {
    uint32_t thr;      // keep iff word >= thr
    float scale;       // 1 / (1 - q)
    uint32_t k0, k1;   // key
    uint32_t c2, c3;   // counter words 2 and 3 (step, layer)
};

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// keep factors (0 or scale) of the VEC elements starting at element number e
template <int VEC> __device__ __forceinline__ void drop_factors(float (&m)[VEC], const tail_drop &dp, uint64_t e)
{
    if (dp.thr == 0) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) m[i] = 1.f;
        return;
    }
    if constexpr (VEC == 4) {
        // e is a multiple of 4 here (d and the column are): one block covers the four elements
        const uint64_t blk = e >> 2;
        const philox_out o = philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), dp.c2, dp.c3, dp.k0, dp.k1);
        m[0] = o.w0 >= dp.thr ? dp.scale : 0.f;
        m[1] = o.w1 >= dp.thr ? dp.scale : 0.f;
        m[2] = o.w2 >= dp.thr ? dp.scale : 0.f;
        m[3] = o.w3 >= dp.thr ? dp.scale : 0.f;
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const uint64_t ei = e + i, blk = ei >> 2;
            const philox_out o = philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), dp.c2, dp.c3, dp.k0, dp.k1);
            const uint32_t w = (ei & 3) == 0 ? o.w0 : ((ei & 3) == 1 ? o.w1 : ((ei & 3) == 2 ? o.w2 : o.w3));
            m[i] = w >= dp.thr ? dp.scale : 0.f;
        }
    }
}

template <int VEC> __device__ __forceinline__ void load_vec(float (&v)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const f32x4 x = *reinterpret_cast<const f32x4 *>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = x[i];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = p[i];
    }
}

template <int VEC> __device__ __forceinline__ void store_vec(float *p, const float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        f32x4 x;
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = v[i];
        *reinterpret_cast<f32x4 *>(p) = x;
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[i] = v[i];
    }
}

// One row per wavefront (grid-stride over the rows).  Columns of lane l: (m * 64 + l) * VEC + {0..VEC-1}.
template <int VEC, int CH>
__global__ __launch_bounds__(256) void tail_fwd_kernel(int64_t rows, int d, const float *__restrict__ Z, int64_t ldz,
                                                       const float *__restrict__ gamma, float eps,
                                                       const float *__restrict__ R, int64_t ldr, tail_drop dp,
                                                       float *__restrict__ Y, int64_t ldy, float *__restrict__ inv_rms)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
    float g[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * 64 + lane) * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) g[m][i] = (gamma && col + i < d) ? gamma[col + i] : 1.f;
    }
    for (int64_t row = wave; row < rows; row += nwaves) {
        float z[CH][VEC];
        float ss = 0.f;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * 64 + lane) * VEC;
#pragma unroll
            for (int i = 0; i < VEC; ++i) z[m][i] = 0.f;
            if (col < d) load_vec<VEC>(z[m], Z + row * ldz + col);
#pragma unroll
            for (int i = 0; i < VEC; ++i) ss = fmaf(z[m][i], z[m][i], ss);
        }
        ss = wave_sum(ss);
        const float ir = 1.f / sqrtf(ss / (float)d + eps);                           // Eq. 7
        if (inv_rms && lane == 0) inv_rms[row] = ir;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * 64 + lane) * VEC;
            if (col < d) {
                float keep[VEC], r[VEC], y[VEC];
                drop_factors<VEC>(keep, dp, (uint64_t)row * (uint64_t)d + (uint64_t)col);
#pragma unroll
                for (int i = 0; i < VEC; ++i) r[i] = 0.f;
                if (R) load_vec<VEC>(r, R + row * ldr + col);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const float n = g[m][i] * z[m][i] * ir;
                    y[i] = fmaxf(n, 0.f) * keep[i] + r[i];                           // Eqs. 8-10
                }
                store_vec<VEC>(Y + row * ldy + col, y);
            }
        }
    }
}

// dZ for a row per wavefront; the column sums of dn * zhat (-> dgamma) and of dZ (-> dbias) over the
// rows of a workgroup go to partial[workgroup][2][d], summed wave by wave through LDS in a fixed order.
template <int VEC, int CH>
__global__ __launch_bounds__(256) void tail_bwd_kernel(int64_t rows, int d, const float *__restrict__ Z, int64_t ldz,
                                                       const float *__restrict__ inv_rms, const float *__restrict__ gamma,
                                                       tail_drop dp, const float *__restrict__ dY, int64_t lddy,
                                                       float *__restrict__ dZ, int64_t lddz, float *__restrict__ partial)
{
    extern __shared__ float red[];   // [4 waves][2][d]
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t wave = (int64_t)blockIdx.x * 4 + w, nwaves = (int64_t)gridDim.x * 4;
    float g[CH][VEC], sg[CH][VEC], sb[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * 64 + lane) * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            g[m][i] = (gamma && col + i < d) ? gamma[col + i] : 1.f;
            sg[m][i] = 0.f;
            sb[m][i] = 0.f;
        }
    }
    for (int64_t row = wave; row < rows; row += nwaves) {
        const float ir = inv_rms[row];
        float zh[CH][VEC], dn[CH][VEC];
        float dot = 0.f;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * 64 + lane) * VEC;
#pragma unroll
            for (int i = 0; i < VEC; ++i) { zh[m][i] = 0.f; dn[m][i] = 0.f; }
            if (col < d) {
                float z[VEC], dy[VEC], keep[VEC];
                load_vec<VEC>(z, Z + row * ldz + col);
                load_vec<VEC>(dy, dY + row * lddy + col);
                drop_factors<VEC>(keep, dp, (uint64_t)row * (uint64_t)d + (uint64_t)col);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    zh[m][i] = z[i] * ir;
                    const float n = g[m][i] * zh[m][i];
                    dn[m][i] = n > 0.f ? dy[i] * keep[i] : 0.f;      // dropout mask, ReLU mask
                    sg[m][i] += dn[m][i] * zh[m][i];
                    dot = fmaf(dn[m][i] * g[m][i], zh[m][i], dot);
                }
            }
        }
        dot = wave_sum(dot) / (float)d;
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * 64 + lane) * VEC;
            if (col < d) {
                float dz[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    dz[i] = (dn[m][i] * g[m][i] - zh[m][i] * dot) * ir;     // RMSNorm backward
                    sb[m][i] += dz[i];
                }
                store_vec<VEC>(dZ + row * lddz + col, dz);
            }
        }
    }
    if (!partial) return;
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * 64 + lane) * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (col + i < d) {
                red[(w * 2 + 0) * d + col + i] = sg[m][i];
                red[(w * 2 + 1) * d + col + i] = sb[m][i];
            }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 2 * d; j += 256) {
        const float s = ((red[0 * 2 * d + j] + red[1 * 2 * d + j]) + red[2 * 2 * d + j]) + red[3 * 2 * d + j];
        partial[(int64_t)blockIdx.x * 2 * d + j] = s;
    }
}

// out[which][col] = sum over workgroups of partial[w][which][col], sixteen interleaved chains a column and
// then the sixteen chain sums in order (bit-reproducible).
__global__ __launch_bounds__(1024) void tail_colsum_final_kernel(const float *__restrict__ partial, int nwg, int d,
                                                                 float *__restrict__ dgamma, float *__restrict__ dbias)
{
    __shared__ float red[1024];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + tx;   // index into [2][d]
    float s = 0.f;
    if (j < 2 * d) {
#pragma unroll 8
        for (int w = ty; w < nwg; w += 16) s += partial[(int64_t)w * 2 * d + j];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (ty == 0 && j < 2 * d) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w * 64 + tx];
        if (j < d) { if (dgamma) dgamma[j] = t; }
        else if (dbias) dbias[j - d] = t;
    }
}

bool make_drop(float q, uint64_t seed, uint32_t layer, uint64_t step, tail_drop *dp)
{
    if (!(q >= 0.f) || !(q < 1.f)) return false;
    dp->thr = (uint32_t)floor((double)q * 4294967296.0);
    dp->scale = q > 0.f ? (float)(1.0 / (1.0 - (double)q)) : 1.f;
    dp->k0 = (uint32_t)seed;
    dp->k1 = (uint32_t)(seed >> 32);
    dp->c2 = (uint32_t)step;
    dp->c3 = 0x80000000u + layer;
    return true;
}

template <int VEC, int CH> struct tail_launch {
    static int fwd(sgnn_ctx *ctx, int64_t rows, int d, const float *Z, int64_t ldz, const float *gamma, float eps,
                   const float *R, int64_t ldr, const tail_drop &dp, float *Y, int64_t ldy, float *inv_rms, hipStream_t st)
    {
        const unsigned nwg = (unsigned)std::min<int64_t>((rows + 3) / 4, 1 << 20);
        SGNN_LAUNCH(ctx, st, "tail_fwd_kernel", SGNN_TAG, (tail_fwd_kernel<VEC, CH>), dim3(nwg), dim3(256), 0, st, rows, d, Z,
                    ldz, gamma, eps, R, ldr, dp, Y, ldy, inv_rms);
        return SGNN_OK;
    }
    static int bwd(sgnn_ctx *ctx, int64_t rows, int d, const float *Z, int64_t ldz, const float *inv_rms, const float *gamma,
                   const tail_drop &dp, const float *dY, int64_t lddy, float *dZ, int64_t lddz, float *partial, unsigned nwg,
                   hipStream_t st)
    {
        SGNN_LAUNCH(ctx, st, "tail_bwd_kernel", SGNN_TAG, (tail_bwd_kernel<VEC, CH>), dim3(nwg), dim3(256),
                    (size_t)8 * d * sizeof(float), st, rows, d, Z, ldz, inv_rms, gamma, dp, dY, lddy, dZ, lddz, partial);
        return SGNN_OK;
    }
};

#define SGNN_TAIL_DISPATCH(VEC_, ch, CALL)                                  \
    switch (ch) {                                                           \
    case 1: return tail_launch<VEC_, 1>::CALL;                              \
    case 2: return tail_launch<VEC_, 2>::CALL;                              \
    case 3: return tail_launch<VEC_, 3>::CALL;                              \
    case 4: return tail_launch<VEC_, 4>::CALL;                              \
    case 5: return tail_launch<VEC_, 5>::CALL;                              \
    case 6: return tail_launch<VEC_, 6>::CALL;                              \
    case 7: return tail_launch<VEC_, 7>::CALL;                              \
    case 8: return tail_launch<VEC_, 8>::CALL;                              \
    default: break;                                                         \
    }

} // namespace

// widest row the kernels keep in registers
static const int TAIL_MAX_D_VEC4 = 64 * 8 * 4, TAIL_MAX_D_VEC1 = 64 * 8;

int sgnn_launch_tail_fwd(sgnn_ctx *ctx, int64_t rows, int64_t d, const float *Z, int64_t ldz, const float *gamma, float eps,
                         const float *R, int64_t ldr, float q, uint64_t seed, uint32_t layer, uint64_t step, float *Y,
                         int64_t ldy, float *inv_rms, hipStream_t st)
{
    tail_drop dp;
    if (!make_drop(q, seed, layer, step, &dp)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_fwd: need 0 <= drop_q < 1");
    if (rows == 0 || d == 0) return SGNN_OK;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(Z) | reinterpret_cast<uintptr_t>(Y) | reinterpret_cast<uintptr_t>(R);
    const bool v4 = d % 4 == 0 && ldz % 4 == 0 && ldy % 4 == 0 && (!R || ldr % 4 == 0) && (bits & 15) == 0;
    if (v4 && d <= TAIL_MAX_D_VEC4) {
        const int ch = (int)((d / 4 + 63) / 64);
        SGNN_TAIL_DISPATCH(4, ch, fwd(ctx, rows, (int)d, Z, ldz, gamma, eps, R, ldr, dp, Y, ldy, inv_rms, st))
    } else if (d <= TAIL_MAX_D_VEC1) {
        const int ch = (int)((d + 63) / 64);
        SGNN_TAIL_DISPATCH(1, ch, fwd(ctx, rows, (int)d, Z, ldz, gamma, eps, R, ldr, dp, Y, ldy, inv_rms, st))
    }
    return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_tail_fwd: rows of %lld values are not supported (at most %d, or %d unaligned)",
                     (long long)d, TAIL_MAX_D_VEC4, TAIL_MAX_D_VEC1);
}

int sgnn_launch_tail_bwd(sgnn_ctx *ctx, int64_t rows, int64_t d, const float *Z, int64_t ldz, const float *inv_rms,
                         const float *gamma, float q, uint64_t seed, uint32_t layer, uint64_t step, const float *dY,
                         int64_t lddy, float *dZ, int64_t lddz, float *dgamma, float *dbias, ws_alloc *ws, hipStream_t st)
{
    tail_drop dp;
    if (!make_drop(q, seed, layer, step, &dp)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_tail_bwd: need 0 <= drop_q < 1");
    if (d == 0) return SGNN_OK;
    const bool sums = dgamma || dbias;
    const unsigned nwg = (unsigned)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, 1024));
    float *partial = nullptr;
    if (sums) {
        partial = ws->get<float>((size_t)nwg * 2 * d);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_tail_bwd: scratch too small: call sgnn_ctx_reserve");
    }
    const uintptr_t bits = reinterpret_cast<uintptr_t>(Z) | reinterpret_cast<uintptr_t>(dY) | reinterpret_cast<uintptr_t>(dZ);
    const bool v4 = d % 4 == 0 && ldz % 4 == 0 && lddy % 4 == 0 && lddz % 4 == 0 && (bits & 15) == 0;
    int rc = SGNN_ERR_UNSUPPORTED;
    auto run = [&]() -> int {
        if (v4 && d <= TAIL_MAX_D_VEC4) {
            const int ch = (int)((d / 4 + 63) / 64);
            SGNN_TAIL_DISPATCH(4, ch, bwd(ctx, rows, (int)d, Z, ldz, inv_rms, gamma, dp, dY, lddy, dZ, lddz, partial, nwg, st))
        } else if (d <= TAIL_MAX_D_VEC1) {
            const int ch = (int)((d + 63) / 64);
            SGNN_TAIL_DISPATCH(1, ch, bwd(ctx, rows, (int)d, Z, ldz, inv_rms, gamma, dp, dY, lddy, dZ, lddz, partial, nwg, st))
        }
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_tail_bwd: rows of %lld values are not supported", (long long)d);
    };
    rc = run();
    if (rc) return rc;
    if (sums)
        SGNN_LAUNCH(ctx, st, "tail_colsum_final_kernel", SGNN_TAG, tail_colsum_final_kernel, dim3(cdiv(2 * d, 64)), dim3(1024), 0,
                    st, partial, (int)nwg, (int)d, dgamma, dbias);
    return SGNN_OK;
}
