// Dense transform of the GCN layer on the matrix cores (Sec. III-B Eq. 6 and the two GEMMs of the
// layer backward, Sec. III-C):   C = act(op(A) op(B) + bias).
//
// fp32 path:  v_mfma_f32_32x32x2_f32  (fp32 operands, fp32 accumulate - the paper's precision)
// bf16 path:  v_mfma_f32_32x32x16_bf16, operands rounded to bfloat16 (nearest even) while they
//             are staged into LDS, fp32 accumulate.
//
// A workgroup of four wavefronts owns a BM x BN tile of C; each wavefront owns a WM x WN sub-tile
// made of 32x32 MFMA blocks whose accumulators stay in registers for the whole reduction.  Both
// operands are staged through LDS in slices of BK along the reduction, the next slice being
// fetched from HBM into registers while the current one is multiplied.
//
// MFMA operand convention used here (64 lanes, lane = 32*kh + i):
//   fp32 32x32x2 : A operand lane holds A[i][k = kh],        B operand lane holds B[k = kh][j = i]
//   bf16 32x32x16: A operand lane holds A[i][8*kh .. 8*kh+7], B operand lane holds B[8*kh..][j = i]
//   result register r of lane (kh, j) is C[8*(r/4) + 4*kh + r%4][j].
// The order in which the reduction index is fed is free as long as both operands agree, so for fp32
// the slice of 16 is fed as k = 8*kh + s at step s: every lane then reads 8 consecutive values.
#include "common.h"

#ifndef SGNN_GEMM_BK_F32
#define SGNN_GEMM_BK_F32 32   // reduction slice of the fp32 path (a multiple of 16)
#endif

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16;

struct gemm_args {
    int64_t M, N, K;          // C is M x N, reduction length K
    const float *A; int64_t lda;
    const int32_t *a_row_index;   // optional gather of the rows of A as stored in memory
    const float *B; int64_t ldb;
    const float *bias;
    float *C; int64_t ldc;
    int relu;
    int alignedA, alignedB;   // 16-byte aligned base and leading dimension a multiple of 4
    int64_t k_per_split;      // reduction range of one blockIdx.z (a multiple of BK); K when unsplit
    float *partial;           // split-K: [splits][M][N] partial products, else NULL
};

__device__ __forceinline__ u16 to_bf16_bits(float x)
{
    __bf16 h = (__bf16)x;   // v_cvt_pk_bf16_f32: round to nearest even
    return __builtin_bit_cast(u16, h);
}

// ---------------------------------------------------------------------------------------------
// Global -> register fetch of one operand slice, and register -> LDS store.
// RED_CONTIG: the operand is stored [rows][reduction] (reduction index contiguous in memory).
// otherwise : the operand is stored [reduction][rows].
// R = rows of the tile (BM or BN), BK = slice length.  Every thread fetches NV float4 chunks.
// ---------------------------------------------------------------------------------------------
template <int R, int BK, bool RED_CONTIG> struct fetch_geom {
    // chunks of 4 along the contiguous direction
    static constexpr int CHUNKS_PER_LINE = RED_CONTIG ? BK / 4 : R / 4;
    static constexpr int LINES = RED_CONTIG ? R : BK;
    static constexpr int TOTAL = CHUNKS_PER_LINE * LINES;
    static constexpr int NV = (TOTAL + 255) / 256;
};

template <int R, int BK, bool RED_CONTIG>
__device__ __forceinline__ void fetch_operand(f32x4 *reg, const float *__restrict__ G,
                                              int64_t ld, int64_t row0, int64_t rows_total, int64_t k0, int64_t k_end,
                                              int aligned, const int32_t *__restrict__ ridx = nullptr)
{
    using g = fetch_geom<R, BK, RED_CONTIG>;
#pragma unroll
    for (int v = 0; v < g::NV; ++v) {
        const int idx = v * 256 + (int)threadIdx.x;
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (g::TOTAL % 256 == 0 || idx < g::TOTAL) {
            const int line = idx / g::CHUNKS_PER_LINE, ch = idx % g::CHUNKS_PER_LINE;
            int64_t gr, gc, lim;   // line index in memory, first contiguous element, contiguous limit
            bool line_ok;
            if (RED_CONTIG) { gr = row0 + line; gc = k0 + 4 * ch; lim = k_end; line_ok = gr < rows_total; }
            else            { gr = k0 + line;  gc = row0 + 4 * ch; lim = rows_total; line_ok = gr < k_end; }
            if (line_ok) {
                if (ridx) gr = ridx[gr];
                const float *p = G + gr * ld + gc;
                if (aligned && gc + 4 <= lim) x = *reinterpret_cast<const f32x4 *>(p);
                else {
                    if (gc + 0 < lim) x[0] = p[0];
                    if (gc + 1 < lim) x[1] = p[1];
                    if (gc + 2 < lim) x[2] = p[2];
                    if (gc + 3 < lim) x[3] = p[3];
                }
            }
        }
        reg[v] = x;
    }
}

// LDS layouts
//  fp32, RED_CONTIG : [R][BK + 4]           operand read = two 16-byte loads per lane
//  fp32, otherwise  : [BK][R + 4]           operand read = eight 4-byte loads per lane (conflict free)
//  bf16 (both)      : [R][BK + 8] of 16-bit  operand read = one 16-byte load per lane
template <int R, int BK, bool RED_CONTIG, bool BF16> struct lds_geom {
    static constexpr int ELEMS = BF16 ? R * (BK + 8) : (RED_CONTIG ? R * (BK + 4) : BK * (R + 4));
    static constexpr int BYTES = ELEMS * (BF16 ? 2 : 4);
};

template <int R, int BK, bool RED_CONTIG, bool BF16>
__device__ __forceinline__ void store_operand(void *lds, const f32x4 *reg)
{
    using g = fetch_geom<R, BK, RED_CONTIG>;
#pragma unroll
    for (int v = 0; v < g::NV; ++v) {
        const int idx = v * 256 + (int)threadIdx.x;
        if (g::TOTAL % 256 != 0 && idx >= g::TOTAL) continue;
        const int line = idx / g::CHUNKS_PER_LINE, ch = idx % g::CHUNKS_PER_LINE;
        if (!BF16) {
            float *L = static_cast<float *>(lds);
            if (RED_CONTIG) *reinterpret_cast<f32x4 *>(L + line * (BK + 4) + 4 * ch) = reg[v];
            else            *reinterpret_cast<f32x4 *>(L + line * (R + 4) + 4 * ch) = reg[v];
        } else {
            u16 *L = static_cast<u16 *>(lds);
            if (RED_CONTIG) {
                // row = line, reduction offsets 4*ch .. 4*ch+3
                uint32_t lo = (uint32_t)to_bf16_bits(reg[v][0]) | ((uint32_t)to_bf16_bits(reg[v][1]) << 16);
                uint32_t hi = (uint32_t)to_bf16_bits(reg[v][2]) | ((uint32_t)to_bf16_bits(reg[v][3]) << 16);
                uint32_t *q = reinterpret_cast<uint32_t *>(L + line * (BK + 8) + 4 * ch);
                q[0] = lo; q[1] = hi;
            } else {
                // reduction index = line, rows 4*ch .. 4*ch+3: transposing store
#pragma unroll
                for (int c = 0; c < 4; ++c) L[(4 * ch + c) * (BK + 8) + line] = to_bf16_bits(reg[v][c]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool TA, bool TB, bool BF16>
__global__ __launch_bounds__(256) void gemm_kernel(gemm_args a)
{
    constexpr int BK = BF16 ? 32 : SGNN_GEMM_BK_F32;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts per workgroup");
    constexpr bool A_RC = !TA;   // A given as M x K: reduction contiguous
    constexpr bool B_RC = TB;    // B given as N x K: reduction contiguous
    using gA = fetch_geom<BM, BK, A_RC>;
    using gB = fetch_geom<BN, BK, B_RC>;

    __shared__ __attribute__((aligned(16))) unsigned char ldsA[lds_geom<BM, BK, A_RC, BF16>::BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char ldsB[lds_geom<BN, BK, B_RC, BF16>::BYTES];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const int64_t m0 = (int64_t)blockIdx.x * BM, n0 = (int64_t)blockIdx.y * BN;
    const int64_t kbeg = (int64_t)blockIdx.z * a.k_per_split;
    const int64_t kend = min(a.K, kbeg + a.k_per_split);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f32x4 ra[gA::NV], rb[gB::NV];
    if (kbeg < kend) {
        fetch_operand<BM, BK, A_RC>(ra, a.A, a.lda, m0, a.M, kbeg, kend, a.alignedA, a.a_row_index);
        fetch_operand<BN, BK, B_RC>(rb, a.B, a.ldb, n0, a.N, kbeg, kend, a.alignedB);
    }
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
        store_operand<BM, BK, A_RC, BF16>(ldsA, ra);
        store_operand<BN, BK, B_RC, BF16>(ldsB, rb);
        __syncthreads();
        if (k0 + BK < kend) {
            fetch_operand<BM, BK, A_RC>(ra, a.A, a.lda, m0, a.M, k0 + BK, kend, a.alignedA, a.a_row_index);
            fetch_operand<BN, BK, B_RC>(rb, a.B, a.ldb, n0, a.N, k0 + BK, kend, a.alignedB);
        }
        if constexpr (!BF16) {
            const float *LA = reinterpret_cast<const float *>(ldsA);
            const float *LB = reinterpret_cast<const float *>(ldsB);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                float av[TM][8], bv[TN][8];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = wm0 + 32 * i + li;
                    if (A_RC) {
                        const f32x4 x0 = *reinterpret_cast<const f32x4 *>(LA + row * (BK + 4) + kk + 8 * kh);
                        const f32x4 x1 = *reinterpret_cast<const f32x4 *>(LA + row * (BK + 4) + kk + 8 * kh + 4);
#pragma unroll
                        for (int s = 0; s < 4; ++s) { av[i][s] = x0[s]; av[i][4 + s] = x1[s]; }
                    } else {
#pragma unroll
                        for (int s = 0; s < 8; ++s) av[i][s] = LA[(kk + 8 * kh + s) * (BM + 4) + row];
                    }
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = wn0 + 32 * j + li;
                    if (B_RC) {
                        const f32x4 x0 = *reinterpret_cast<const f32x4 *>(LB + col * (BK + 4) + kk + 8 * kh);
                        const f32x4 x1 = *reinterpret_cast<const f32x4 *>(LB + col * (BK + 4) + kk + 8 * kh + 4);
#pragma unroll
                        for (int s = 0; s < 4; ++s) { bv[j][s] = x0[s]; bv[j][4 + s] = x1[s]; }
                    } else {
#pragma unroll
                        for (int s = 0; s < 8; ++s) bv[j][s] = LB[(kk + 8 * kh + s) * (BN + 4) + col];
                    }
                }
#pragma unroll
                for (int s = 0; s < 8; ++s)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][s], bv[j][s], acc[i][j], 0, 0, 0);
            }
        } else {
            const u16 *LA = reinterpret_cast<const u16 *>(ldsA);
            const u16 *LB = reinterpret_cast<const u16 *>(ldsB);
#pragma unroll
            for (int s = 0; s < BK / 16; ++s) {
                bf16x8 av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    av[i] = *reinterpret_cast<const bf16x8 *>(LA + (wm0 + 32 * i + li) * (BK + 8) + 16 * s + 8 * kh);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bv[j] = *reinterpret_cast<const bf16x8 *>(LB + (wn0 + 32 * j + li) * (BK + 8) + 16 * s + 8 * kh);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
        }
    }

    // epilogue
    float *Cout = a.partial ? a.partial + (int64_t)blockIdx.z * a.M * a.N : a.C;
    const int64_t ldc = a.partial ? a.N : a.ldc;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = n0 + wn0 + 32 * j + li;
            if (col >= a.N) continue;
            const float bj = (!a.partial && a.bias) ? a.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm0 + 32 * i + 8 * (r / 4) + 4 * kh + (r % 4);
                if (row < a.M) {
                    float z = acc[i][j][r] + bj;
                    if (!a.partial && a.relu) z = fmaxf(z, 0.f);
                    Cout[row * ldc + col] = z;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Fast fp32 path: every 16-byte chunk of an operand is either wholly inside the matrix or wholly
// outside (leading dimensions, pointers and the contiguous extents are multiples of four), so
// the fetch is branch-free: rows past the edge are clamped to the last row (they only feed
// results that are never stored) and the reduction tail is zeroed with selects.  LDS is double
// buffered: one barrier per slice; the slice after next is fetched from memory while the
// current one is multiplied.
//
// Operand staged reduction-contiguous ([R][BK+4]): tile i of the wavefront covers rows
// w0 + 32 i + li, a lane reads eight consecutive reduction values with two 16-byte loads.
// Operand staged [BK][R+4]: the T tiles of the wavefront are interleaved, tile i covers rows
// w0 + T li + i, so one 4T-byte load gives a lane its value for all T tiles.
// ---------------------------------------------------------------------------------------------
template <int R, int BK, bool RC>
__device__ __forceinline__ void fetch_fast(f32x4 *reg, const float *__restrict__ G, int64_t ld, int64_t row0,
                                           int64_t rows_total, int64_t k0, int64_t k_end, int64_t k_total,
                                           const int32_t *__restrict__ ridx = nullptr)
{
    using g = fetch_geom<R, BK, RC>;
#pragma unroll
    for (int v = 0; v < g::NV; ++v) {
        const int idx = v * 256 + (int)threadIdx.x;
        const int line = idx / g::CHUNKS_PER_LINE, ch = idx % g::CHUNKS_PER_LINE;
        int64_t gr, gc;
        bool valid;
        if (RC) {
            gr = min(row0 + line, rows_total - 1);
            gc = k0 + 4 * ch;
            valid = gc < k_end;
            gc = min(gc, k_total - 4);
        } else {
            gr = k0 + line;
            valid = gr < k_end;
            gr = min(gr, k_total - 1);
            gc = min(row0 + 4 * ch, rows_total - 4);
        }
        if (ridx) gr = ridx[gr];
        (void)valid;   // the reduction tail is zeroed by mask_fast when the slice is stored to LDS,
                       // so that nothing here waits for the load
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (g::TOTAL % 256 == 0 || idx < g::TOTAL) x = *reinterpret_cast<const f32x4 *>(G + gr * ld + gc);
        reg[v] = x;
    }
}

// zero the chunks of a fetched slice that lie at or beyond the end of the reduction range
template <int R, int BK, bool RC>
__device__ __forceinline__ void mask_fast(f32x4 *reg, int64_t k0, int64_t k_end)
{
    using g = fetch_geom<R, BK, RC>;
#pragma unroll
    for (int v = 0; v < g::NV; ++v) {
        const int idx = v * 256 + (int)threadIdx.x;
        const int line = idx / g::CHUNKS_PER_LINE, ch = idx % g::CHUNKS_PER_LINE;
        const bool valid = RC ? (k0 + 4 * ch < k_end) : (k0 + line < k_end);
        if (!valid) reg[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

template <int T> struct fvec;
template <> struct fvec<1> { typedef float type; };
template <> struct fvec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct fvec<4> { typedef f32x4 type; };

// One slice of BK reduction steps from LDS: 32x32x2 MFMAs over sixteen steps at a time.
template <int BM, int BN, int WM, int WN, int BK, bool A_RC, bool B_RC>
__device__ __forceinline__ void mma_slice(f32x16 (&acc)[WM / 32][WN / 32], const float *LA, const float *LB, int wm0, int wn0,
                                          int li, int kh)
{
    constexpr int TM = WM / 32, TN = WN / 32;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
        float av[TM][8], bv[TN][8];
        if constexpr (A_RC) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float *p = LA + (wm0 + 32 * i + li) * (BK + 4) + kk + 8 * kh;
                const f32x4 x0 = *reinterpret_cast<const f32x4 *>(p), x1 = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
                for (int s = 0; s < 4; ++s) { av[i][s] = x0[s]; av[i][4 + s] = x1[s]; }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const typename fvec<TM>::type x =
                    *reinterpret_cast<const typename fvec<TM>::type *>(LA + (kk + 8 * kh + s) * (BM + 4) + wm0 + TM * li);
                if constexpr (TM == 1) av[0][s] = x;
                else {
#pragma unroll
                    for (int i = 0; i < TM; ++i) av[i][s] = x[i];
                }
            }
        }
        if constexpr (B_RC) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float *p = LB + (wn0 + 32 * j + li) * (BK + 4) + kk + 8 * kh;
                const f32x4 x0 = *reinterpret_cast<const f32x4 *>(p), x1 = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
                for (int s = 0; s < 4; ++s) { bv[j][s] = x0[s]; bv[j][4 + s] = x1[s]; }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const typename fvec<TN>::type x =
                    *reinterpret_cast<const typename fvec<TN>::type *>(LB + (kk + 8 * kh + s) * (BN + 4) + wn0 + TN * li);
                if constexpr (TN == 1) bv[0][s] = x;
                else {
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv[j][s] = x[j];
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][s], bv[j][s], acc[i][j], 0, 0, 0);
    }
}

// Pipeline: slice s+2 is fetched from memory into registers while slice s is multiplied from LDS
// buffer s & 1; the registers are stored to the other buffer after the multiply, so there is one
// barrier per slice.
template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_fast_kernel(gemm_args a)
{
    constexpr int BK = 32;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts per workgroup");
    constexpr bool A_RC = !TA, B_RC = TB;
    using gA = fetch_geom<BM, BK, A_RC>;
    using gB = fetch_geom<BN, BK, B_RC>;
    constexpr int LA_ELEMS = lds_geom<BM, BK, A_RC, false>::ELEMS;
    constexpr int LB_ELEMS = lds_geom<BN, BK, B_RC, false>::ELEMS;
    __shared__ __attribute__((aligned(16))) float ldsA[2][LA_ELEMS];
    __shared__ __attribute__((aligned(16))) float ldsB[2][LB_ELEMS];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const int64_t m0 = (int64_t)blockIdx.x * BM, n0 = (int64_t)blockIdx.y * BN;
    const int64_t kbeg = (int64_t)blockIdx.z * a.k_per_split;
    const int64_t kend = min(a.K, kbeg + a.k_per_split);
    const int nslices = (int)((kend - kbeg + BK - 1) / BK);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f32x4 ra[gA::NV], rb[gB::NV];
    auto fetch = [&](int s) {
        fetch_fast<BM, BK, A_RC>(ra, a.A, a.lda, m0, a.M, kbeg + (int64_t)s * BK, kend, a.K, a.a_row_index);
        fetch_fast<BN, BK, B_RC>(rb, a.B, a.ldb, n0, a.N, kbeg + (int64_t)s * BK, kend, a.K);
    };
    auto stage = [&](int s) {
        mask_fast<BM, BK, A_RC>(ra, kbeg + (int64_t)s * BK, kend);
        mask_fast<BN, BK, B_RC>(rb, kbeg + (int64_t)s * BK, kend);
        store_operand<BM, BK, A_RC, false>(ldsA[s & 1], ra);
        store_operand<BN, BK, B_RC, false>(ldsB[s & 1], rb);
    };
    if (nslices > 0) {
        fetch(0);
        stage(0);
        if (nslices > 1) fetch(1);
    }
    __syncthreads();
    for (int it = 0; it < nslices; ++it) {
        mma_slice<BM, BN, WM, WN, BK, A_RC, B_RC>(acc, ldsA[it & 1], ldsB[it & 1], wm0, wn0, li, kh);
        if (it + 1 < nslices) {
            // the other buffer was last read in iteration it-1, which every wave has left
            stage(it + 1);
            if (it + 2 < nslices) fetch(it + 2);
        }
        __syncthreads();
    }

    float *Cout = a.partial ? a.partial + (int64_t)blockIdx.z * a.M * a.N : a.C;
    const int64_t ldc = a.partial ? a.N : a.ldc;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = n0 + wn0 + (B_RC ? 32 * j + li : TN * li + j);
            if (col >= a.N) continue;
            const float bj = (!a.partial && a.bias) ? a.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                const int64_t row = m0 + wm0 + (A_RC ? 32 * i + rho : TM * rho + i);
                if (row < a.M) {
                    float z = acc[i][j][r] + bj;
                    if (!a.partial && a.relu) z = fmaxf(z, 0.f);
                    Cout[row * ldc + col] = z;
                }
            }
        }
}

// Sum of the split-K partial products in a fixed order (bit-reproducible).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int splits, int64_t MN,
                                                            int64_t N, float *__restrict__ C, int64_t ldc)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    // four interleaved chains, combined in a fixed order
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int z = 0;
#pragma unroll 2
    for (; z + 3 < splits; z += 4) {
        s0 += partial[(int64_t)z * MN + i];
        s1 += partial[(int64_t)(z + 1) * MN + i];
        s2 += partial[(int64_t)(z + 2) * MN + i];
        s3 += partial[(int64_t)(z + 3) * MN + i];
    }
    for (; z < splits; ++z) s0 += partial[(int64_t)z * MN + i];
    C[(i / N) * ldc + (i % N)] = (s0 + s1) + (s2 + s3);
}

template <int BM, int BN, int WM, int WN>
int launch_cfg(sgnn_ctx *ctx, int ta, int tb, int bf16, const gemm_args &a, int splits, hipStream_t st)
{
    dim3 grid(cdiv(a.M, BM), cdiv(a.N, BN), splits), block(256);
    char tag[56];
    // fast path: fp32, every 16-byte chunk wholly inside or outside the operands
    const int64_t a_contig = ta ? a.M : a.K, b_contig = tb ? a.K : a.N;
    const bool fast = !bf16 && a.alignedA && a.alignedB && a_contig % 4 == 0 && b_contig % 4 == 0 && a_contig >= 4 &&
                      b_contig >= 4 && a.K >= 1 && a.M >= 1 && a.N >= 1;
    if (fast) {
        snprintf(tag, sizeof(tag), "%c%c %dx%d %lldx%lldx%lld f32", ta ? 'T' : 'N', tb ? 'T' : 'N', BM, BN, (long long)a.M,
                 (long long)a.N, (long long)a.K);
        if (!ta && !tb) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, false, false>), grid, block, 0, st, a); return SGNN_OK; }
        if (!ta && tb) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, false, true>), grid, block, 0, st, a); return SGNN_OK; }
        if (ta && !tb) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, true, false>), grid, block, 0, st, a); return SGNN_OK; }
    }
    snprintf(tag, sizeof(tag), "%c%c %dx%d %lldx%lldx%lld %s", ta ? 'T' : 'N', tb ? 'T' : 'N', BM, BN, (long long)a.M,
             (long long)a.N, (long long)a.K, bf16 ? "bf16" : "f32");
#define SGNN_GEMM_CASE(TA_, TB_, BF_)                                                                        \
    if (ta == TA_ && tb == TB_ && bf16 == BF_) {                                                             \
        SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_kernel<BM, BN, WM, WN, TA_, TB_, BF_>), grid, block, 0, st, a); \
        return SGNN_OK;                                                                                      \
    }
    SGNN_GEMM_CASE(false, false, false)
    SGNN_GEMM_CASE(false, true, false)
    SGNN_GEMM_CASE(true, false, false)
    SGNN_GEMM_CASE(false, false, true)
    SGNN_GEMM_CASE(false, true, true)
    SGNN_GEMM_CASE(true, false, true)
#undef SGNN_GEMM_CASE
    return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gemm: trans_a and trans_b together are not implemented");
}

} // namespace

size_t sgnn_gemm_ws_bytes(uint32_t d_max) { return (size_t)256 * d_max * d_max * 4 + 256; }

int sgnn_launch_gemm(sgnn_ctx *ctx, int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                     const int32_t *a_row_index, const float *B, int64_t ldb, const float *bias, int flags, float *C,
                     int64_t ldc, ws_alloc *ws, hipStream_t st)
{
    gemm_args a;
    a.a_row_index = a_row_index;
    a.M = M; a.N = N; a.K = K;
    a.A = A; a.lda = lda; a.B = B; a.ldb = ldb; a.bias = bias; a.C = C; a.ldc = ldc;
    a.relu = (flags & SGNN_RELU) ? 1 : 0;
    a.alignedA = ((reinterpret_cast<uintptr_t>(A) & 15) == 0 && lda % 4 == 0) ? 1 : 0;
    a.alignedB = ((reinterpret_cast<uintptr_t>(B) & 15) == 0 && ldb % 4 == 0) ? 1 : 0;
    a.k_per_split = K;
    a.partial = nullptr;
    const int bf16 = (flags & SGNN_BF16_MFMA) ? 1 : 0;
    const int BK = bf16 ? 32 : SGNN_GEMM_BK_F32;

    // tile shape by the width of C
    const int bn = N > 64 ? 128 : (N > 32 ? 64 : 32);
    const int bm = bn == 32 ? 256 : 128;
    int splits = 1;
    const int64_t tiles = (int64_t)cdiv(M, bm) * cdiv(N, bn);
    if (tiles < 256 && K >= 4096 && !bias && !(flags & SGNN_RELU)) {
        // long reduction onto a small result (the weight gradient): split the reduction
        int64_t want = (256 + tiles - 1) / tiles;
        int64_t kps = ((K + want - 1) / want + BK - 1) / BK * BK;
        if (kps < 8 * BK) kps = 8 * BK;
        splits = (int)((K + kps - 1) / kps);
        if (splits > 256) { splits = 256; kps = ((K + splits - 1) / splits + BK - 1) / BK * BK; splits = (int)((K + kps - 1) / kps); }
        if (splits > 1) {
            a.k_per_split = kps;
            a.partial = ws->get<float>((size_t)splits * M * N);
            if (!ws->ok)
                return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small for the split reduction: call sgnn_ctx_reserve");
        } else splits = 1;
    }
    int rc;
    if (bn == 128) rc = launch_cfg<128, 128, 64, 64>(ctx, ta, tb, bf16, a, splits, st);
    else if (bn == 64) rc = launch_cfg<128, 64, 64, 32>(ctx, ta, tb, bf16, a, splits, st);
    else rc = launch_cfg<256, 32, 64, 32>(ctx, ta, tb, bf16, a, splits, st);
    if (rc) return rc;
    if (splits > 1) {
        SGNN_LAUNCH(ctx, st, "splitk_reduce_kernel", SGNN_TAG, splitk_reduce_kernel, dim3(cdiv(M * N, 256)), dim3(256), 0, st, a.partial, splits, M * N, N, C,
                           ldc);
    }
    return SGNN_OK;
}
