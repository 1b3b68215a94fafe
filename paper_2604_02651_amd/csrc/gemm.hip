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
#include <math.h>

#include <algorithm>
#include <type_traits>

#include "common.h"
#include "philox.h"

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
    const float *mask; int64_t ldm;   // optional: C is zeroed where this M x N matrix is not positive
    int alignedA, alignedB;   // 16-byte aligned base and leading dimension a multiple of 4
    int vecC;                 // C (and the mask, the bias) can be written / read 16 bytes at a time: aligned, N and the leading dimensions multiples of 4
    int64_t k_per_split;      // reduction range of one blockIdx.z (a multiple of BK); K when unsplit
    float *partial;           // split-K: [splits][M][N] partial products, else NULL
    uint32_t mtiles, ntiles, splits;   // the tile grid, walked by tile_of_block()
    float *colsum;            // optional (A^T B products): column sums of B; [splits][N] partial sums when split
    int b_bf16;                   // B is stored as bfloat16 (A^T B on the chunked tile kernel only)
    int a_bf16, c_bf16, m_bf16;   // A / C / the mask are stored as bfloat16 (16-bit patterns; leading dimensions in elements).
                                  // Only the kernels that say so look at these; the launcher converts for the others.
    int vecM;                     // the mask can be read in chunks of four elements (aligned, N and ldm multiples of 4)
    int c_pair;                   // a bfloat16 C can be written two columns (4 bytes) at a time
};

// Tile of a workgroup.  The grid is one-dimensional and the hardware hands consecutive workgroup
// numbers to the eight XCDs in turn, each with an L2 of its own.  Tiles that read the same
// operand data form a group (the column tiles of one row block; with a split reduction all tiles
// of one reduction range) and are numbered so that a group's members run on one XCD next to each
// other: the shared rows then come from HBM once and from that L2 afterwards.
struct gemm_tile { uint32_t bx, by, bz; bool valid; };
__device__ __forceinline__ gemm_tile tile_of_block(const gemm_args &a)
{
    const uint32_t members = a.splits > 1 ? a.mtiles * a.ntiles : a.ntiles;
    const uint32_t groups = a.splits > 1 ? a.splits : a.mtiles;
    const uint32_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const uint32_t group = (slot / members) * 8 + xcd, mem = slot % members;
    gemm_tile t;
    t.valid = group < groups;
    if (a.splits > 1) { t.bz = group; t.bx = mem % a.mtiles; t.by = mem / a.mtiles; }
    else              { t.bz = 0; t.bx = group; t.by = mem; }
    return t;
}

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
    const gemm_tile tb_ = tile_of_block(a);
    if (!tb_.valid) return;
    const int64_t m0 = (int64_t)tb_.bx * BM, n0 = (int64_t)tb_.by * BN;
    const int64_t kbeg = (int64_t)tb_.bz * a.k_per_split;
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
    float *Cout = a.partial ? a.partial + (int64_t)tb_.bz * a.M * a.N : a.C;
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
                    if (!a.partial && a.mask && !(a.mask[row * a.ldm + col] > 0.f)) z = 0.f;
                    Cout[row * ldc + col] = z;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Fast path: every 16-byte chunk of an operand is either wholly inside the matrix or wholly
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
// SRC16: the operand is stored as bfloat16 (G points at 16-bit patterns, ld in elements): a chunk of four is
// 8 bytes and is widened to fp32 in registers, everything behind the fetch is unchanged.
__device__ __forceinline__ f32x4 widen_bf16x4(uint2 w)
{
    return f32x4{__builtin_bit_cast(float, w.x << 16), __builtin_bit_cast(float, w.x & 0xffff0000u),
                 __builtin_bit_cast(float, w.y << 16), __builtin_bit_cast(float, w.y & 0xffff0000u)};
}

template <int R, int BK, bool RC, bool SRC16 = false>
__device__ __forceinline__ void fetch_fast(typename std::conditional<SRC16, uint2, f32x4>::type *reg, const float *__restrict__ G, int64_t ld, int64_t row0,
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
        if constexpr (SRC16) {
            // kept as loaded (8 bytes of bit patterns): widened by widen_fast() when the slice is staged, so that
            // nothing but the staging waits for a load of the slice
            uint2 w = make_uint2(0u, 0u);
            if (g::TOTAL % 256 == 0 || idx < g::TOTAL) w = *reinterpret_cast<const uint2 *>(reinterpret_cast<const u16 *>(G) + gr * ld + gc);
            reg[v] = w;
        } else {
            f32x4 x = {0.f, 0.f, 0.f, 0.f};
            if (g::TOTAL % 256 == 0 || idx < g::TOTAL) x = *reinterpret_cast<const f32x4 *>(G + gr * ld + gc);
            reg[v] = x;
        }
    }
}

// chunks fetched from a bfloat16 operand (8 bytes of bit patterns) to four fp32 values
template <int R, int BK, bool RC>
__device__ __forceinline__ void widen_fast(f32x4 *reg, const uint2 *raw)
{
    using g = fetch_geom<R, BK, RC>;
#pragma unroll
    for (int v = 0; v < g::NV; ++v) reg[v] = widen_bf16x4(raw[v]);
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

// The same for the bf16 path, 32x32x16 MFMAs.  An operand staged reduction-contiguous lies in LDS
// as bfloat16 ([R][BK+8], one 16-byte load per lane and tile); an operand staged [BK][R+4] stays
// fp32 in LDS, tiles interleaved as above, and is rounded to bfloat16 when it is read.
template <int BM, int BN, int WM, int WN, int BK, bool A_RC, bool B_RC>
__device__ __forceinline__ void mma_slice_bf16(f32x16 (&acc)[WM / 32][WN / 32], const void *LAv, const void *LBv, int wm0,
                                               int wn0, int li, int kh)
{
    constexpr int TM = WM / 32, TN = WN / 32;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
        bf16x8 av[TM], bv[TN];
        if constexpr (A_RC) {
            const u16 *LA = static_cast<const u16 *>(LAv);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                av[i] = *reinterpret_cast<const bf16x8 *>(LA + (wm0 + 32 * i + li) * (BK + 8) + 16 * s + 8 * kh);
        } else {
            const float *LA = static_cast<const float *>(LAv);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const typename fvec<TM>::type x =
                    *reinterpret_cast<const typename fvec<TM>::type *>(LA + (16 * s + 8 * kh + t) * (BM + 4) + wm0 + TM * li);
                if constexpr (TM == 1) av[0][t] = (__bf16)x;
                else {
#pragma unroll
                    for (int i = 0; i < TM; ++i) av[i][t] = (__bf16)x[i];
                }
            }
        }
        if constexpr (B_RC) {
            const u16 *LB = static_cast<const u16 *>(LBv);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bv[j] = *reinterpret_cast<const bf16x8 *>(LB + (wn0 + 32 * j + li) * (BK + 8) + 16 * s + 8 * kh);
        } else {
            const float *LB = static_cast<const float *>(LBv);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const typename fvec<TN>::type x =
                    *reinterpret_cast<const typename fvec<TN>::type *>(LB + (16 * s + 8 * kh + t) * (BN + 4) + wn0 + TN * li);
                if constexpr (TN == 1) bv[0][t] = (__bf16)x;
                else {
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv[j][t] = (__bf16)x[j];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
    }
}

// Result tile of a wavefront (TM x TN blocks of 32 x 32, MFMA accumulator layout: lane (li, kh) holds
// column li of rows 8 (r / 4) + 4 kh + r % 4, r = 0..15) to memory with bias / ReLU / mask.
//   columns interleaved (B given [reduction][columns]): a lane owns TN adjacent columns: one vector store each;
//   columns in blocks of 32 (B reduction-contiguous): a band of 32 rows goes through the wavefront's LDS slot
//     (32 x (32 TN + 4) floats) and leaves as rows of 16 bytes per lane, the mask read the same way.
// Without a.vecC (odd sizes, unaligned C): one element at a time.
template <int TM, int TN, bool A_RC, bool B_RC>
__device__ __forceinline__ void store_tile(const gemm_args &a, const f32x16 (&acc)[TM][TN], float *__restrict__ Cout, int64_t ldc,
                                           int64_t row0, int64_t col0, int li, int kh, float *stage)
{
    const bool plain = a.partial != nullptr;     // partial products of a split reduction: no epilogue
    if (!a.vecC) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = col0 + (B_RC ? 32 * j + li : TN * li + j);
                if (col >= a.N) continue;
                const float bj = (!plain && a.bias) ? a.bias[col] : 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                    const int64_t row = row0 + (A_RC ? 32 * i + rho : TM * rho + i);
                    if (row < a.M) {
                        float z = acc[i][j][r] + bj;
                        if (!plain && a.relu) z = fmaxf(z, 0.f);
                        if (!plain && a.mask && !(a.mask[row * a.ldm + col] > 0.f)) z = 0.f;
                        Cout[row * ldc + col] = z;
                    }
                }
            }
        return;
    }
    if constexpr (!B_RC) {
        // the lane's TN columns are adjacent
        const int64_t col = col0 + TN * li;
        if (col >= a.N) return;          // N is a multiple of 4 and TN divides 4: the group is wholly inside or outside
        float bj[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) bj[j] = (!plain && a.bias) ? a.bias[col + j] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            typename fvec<TN>::type m[16];
            if (!plain && a.mask) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                    const int64_t row = row0 + (A_RC ? 32 * i + rho : TM * rho + i);
                    if (row < a.M) m[r] = *reinterpret_cast<const typename fvec<TN>::type *>(a.mask + row * a.ldm + col);
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                const int64_t row = row0 + (A_RC ? 32 * i + rho : TM * rho + i);
                if (row >= a.M) continue;
                typename fvec<TN>::type z;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    float t = acc[i][j][r] + bj[j];
                    if (!plain && a.relu) t = fmaxf(t, 0.f);
                    if (!plain && a.mask) {
                        float mv;
                        if constexpr (TN == 1) mv = m[r]; else mv = m[r][j];
                        if (!(mv > 0.f)) t = 0.f;
                    }
                    if constexpr (TN == 1) z = t; else z[j] = t;
                }
                *reinterpret_cast<typename fvec<TN>::type *>(Cout + row * ldc + col) = z;
            }
        }
    } else {
        constexpr int LDW = 32 * TN + 4;          // floats per staged row: 16-byte aligned rows, banks shifted row to row
        const int lane = li + 32 * kh;
        float bj[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = col0 + 32 * j + li;
            bj[j] = (!plain && a.bias && col < a.N) ? a.bias[col] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            static_assert(A_RC, "a reduction-contiguous B comes with a reduction-contiguous A");
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                    float t = acc[i][j][r] + bj[j];
                    if (!plain && a.relu) t = fmaxf(t, 0.f);
                    stage[rho * LDW + 32 * j + li] = t;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            constexpr int C4 = 8 * TN;            // groups of 4 columns per row
            constexpr int PASSES = 32 * C4 / 64;
            f32x4 z[PASSES], m[PASSES];
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int idx = p * 64 + lane, rr = idx / C4, c4 = idx % C4;
                const int64_t row = row0 + 32 * i + rr, col = col0 + 4 * c4;
                z[p] = *reinterpret_cast<const f32x4 *>(stage + rr * LDW + 4 * c4);
                if (!plain && a.mask && row < a.M && col < a.N) m[p] = *reinterpret_cast<const f32x4 *>(a.mask + row * a.ldm + col);
            }
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int idx = p * 64 + lane, rr = idx / C4, c4 = idx % C4;
                const int64_t row = row0 + 32 * i + rr, col = col0 + 4 * c4;
                if (row >= a.M || col >= a.N) continue;
                if (!plain && a.mask) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (!(m[p][e] > 0.f)) z[p][e] = 0.f;
                }
                *reinterpret_cast<f32x4 *>(Cout + row * ldc + col) = z[p];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Pipeline: slice s+2 is fetched from memory into registers while slice s is multiplied from LDS
// buffer s & 1; the registers are stored to the other buffer after the multiply, so there is one
// barrier per slice.
// ABF: A is stored as bfloat16 (the saved aggregate of a layer whose activations are kept in bfloat16).
template <int BM, int BN, int WM, int WN, bool TA, bool TB, bool BF16, bool ABF = false, bool BBF = false>
__global__ __launch_bounds__(256) void gemm_fast_kernel(gemm_args a)
{
    constexpr int BK = 32;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts per workgroup");
    constexpr bool A_RC = !TA, B_RC = TB;
    using gA = fetch_geom<BM, BK, A_RC>;
    using gB = fetch_geom<BN, BK, B_RC>;
    constexpr bool A16 = BF16 && A_RC, B16 = BF16 && B_RC;   // staged as bfloat16 (else fp32)
    constexpr int LA_BYTES = lds_geom<BM, BK, A_RC, A16>::BYTES;
    constexpr int LB_BYTES = lds_geom<BN, BK, B_RC, B16>::BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char ldsA[2][LA_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char ldsB[2][LB_BYTES];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const gemm_tile tb_ = tile_of_block(a);
    if (!tb_.valid) return;
    const int64_t m0 = (int64_t)tb_.bx * BM, n0 = (int64_t)tb_.by * BN;
    const int64_t kbeg = (int64_t)tb_.bz * a.k_per_split;
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
    typename std::conditional<ABF, uint2, f32x4>::type *ra_fetch;      // where the fetch puts A: ra itself, or the raw 16-bit chunks
    uint2 ra16[ABF ? gA::NV : 1];
    if constexpr (ABF) ra_fetch = ra16; else ra_fetch = ra;
    typename std::conditional<BBF, uint2, f32x4>::type *rb_fetch;
    uint2 rb16[BBF ? gB::NV : 1];
    if constexpr (BBF) rb_fetch = rb16; else rb_fetch = rb;
    auto fetch = [&](int s) {
        fetch_fast<BM, BK, A_RC, ABF>(ra_fetch, a.A, a.lda, m0, a.M, kbeg + (int64_t)s * BK, kend, a.K, a.a_row_index);
        fetch_fast<BN, BK, B_RC, BBF>(rb_fetch, a.B, a.ldb, n0, a.N, kbeg + (int64_t)s * BK, kend, a.K);
    };
    // column sums of B (the bias gradient next to dW = T^T dZ): every thread fetches the same four columns
    // of B in every slice, so it adds its chunks up as they pass; only the first row block of tiles does it
    f32x4 cs = {0.f, 0.f, 0.f, 0.f};
    const bool do_cs = TA && !TB && a.colsum && tb_.bx == 0;
    auto stage = [&](int s) {
        if constexpr (ABF) widen_fast<BM, BK, A_RC>(ra, ra16);
        if constexpr (BBF) widen_fast<BN, BK, B_RC>(rb, rb16);
        mask_fast<BM, BK, A_RC>(ra, kbeg + (int64_t)s * BK, kend);
        mask_fast<BN, BK, B_RC>(rb, kbeg + (int64_t)s * BK, kend);
        if constexpr (TA && !TB) {
            if (do_cs) {
#pragma unroll
                for (int v = 0; v < gB::NV; ++v) cs += rb[v];
            }
        }
        store_operand<BM, BK, A_RC, A16>(ldsA[s & 1], ra);
        store_operand<BN, BK, B_RC, B16>(ldsB[s & 1], rb);
    };
    if (nslices > 0) {
        fetch(0);
        stage(0);
        if (nslices > 1) fetch(1);
    }
    __syncthreads();
    for (int it = 0; it < nslices; ++it) {
        if constexpr (BF16) mma_slice_bf16<BM, BN, WM, WN, BK, A_RC, B_RC>(acc, ldsA[it & 1], ldsB[it & 1], wm0, wn0, li, kh);
        else
            mma_slice<BM, BN, WM, WN, BK, A_RC, B_RC>(acc, reinterpret_cast<const float *>(ldsA[it & 1]),
                                                      reinterpret_cast<const float *>(ldsB[it & 1]), wm0, wn0, li, kh);
        if (it + 1 < nslices) {
            // the other buffer was last read in iteration it-1, which every wave has left
            stage(it + 1);
            if (it + 2 < nslices) fetch(it + 2);
        }
        __syncthreads();
    }

    if constexpr (TA && !TB) {
        if (do_cs) {   // the loop ended with a barrier: the staging buffers are free
            static_assert(gB::TOTAL % 256 == 0 && 256 % gB::CHUNKS_PER_LINE == 0, "a thread keeps its columns in every slice");
            constexpr int CPL = gB::CHUNKS_PER_LINE, G = 256 / CPL;
            float *red = reinterpret_cast<float *>(ldsA[0]);
#pragma unroll
            for (int e = 0; e < 4; ++e) red[threadIdx.x * 4 + e] = cs[e];
            __syncthreads();
            if (threadIdx.x < BN) {
                const int ch = threadIdx.x >> 2, e = threadIdx.x & 3;
                float t = 0.f;
                for (int q = 0; q < G; ++q) t += red[(ch + CPL * q) * 4 + e];
                const int64_t col = n0 + threadIdx.x;
                if (col < a.N) a.colsum[(a.partial ? (int64_t)tb_.bz * a.N : 0) + col] = t;
            }
        }
    }

    float *Cout = a.partial ? a.partial + (int64_t)tb_.bz * a.M * a.N : a.C;
    const int64_t ldc = a.partial ? a.N : a.ldc;
    // staging area of the epilogue (a slot per wavefront; only the block-column layout needs it)
    __shared__ __attribute__((aligned(16))) float epi_stage[B_RC ? 4 * 32 * (32 * TN + 4) : 4];
    float *epi_lds = epi_stage + (B_RC ? (threadIdx.x >> 6) * 32 * (32 * TN + 4) : 0);
    store_tile<TM, TN, A_RC, B_RC>(a, acc, Cout, ldc, m0 + wm0, n0 + wn0, li, kh, epi_lds);
}

// ---------------------------------------------------------------------------------------------
// fp32 path with direct global -> LDS loads (global_load_lds_dwordx4: lane l's 16 bytes land at
// a wave-uniform LDS base + 16 l, no register staging).  256 x 128 tile, eight wavefronts with
// 64 x 64 sub-tiles (two per SIMD) - or, for the split reductions of the weight gradients, a
// 128 x 128 tile, eight wavefronts with 64 x 32 sub-tiles - slices of 32 along the reduction in a ring of three LDS
// stages: slice s + 2 is in flight while slice s is multiplied, one barrier per slice placed in the
// middle of the slice's multiplies, waits on the loads stated explicitly (vmcnt).  Needs whole 16-byte chunks (as the fast path) and a
// reduction range that is a multiple of 32.
//
// LDS layouts (no padding, a wavefront load covers 1 KB of contiguous LDS):
//   reduction-contiguous operand: [row][8 chunks of 16 bytes]; position p of row r holds chunk
//     p ^ ((r >> 1) & 7) of the slice, so that the 32 rows a half-wavefront reads at one reduction
//     offset fall into different banks;
//   operand given [reduction][rows]: [k][R] as in memory; a lane reads its tiles' values at
//     consecutive addresses (tiles interleaved as in the fast path).
// ---------------------------------------------------------------------------------------------
#define SGNN_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SGNN_LPTR(p) ((__attribute__((address_space(3))) void *)(p))
constexpr int DIRECT_BM = 256, DIRECT_BN = 128, DIRECT_BK = 32, DIRECT_STAGES = 3, DIRECT_WAVES = 8;

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left at their maxima), gfx9 encoding
#define SGNN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

// Issues the loads of one operand slice: R rows, wave-loads dealt round-robin to the WAVES wavefronts.
template <int R, bool RC, int WAVES>
__device__ __forceinline__ void direct_issue(float *lds, const float *__restrict__ G, int64_t ld, int64_t row0, int64_t rows_total,
                                             int64_t k0, const int32_t *__restrict__ ridx, int lane, int wave)
{
    constexpr int LOADS = R * DIRECT_BK / 4 / 64 / WAVES;   // wave-loads per wavefront
    static_assert(LOADS * 64 * WAVES * 4 == R * DIRECT_BK, "the wavefronts share the slice evenly");
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int q = wave + WAVES * j;   // wave-load number: LDS floats [256 q, 256 q + 256)
        const float *g;
        if (RC) {
            const int r = 8 * q + (lane >> 3), pos = lane & 7;
            int64_t gr = min(row0 + r, rows_total - 1);
            if (ridx) gr = ridx[gr];
            g = G + gr * ld + k0 + 4 * (pos ^ ((r >> 1) & 7));
        } else {
            const int f = 64 * q + lane;                   // chunk number in the [k][R / 4] array
            const int k = f / (R / 4), ch = f % (R / 4);
            g = G + (k0 + k) * ld + min(row0 + 4 * ch, rows_total - 4);
        }
        __builtin_amdgcn_global_load_lds(SGNN_GPTR(g), SGNN_LPTR(lds + 256 * q), 16, 0, 0);
    }
}

// The same for a transposed operand whose reduction rows are gathered (row k of the operand is row ridx[k] of G).
// The indices of a slice are fetched one slice ahead, before the loads of the current slice are issued: by the time
// they are used, only loads issued after them are outstanding, so the wait the compiler places before their use
// does not drain the slice in flight.  Whatever order the loads end up in, the wait before the barrier
// (at most as many operations outstanding as one slice has loads) still covers every older slice.
template <int R, int WAVES>
__device__ __forceinline__ void direct_issue_gathered_t(float *lds, const float *__restrict__ G, int64_t ld, int64_t row0,
                                                        int64_t rows_total, int64_t k0_next, const int32_t *__restrict__ ridx,
                                                        int lane, int wave, int32_t (&rows)[R * DIRECT_BK / 4 / 64 / WAVES])
{
    constexpr int LOADS = R * DIRECT_BK / 4 / 64 / WAVES;
    int32_t cur[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) cur[j] = rows[j];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) rows[j] = ridx[k0_next + (64 * (wave + WAVES * j) + lane) / (R / 4)];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int q = wave + WAVES * j, ch = (64 * q + lane) % (R / 4);
        const float *g = G + (int64_t)cur[j] * ld + min(row0 + 4 * ch, rows_total - 4);
        __builtin_amdgcn_global_load_lds(SGNN_GPTR(g), SGNN_LPTR(lds + 256 * q), 16, 0, 0);
    }
}

// Operand values of one quad of a slice: reduction steps kk + 8 kh + 4 half + {0..3} for the T tiles of the wavefront.
template <int R, bool RC, int T>
__device__ __forceinline__ void direct_frag(float (&v)[T][4], const float *L, int w0, int kk, int half, int li, int kh)
{
    if constexpr (RC) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int r = w0 + 32 * t + li, c = kk / 4 + 2 * kh + half;
            const f32x4 x = *reinterpret_cast<const f32x4 *>(L + r * 32 + 4 * (c ^ ((r >> 1) & 7)));
#pragma unroll
            for (int s = 0; s < 4; ++s) v[t][s] = x[s];
        }
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const typename fvec<T>::type x =
                *reinterpret_cast<const typename fvec<T>::type *>(L + (kk + 8 * kh + 4 * half + s) * R + w0 + T * li);
            if constexpr (T == 1) v[0][s] = x;
            else {
#pragma unroll
                for (int t = 0; t < T; ++t) v[t][s] = x[t];
            }
        }
    }
}

template <int BM, int WAVES, int TN, bool TA, bool TB, bool GATHER>
__global__ __launch_bounds__(64 * WAVES) void gemm_direct_kernel(gemm_args a)
{
    constexpr int BN = DIRECT_BN, BK = DIRECT_BK, TM = 2;
    constexpr int WAVES_N = BN / (32 * TN);
    static_assert(BM * BN == WAVES * 64 * 32 * TN, "a 64 x 32 TN sub-tile per wavefront");
    constexpr int STAGE_FLOATS = (BM + BN) * BK;
    constexpr bool A_RC = !TA, B_RC = TB;
    constexpr int LOADS = (BM + BN) * BK / 4 / 64 / WAVES;   // loads per thread and slice
    extern __shared__ __attribute__((aligned(16))) float direct_smem[];
    const gemm_tile tb_ = tile_of_block(a);
    if (!tb_.valid) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    const int wm0 = (wave / WAVES_N) * 64, wn0 = (wave % WAVES_N) * (32 * TN);
    const int64_t m0 = (int64_t)tb_.bx * BM, n0 = (int64_t)tb_.by * BN;
    const int64_t kbeg = (int64_t)tb_.bz * a.k_per_split;
    const int64_t kend = min(a.K, kbeg + a.k_per_split);
    const int nslices = (int)((kend - kbeg) / BK);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // a slice number past the end loads the last slice again, into a stage nobody reads any more:
    // the loop body then has no branch, and every wait in it counts a fixed number of operations
    constexpr int LOADS_A = BM * BK / 4 / 64 / WAVES;
    [[maybe_unused]] int32_t a_rows[LOADS_A];   // gathered A^T: the rows of the slice issued next
    if constexpr (GATHER && TA) {
        if (nslices > 0) {
#pragma unroll
            for (int j = 0; j < LOADS_A; ++j) a_rows[j] = a.a_row_index[kbeg + (64 * (wave + WAVES * j) + lane) / (BM / 4)];
        }
    }
    auto issue = [&](int s) {
        float *st = direct_smem + (s % DIRECT_STAGES) * STAGE_FLOATS;
        const int64_t k0 = kbeg + (int64_t)min(s, nslices - 1) * BK;
        if constexpr (GATHER && TA) {
            const int64_t k0_next = kbeg + (int64_t)min(s + 1, nslices - 1) * BK;
            direct_issue_gathered_t<BM, WAVES>(st, a.A, a.lda, m0, a.M, k0_next, a.a_row_index, lane, wave, a_rows);
        } else
        direct_issue<BM, A_RC, WAVES>(st, a.A, a.lda, m0, a.M, k0, GATHER ? a.a_row_index : nullptr, lane, wave);
        direct_issue<BN, B_RC, WAVES>(st + BM * BK, a.B, a.ldb, n0, a.N, k0, nullptr, lane, wave);
    };
    // Schedule of a slice (four quads of four reduction steps each, operand values double buffered in
    // registers):   read q1 | multiply q0 | read q2 | multiply q1 | wait + barrier + issue slice it+2 |
    //               read q3 | multiply q2 | read q0 of slice it+1 | multiply q3
    // The barrier sits in the middle of the multiplies: it publishes slice it + 1 (loaded one slice
    // ago) and proves that everyone has left slice it - 1, whose stage the new loads overwrite, so
    // no wavefront ever waits on memory or LDS latency with an empty MFMA queue behind it.
    float av[2][TM][4], bv[2][TN][4];
    auto frags = [&](int buf, int slice, int q) {
        const float *LA = direct_smem + (slice % DIRECT_STAGES) * STAGE_FLOATS, *LB = LA + BM * BK;
        direct_frag<BM, A_RC, TM>(av[buf], LA, wm0, 16 * (q / 2), q & 1, li, kh);
        direct_frag<BN, B_RC, TN>(bv[buf], LB, wn0, 16 * (q / 2), q & 1, li, kh);
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[buf][i][s], bv[buf][j][s], acc[i][j], 0, 0, 0);
    };
    if (nslices > 0) {
        issue(0);
        issue(1);
        SGNN_WAIT_VMCNT(LOADS);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        frags(0, 0, 0);
    }
    // column sums of B (the bias gradient next to dW = T^T dZ), by the first row block of tiles only: B of a
    // slice lies in LDS as [32 reduction steps][128 columns]; a thread adds up its column over every
    // (threads / 128)-th reduction step while the slice is current
    constexpr int CS_PARTS = WAVES * 64 / BN;
    const bool do_cs = TA && !TB && a.colsum && tb_.bx == 0;
    float cs = 0.f;
    for (int it = 0; it < nslices; ++it) {
        frags(1, it, 1);
        if constexpr (TA && !TB) {
            if (do_cs) {
                const float *LB = direct_smem + (it % DIRECT_STAGES) * STAGE_FLOATS + BM * BK;
#pragma unroll
                for (int k = 0; k < BK / CS_PARTS; ++k) cs += LB[(k * CS_PARTS + threadIdx.x / BN) * BN + threadIdx.x % BN];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        multiply(0);
        __builtin_amdgcn_sched_barrier(0);
        frags(0, it, 2);
        __builtin_amdgcn_sched_barrier(0);
        multiply(1);
        __builtin_amdgcn_sched_barrier(0);
        SGNN_WAIT_VMCNT(0);   // this thread's part of slice it + 1 (the only loads in flight) has landed
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(it + 2);   // into the stage slice it - 1 was read from
        frags(1, it, 3);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0);
        __builtin_amdgcn_sched_barrier(0);
        frags(0, it + 1, 0);   // (after the last slice: values nobody uses)
        __builtin_amdgcn_sched_barrier(0);
        multiply(1);
        __builtin_amdgcn_sched_barrier(0);
    }

    if constexpr (TA && !TB) {
        if (do_cs) {
            __syncthreads();      // every wavefront is through its last slice: the stages are free
            direct_smem[threadIdx.x] = cs;
            __syncthreads();
            const int64_t col = n0 + threadIdx.x;
            if (threadIdx.x < BN && col < a.N) {
                float t = 0.f;
#pragma unroll
                for (int p = 0; p < CS_PARTS; ++p) t += direct_smem[p * BN + threadIdx.x];
                a.colsum[(a.partial ? (int64_t)tb_.bz * a.N : 0) + col] = t;
            }
        }
    }
    float *Cout = a.partial ? a.partial + (int64_t)tb_.bz * a.M * a.N : a.C;
    const int64_t ldc = a.partial ? a.N : a.ldc;
    float *stage = nullptr;
    if constexpr (B_RC) {
        __syncthreads();      // every wavefront is through its last slice: the stages are free
        stage = direct_smem + (threadIdx.x >> 6) * 32 * (32 * TN + 4);
    }
    store_tile<TM, TN, A_RC, B_RC>(a, acc, Cout, ldc, m0 + wm0, n0 + wn0, li, kh, stage);
}

int launch_direct(sgnn_ctx *ctx, int ta, int tb, gemm_args a, int splits, bool bm128, hipStream_t st)
{
    const int bm = bm128 ? 128 : DIRECT_BM, waves = DIRECT_WAVES;
    a.mtiles = (uint32_t)cdiv(a.M, bm);
    a.ntiles = (uint32_t)cdiv(a.N, DIRECT_BN);
    a.splits = (uint32_t)splits;
    const uint64_t members = splits > 1 ? (uint64_t)a.mtiles * a.ntiles : a.ntiles;
    const uint64_t groups = splits > 1 ? (uint64_t)splits : a.mtiles;
    const uint64_t nblocks = cdiv(groups, 8) * 8 * members;
    if (nblocks > 0x7fffffffull) return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gemm: more than 2^31 tiles");
    char tag[56];
    snprintf(tag, sizeof(tag), "%c%c %dx%d %lldx%lldx%lld f32", ta ? 'T' : 'N', tb ? 'T' : 'N', bm, DIRECT_BN, (long long)a.M,
             (long long)a.N, (long long)a.K);
    dim3 grid((unsigned)nblocks), block(64 * waves);
    const size_t lds_bytes = (size_t)DIRECT_STAGES * (bm + DIRECT_BN) * DIRECT_BK * sizeof(float);
    const bool gather = a.a_row_index != nullptr;
#define SGNN_DIRECT_CASE_BM(BM_, W_, TN_, TA_, TB_, G_)                                                                 \
    if (bm == BM_ && ta == TA_ && tb == TB_ && gather == G_) {                                                          \
        static bool attr_set = false;                                                                                   \
        if (!attr_set) {                                                                                                \
            SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_direct_kernel<BM_, W_, TN_, TA_, TB_, G_>), \
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));                 \
            attr_set = true;                                                                                            \
        }                                                                                                               \
        SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_direct_kernel<BM_, W_, TN_, TA_, TB_, G_>), grid, block, lds_bytes, st, a); \
        return SGNN_OK;                                                                                                 \
    }
#define SGNN_DIRECT_CASE(TA_, TB_, G_) SGNN_DIRECT_CASE_BM(DIRECT_BM, DIRECT_WAVES, 2, TA_, TB_, G_)
    SGNN_DIRECT_CASE_BM(128, 8, 1, true, false, false)
    SGNN_DIRECT_CASE_BM(128, 8, 1, true, false, true)
    SGNN_DIRECT_CASE(false, false, false)
    SGNN_DIRECT_CASE(false, true, false)
    SGNN_DIRECT_CASE(true, false, false)
    SGNN_DIRECT_CASE(false, false, true)
    SGNN_DIRECT_CASE(false, true, true)
    SGNN_DIRECT_CASE(true, false, true)
#undef SGNN_DIRECT_CASE_BM
#undef SGNN_DIRECT_CASE
    return SGNN_OK;
}

// ---------------------------------------------------------------------------------------------
// bf16 path, tall A and a small B (K <= 256, N <= 256: the layer transform and the feature
// gradient of a mini-batch with hundreds of thousands of rows).  The product is bound by reading
// A and writing C once, so the kernel is built around that stream:
//  - B is rounded to bfloat16 once per workgroup and stays in LDS ([n][K rounded up + 8]) for the
//    whole launch; workgroups are persistent and walk blocks of 256 rows;
//  - a wavefront owns 32 rows of the block and all N columns.  It reads its rows in slices of 32
//    along K with full 128-byte row segments, up to four slices ahead in registers, turns a
//    slice into MFMA operand order through an LDS patch of its own (no workgroup barrier), and
//    keeps the 32 x N accumulators in registers until the row block is complete.
// ---------------------------------------------------------------------------------------------
constexpr int SKINNY_WAVES = 8;
constexpr int SKINNY_PATCH = 32 * 40;   // 16-bit elements of a wavefront's patch: [32][32 + 8]

inline size_t skinny_lds_bytes(int nt8, int kp)
{
    return ((size_t)32 * nt8 * kp + (size_t)SKINNY_WAVES * SKINNY_PATCH) * 2 + (size_t)2 * 32 * nt8 * sizeof(float);
}

// value of lane k (0..3) of the caller's quad of lanes, in every lane of the quad (DPP quad_perm, no LDS)
__device__ __forceinline__ uint32_t quad_broadcast(uint32_t v, int k)
{
    switch (k) {
    case 0: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x00, 0xF, 0xF, false);
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x55, 0xF, 0xF, false);
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xAA, 0xF, 0xF, false);
    default: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xFF, 0xF, 0xF, false);
    }
}

// Optional layer tail fused into the epilogue (Sec. III-B Eqs. 7-10; Sec. V "Kernel Fusion"): a wavefront
// owns whole rows of the result, so the RMS of a row is a reduction inside the wavefront and
// Y = dropout(relu(rmsnorm(Z))) + R is written next to Z without reading Z back.
struct skinny_tail {
    const float *gamma;   // [N] or NULL
    float eps;
    const float *R; int64_t ldr;   // residual input or NULL
    float *Y; int64_t ldy;
    float *inv_rms;       // [M] or NULL
    uint32_t thr; float scale; uint32_t k0, k1, c2, c3;   // dropout: keep iff word >= thr (thr = 0: none)
};

// NT8 = column tiles of 32 (N <= 32 NT8), S = slices of 32 along the reduction (K <= 32 S).  Both are
// compile-time so that the order of every load and store of a row block is fixed: the waits on the
// slices in flight then count exactly the operations issued after them.
// one element of the mask matrix (fp32 or bfloat16 storage): is it positive?
__device__ __forceinline__ bool skinny_mask_at(const gemm_args &a, int64_t row, int64_t col)
{
    if (a.m_bf16) return (int16_t) reinterpret_cast<const u16 *>(a.mask)[row * a.ldm + col] > 0;
    return a.mask[row * a.ldm + col] > 0.f;
}

// The four ballots of a 16-byte mask chunk (all lanes take part: no divergence around them), and of those the word
// that holds the bits of this lane's column: e = li % 4.
__device__ __forceinline__ uint64_t skinny_mask_word(const f32x4 &m, int li)
{
    const uint64_t b0 = __ballot(m[0] > 0.f), b1 = __ballot(m[1] > 0.f), b2 = __ballot(m[2] > 0.f), b3 = __ballot(m[3] > 0.f);
    const uint64_t w01 = (li & 1) ? b1 : b0, w23 = (li & 1) ? b3 : b2;
    return (li & 2) ? w23 : w01;
}

// MASK: the result is zeroed where a.mask (M x N, 16-byte chunks) is not positive.  That variant reads the mask
// tile by tile during the epilogue and needs registers for it: it does not fetch the next row block's first
// slices behind the current one's last multiplies but after the epilogue.
// ABF: A is stored as bfloat16 (lda in elements, rows 8-byte aligned): a lane's chunk of four reduction values is 8 bytes
// and goes to the LDS patch as it is.  a.c_bf16 (a run-time switch of the epilogue): C is stored as bfloat16, rounded to
// nearest even; neighbouring lanes swap one value of every row pair so that a lane writes two adjacent columns at once.
// a.m_bf16: the mask is stored as bfloat16.
template <int NT8, int S, bool TAIL, bool MASK, bool ABF = false>
__global__ __launch_bounds__(64 * SKINNY_WAVES) void gemm_skinny_bf16_kernel(gemm_args a, int tb, uint32_t n_rowblocks,
                                                                             skinny_tail tl)
{
    constexpr int D = S == 8 ? 4 : (S == 6 ? 3 : S);   // slices in flight; divides S
    constexpr int KP = 32 * S + 8;                      // row length of B in LDS
    constexpr int NP = 32 * NT8;
    extern __shared__ __attribute__((aligned(16))) unsigned char skinny_smem[];
    u16 *LB = reinterpret_cast<u16 *>(skinny_smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    u16 *LA = LB + NP * KP + wave * SKINNY_PATCH;
    const int K = (int)a.K, N = (int)a.N;

    // B -> LDS as bfloat16, zero beyond N and K; eight loads in flight per thread
    constexpr int NTHR = 64 * SKINNY_WAVES;
    if (a.alignedB && (tb ? K : N) % 4 == 0) {
        constexpr int CHUNKS = NP * 8 * S;   // 16-byte chunks of the padded B
        for (int base = threadIdx.x; base < CHUNKS; base += 8 * NTHR) {
            f32x4 x[8];
            int n[8], k[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NTHR;
                if (tb) {   // B given N x K: a chunk is four k of one n
                    n[u] = idx / (8 * S);
                    k[u] = 4 * (idx % (8 * S));
                } else {    // B given K x N: a chunk is four n of one k; 8 chunks x 8 k per wavefront load
                    const int rest = idx >> 6;
                    n[u] = 32 * (rest % NT8) + 4 * (idx & 7);
                    k[u] = 8 * (rest / NT8) + ((idx >> 3) & 7);
                }
                x[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (idx < CHUNKS && n[u] < N && k[u] < K)
                    x[u] = *reinterpret_cast<const f32x4 *>(tb ? a.B + (int64_t)n[u] * a.ldb + k[u] : a.B + (int64_t)k[u] * a.ldb + n[u]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (base + u * NTHR >= CHUNKS) continue;
                if (tb) {
                    uint2 w;
                    w.x = (uint32_t)to_bf16_bits(x[u][0]) | ((uint32_t)to_bf16_bits(x[u][1]) << 16);
                    w.y = (uint32_t)to_bf16_bits(x[u][2]) | ((uint32_t)to_bf16_bits(x[u][3]) << 16);
                    *reinterpret_cast<uint2 *>(LB + n[u] * KP + k[u]) = w;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) LB[(n[u] + c) * KP + k[u]] = to_bf16_bits(x[u][c]);
                }
            }
        }
    } else {
        for (int base = threadIdx.x; base < NP * 32 * S; base += 8 * NTHR) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NTHR;
                const int n = tb ? idx / (32 * S) : idx % NP, k = tb ? idx % (32 * S) : idx / NP;
                x[u] = 0.f;
                if (idx < NP * 32 * S && n < N && k < K) x[u] = tb ? a.B[(int64_t)n * a.ldb + k] : a.B[(int64_t)k * a.ldb + n];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * NTHR;
                const int n = tb ? idx / (32 * S) : idx % NP, k = tb ? idx % (32 * S) : idx / NP;
                if (idx < NP * 32 * S) LB[n * KP + k] = to_bf16_bits(x[u]);
            }
        }
    }
    float *Lbias = reinterpret_cast<float *>(LB + NP * KP + SKINNY_WAVES * SKINNY_PATCH);   // kept in LDS: no load in the stream
    float *Lgamma = Lbias + NP;
    for (int n = threadIdx.x; n < NP; n += 64 * SKINNY_WAVES) {
        Lbias[n] = (a.bias && n < N) ? a.bias[n] : 0.f;
        if (TAIL) Lgamma[n] = (tl.gamma && n < N) ? tl.gamma[n] : 1.f;
    }
    __syncthreads();

    f32x16 acc[NT8];
#pragma unroll
    for (int j = 0; j < NT8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    const bool relu = a.relu != 0;

    // loads: lane -> rows lr + 8 v (v = 0..3) of the wavefront's 32, 16-byte chunk kc of the slice
    const int lr = lane >> 3, kc = lane & 7;
    const int last_chunk = (K - 1) & ~3;
    using ring_t = typename std::conditional<ABF, uint2, f32x4>::type;   // a lane's chunk of four reduction values
    const float *rowp[4];        // with ABF: really 16-bit elements, addressed through elem()
    auto row_pointers = [&](uint32_t rb) {   // a row block past the end repeats the last one (loaded, never used)
        rb = min(rb, n_rowblocks - 1);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int64_t row = min((int64_t)rb * (32 * SKINNY_WAVES) + wave * 32 + lr + 8 * v, a.M - 1);
            if (a.a_row_index) row = a.a_row_index[row];
            if constexpr (ABF) rowp[v] = reinterpret_cast<const float *>(reinterpret_cast<const u16 *>(a.A) + row * a.lda);
            else rowp[v] = a.A + row * a.lda;
        }
    };
    auto issue = [&](ring_t (&r)[4], int slice) {
        const int k = min(32 * slice + 4 * kc, last_chunk);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if constexpr (ABF) r[v] = *reinterpret_cast<const uint2 *>(reinterpret_cast<const u16 *>(rowp[v]) + k);
            else r[v] = *reinterpret_cast<const f32x4 *>(rowp[v] + k);
        }
    };
    auto stage = [&](ring_t (&r)[4], int slice) {
        const int k = 32 * slice + 4 * kc;
        if constexpr (ABF) {
            if (k + 4 > K) {     // the ragged end of the reduction: zero the 16-bit values at or beyond K
                const int left = K - k;      // values of the chunk that count: below 4, possibly <= 0
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    r[v].x = left <= 0 ? 0u : (left == 1 ? (r[v].x & 0xffffu) : r[v].x);
                    r[v].y = left <= 2 ? 0u : (left == 3 ? (r[v].y & 0xffffu) : r[v].y);
                }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) *reinterpret_cast<uint2 *>(LA + (lr + 8 * v) * 40 + 4 * kc) = r[v];
        } else {
            if (k + 4 > K) {     // the ragged end of the reduction
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (k + e >= K) r[v][e] = 0.f;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                uint2 w;
                w.x = (uint32_t)to_bf16_bits(r[v][0]) | ((uint32_t)to_bf16_bits(r[v][1]) << 16);
                w.y = (uint32_t)to_bf16_bits(r[v][2]) | ((uint32_t)to_bf16_bits(r[v][3]) << 16);
                *reinterpret_cast<uint2 *>(LA + (lr + 8 * v) * 40 + 4 * kc) = w;
            }
        }
    };
    auto multiply = [&](int slice) {
        bf16x8 av[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) av[ks] = *reinterpret_cast<const bf16x8 *>(LA + li * 40 + 16 * ks + 8 * kh);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < NT8; ++j) {
                const bf16x8 bv = *reinterpret_cast<const bf16x8 *>(LB + (32 * j + li) * KP + 32 * slice + 16 * ks + 8 * kh);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ks], bv, acc[j], 0, 0, 0);
            }
    };

    ring_t ring[D][4];
    row_pointers(blockIdx.x);
#pragma unroll
    for (int u = 0; u < D; ++u) issue(ring[u], u);
    for (uint32_t rb = blockIdx.x; rb < n_rowblocks; rb += gridDim.x) {
#pragma unroll
        for (int sl = 0; sl < S; ++sl) {
            stage(ring[sl % D], sl);
            if (!MASK || sl + D < S) {
                if (sl + D == S) row_pointers(rb + gridDim.x);       // the loads from here on belong to the next row block
                issue(ring[sl % D], (sl + D) % S);
            }
            multiply(sl);
        }
        // the row block is complete: write it
        const int64_t wrow = (int64_t)rb * (32 * SKINNY_WAVES) + wave * 32;
        const int64_t row0 = wrow + 4 * kh;   // the lane's first row
        float *cl = a.C + row0 * a.ldc + li;      // fp32 result; a bfloat16 result is addressed in the branches below
        if (wrow + 32 <= a.M) {
            // The mask (zero the result where another M x N matrix is not positive: the ReLU backward of the layer
            // below) is read the way A is: 16 bytes a lane, lane (lr, kc) takes columns 4 kc .. 4 kc + 3 of rows
            // lr + 8 v of a 32-column tile, one tile ahead of the stores.  Four ballots per load turn a tile's mask
            // into sixteen wave-uniform 64-bit words (bit 8 lr + kc of word (v, e) = row lr + 8 v, column 4 kc + e),
            // from which every lane picks the bits of its own sixteen elements.  Read element by element in the
            // accumulator layout (4 bytes a lane, a load in front of every store) the mask tripled the kernel's time.
            constexpr bool vmask = MASK;
            f32x4 mreg0, mreg1, mreg2, mreg3;                // with a bfloat16 mask: 8 bytes a lane, in .x and .y as bit patterns
            uint64_t ws0 = 0, ws1 = 0, ws2 = 0, ws3 = 0;      // per v: the word (v, e = li % 4) of the current tile
            const bool m16 = a.m_bf16 != 0, c16 = a.c_bf16 != 0;
            const int64_t m8 = 8 * a.ldm;
#define SKINNY_MASK_ISSUE(j_)                                                                                   \
    {                                                                                                          \
        const int64_t mo_ = (wrow + lr) * a.ldm + min((int64_t)(32 * (j_) + 4 * kc), (int64_t)(N - 4)); /* N is a multiple of 4 here */ \
        if (m16) {                                                                                             \
            const u16 *mp_ = reinterpret_cast<const u16 *>(a.mask) + mo_;                                      \
            const uint2 q0_ = *reinterpret_cast<const uint2 *>(mp_), q1_ = *reinterpret_cast<const uint2 *>(mp_ + m8),          \
                        q2_ = *reinterpret_cast<const uint2 *>(mp_ + 2 * m8), q3_ = *reinterpret_cast<const uint2 *>(mp_ + 3 * m8); \
            mreg0 = widen_bf16x4(q0_); mreg1 = widen_bf16x4(q1_); mreg2 = widen_bf16x4(q2_); mreg3 = widen_bf16x4(q3_);       \
        } else {                                                                                               \
            const float *mp_ = a.mask + mo_;                                                                   \
            mreg0 = *reinterpret_cast<const f32x4 *>(mp_);                                                     \
            mreg1 = *reinterpret_cast<const f32x4 *>(mp_ + m8);                                                \
            mreg2 = *reinterpret_cast<const f32x4 *>(mp_ + 2 * m8);                                            \
            mreg3 = *reinterpret_cast<const f32x4 *>(mp_ + 3 * m8);                                            \
        }                                                                                                      \
    }
            if constexpr (vmask) SKINNY_MASK_ISSUE(0)
#pragma unroll
            for (int j = 0; j < NT8; ++j) {
                if constexpr (vmask) {
                    ws0 = skinny_mask_word(mreg0, li);
                    ws1 = skinny_mask_word(mreg1, li);
                    ws2 = skinny_mask_word(mreg2, li);
                    ws3 = skinny_mask_word(mreg3, li);
                    if (j + 1 < NT8) SKINNY_MASK_ISSUE(j + 1)
                }
                if (32 * j + li < N) {
                    const float bj = Lbias[32 * j + li];
                    float zv[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rr = 8 * (r / 4) + (r % 4);
                        float z = acc[j][r] + bj;
                        z = relu ? fmaxf(z, 0.f) : z;
                        if constexpr (vmask) {
                            // row 8 (r / 4) + 4 kh + r % 4 of the wavefront's 32: v = r / 4, lr = 4 kh + r % 4; column li: kc = li / 4, e = li % 4
                            const uint64_t w = (r / 4) == 0 ? ws0 : ((r / 4) == 1 ? ws1 : ((r / 4) == 2 ? ws2 : ws3));
                            z = ((w >> (8 * (4 * kh + (r % 4)) + (li >> 2))) & 1ull) ? z : 0.f;
                        } else if (a.mask) z = skinny_mask_at(a, row0 + rr, 32 * j + li) ? z : 0.f;
                        zv[r] = z;
                    }
                    if (!c16) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) cl[(int64_t)(8 * (r / 4) + (r % 4)) * a.ldc + 32 * j] = zv[r];
                    } else if (a.c_pair) {
                        // bfloat16 result, two adjacent columns a lane: of every pair of rows (r, r + 1) the even lane
                        // takes row r and the odd lane row r + 1, each receiving its neighbour's value of that row
                        u16 *cp = reinterpret_cast<u16 *>(a.C) + (row0 + (li & 1)) * a.ldc + 32 * j + (li & ~1);
#pragma unroll
                        for (int r = 0; r < 16; r += 2) {
                            const float send = (li & 1) ? zv[r] : zv[r + 1];
                            const float recv = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
                            const float lo = (li & 1) ? recv : zv[r], hi = (li & 1) ? zv[r + 1] : recv;
                            *reinterpret_cast<uint32_t *>(cp + (int64_t)(8 * (r / 4) + (r % 4)) * a.ldc) =
                                (uint32_t)to_bf16_bits(lo) | ((uint32_t)to_bf16_bits(hi) << 16);
                        }
                    } else {
                        u16 *cp = reinterpret_cast<u16 *>(a.C) + row0 * a.ldc + 32 * j + li;
#pragma unroll
                        for (int r = 0; r < 16; ++r) cp[(int64_t)(8 * (r / 4) + (r % 4)) * a.ldc] = to_bf16_bits(zv[r]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NT8; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rr = 8 * (r / 4) + (r % 4);
                    float z = acc[j][r] + Lbias[32 * j + li];
                    z = relu ? fmaxf(z, 0.f) : z;
                    if (32 * j + li < N && row0 + rr < a.M) {
                        if (a.mask) z = skinny_mask_at(a, row0 + rr, 32 * j + li) ? z : 0.f;
                        if (a.c_bf16) reinterpret_cast<u16 *>(a.C)[(row0 + rr) * a.ldc + 32 * j + li] = to_bf16_bits(z);
                        else cl[(int64_t)rr * a.ldc + 32 * j] = z;
                    }
                }
        }
#undef SKINNY_MASK_ISSUE
        if constexpr (TAIL) {
            // 1 / rms of the lane's sixteen rows: squares summed over its columns, then over the 32 lanes that
            // share those rows (xor distances below 32 stay inside the half wavefront)
            float ir[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) ir[r] = 0.f;
#pragma unroll
            for (int j = 0; j < NT8; ++j) {
                if (32 * j + li < N) {
                    const float bj = Lbias[32 * j + li];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float z = acc[j][r] + bj;
                        ir[r] = fmaf(z, z, ir[r]);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) ir[r] += __shfl_xor(ir[r], o);
                ir[r] = 1.f / sqrtf(ir[r] / (float)N + tl.eps);                     // Eq. 7
                const int64_t row = row0 + 8 * (r / 4) + (r % 4);
                if (tl.inv_rms && li == 0 && row < a.M) tl.inv_rms[row] = ir[r];
            }
#pragma unroll
            for (int j = 0; j < NT8; ++j) {
                const int col = 32 * j + li;
                const float bj = Lbias[col], gj = Lgamma[col];
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    // dropout words: the four lanes of a quad hold four consecutive columns = one Philox block per
                    // row; lane k of the quad evaluates the block of row 8 rg + k, the quad then shares the four
                    philox_out o = {0u, 0u, 0u, 0u};
                    if (tl.thr) {
                        const uint64_t e = (uint64_t)(row0 + 8 * rg + (li & 3)) * (uint64_t)N + (uint64_t)(32 * j + (li & ~3));
                        o = philox4x32_10((uint32_t)(e >> 2), (uint32_t)(e >> 34), tl.c2, tl.c3, tl.k0, tl.k1);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int r = 4 * rg + k;
                        const int64_t row = row0 + 8 * rg + k;
                        float keep = 1.f;
                        if (tl.thr) {
                            const uint32_t w0 = quad_broadcast(o.w0, k);
                            const uint32_t w1 = quad_broadcast(o.w1, k);
                            const uint32_t w2 = quad_broadcast(o.w2, k);
                            const uint32_t w3 = quad_broadcast(o.w3, k);
                            const uint32_t w = (li & 2) ? ((li & 1) ? w3 : w2) : ((li & 1) ? w1 : w0);
                            keep = w >= tl.thr ? tl.scale : 0.f;
                        }
                        if (col < N && row < a.M) {
                            const float n = gj * (acc[j][r] + bj) * ir[r];
                            const float res = tl.R ? tl.R[row * tl.ldr + col] : 0.f;
                            tl.Y[row * tl.ldy + col] = fmaxf(n, 0.f) * keep + res;   // Eqs. 8-10
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < NT8; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
        if constexpr (MASK) {
            row_pointers(rb + gridDim.x);
#pragma unroll
            for (int u = 0; u < D; ++u) issue(ring[u], u);
        }
    }
}

template <int NT8, int S, bool TAIL>
int launch_skinny_ns(sgnn_ctx *ctx, const gemm_args &a, int tb, const skinny_tail &tl, hipStream_t st)
{
    const size_t lds = skinny_lds_bytes(NT8, 32 * S + 8);
    static bool attr_set = false;
    if (!attr_set) {
        SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_bf16_kernel<NT8, S, TAIL, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        if constexpr (!TAIL)
            SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_bf16_kernel<NT8, S, false, true>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    const uint32_t n_rowblocks = (uint32_t)cdiv(a.M, 32 * SKINNY_WAVES);
    char tag[56];
    const bool vmask = !TAIL && a.mask && a.vecM;      // the mask in chunks of four; else element by element
    snprintf(tag, sizeof(tag), "N%c skinny%s %lldx%lldx%lld bf16 a=%d c=%d%s", tb ? 'T' : 'N', TAIL ? "+tail" : "", (long long)a.M,
             (long long)a.N, (long long)a.K, a.a_bf16 ? 2 : 4, a.c_bf16 ? 2 : 4, a.mask ? (a.m_bf16 ? " mask m=2" : " mask m=4") : "");
    const dim3 grid(std::min<uint32_t>(n_rowblocks, 256)), block(64 * SKINNY_WAVES);
    if constexpr (!TAIL) {
        if (a.a_bf16 && vmask) {
            static bool attr16m = false;
            if (!attr16m) {
                SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_bf16_kernel<NT8, S, false, true, true>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
                attr16m = true;
            }
            SGNN_LAUNCH(ctx, st, "gemm_skinny_bf16_kernel", tag, (gemm_skinny_bf16_kernel<NT8, S, false, true, true>), grid, block, lds,
                        st, a, tb, n_rowblocks, tl);
            return SGNN_OK;
        }
        if (a.a_bf16) {
            static bool attr16 = false;
            if (!attr16) {
                SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_bf16_kernel<NT8, S, false, false, true>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
                attr16 = true;
            }
            SGNN_LAUNCH(ctx, st, "gemm_skinny_bf16_kernel", tag, (gemm_skinny_bf16_kernel<NT8, S, false, false, true>), grid, block, lds,
                        st, a, tb, n_rowblocks, tl);
            return SGNN_OK;
        }
        if (vmask) {
            SGNN_LAUNCH(ctx, st, "gemm_skinny_bf16_kernel", tag, (gemm_skinny_bf16_kernel<NT8, S, false, true>), grid, block, lds, st, a,
                        tb, n_rowblocks, tl);
            return SGNN_OK;
        }
    }
    SGNN_LAUNCH(ctx, st, "gemm_skinny_bf16_kernel", tag, (gemm_skinny_bf16_kernel<NT8, S, TAIL, false>), grid, block, lds, st, a, tb,
                n_rowblocks, tl);
    return SGNN_OK;
}

template <int NT8, bool TAIL>
int launch_skinny_n(sgnn_ctx *ctx, const gemm_args &a, int tb, const skinny_tail &tl, hipStream_t st)
{
    const int s2 = (int)((a.K + 63) / 64);   // slices, rounded up to an even count
    switch (s2) {
    case 1: return launch_skinny_ns<NT8, 2, TAIL>(ctx, a, tb, tl, st);
    case 2: return launch_skinny_ns<NT8, 4, TAIL>(ctx, a, tb, tl, st);
    case 3: return launch_skinny_ns<NT8, 6, TAIL>(ctx, a, tb, tl, st);
    default: return launch_skinny_ns<NT8, 8, TAIL>(ctx, a, tb, tl, st);
    }
}

template <bool TAIL>
int launch_skinny_t(sgnn_ctx *ctx, const gemm_args &a, int tb, const skinny_tail &tl, hipStream_t st)
{
    switch ((int)((a.N + 63) / 64)) {   // column tiles, rounded up to an even count
    case 1: return launch_skinny_n<2, TAIL>(ctx, a, tb, tl, st);
    case 2: return launch_skinny_n<4, TAIL>(ctx, a, tb, tl, st);
    case 3: return launch_skinny_n<6, TAIL>(ctx, a, tb, tl, st);
    default: return launch_skinny_n<8, TAIL>(ctx, a, tb, tl, st);
    }
}

int launch_skinny(sgnn_ctx *ctx, const gemm_args &a, int tb, hipStream_t st)
{
    const skinny_tail none = {};
    return launch_skinny_t<false>(ctx, a, tb, none, st);
}

// ---------------------------------------------------------------------------------------------
// Thin products of the classifier layer (one dimension of 32 or less), fp32.  At these shapes the tile
// kernels are bound by the latency of their few staging rounds, not by arithmetic or bandwidth: here
// every operand goes from global memory straight into the register layout of v_mfma_f32_32x32x2_f32
// (lane (li, kh) supplies element (li, kh) of a 32 x 2 operand), with all loads of a wavefront in
// flight at once and several wavefronts per SIMD.
//
// gemm_thin_tn_kernel: C = A^T B, A given K x M, B given K x N with N <= 32, K long (the weight
// gradient of the classifier layer, Eq. 24).  A workgroup takes 128 rows of the result and one
// reduction range, split evenly over its eight wavefronts (two per SIMD: one multiplies while the
// other's loads are in flight).  Per pair of reduction steps a lane loads 16 bytes of A (its four
// columns 4 li .. 4 li + 3 of row k + kh: one value for each of four 32-row tiles, whose row i is
// thus column 4 i + j of A) and one value of B.  The eight partial results are added in LDS in a
// fixed order and written as one split-K partial product (the caller sums those with
// splitk_reduce_kernel); the column sums of B go the same way.
// ---------------------------------------------------------------------------------------------
constexpr int THIN_WAVES = 8;    // wavefronts per workgroup
constexpr int THIN_PAIRS = 16;   // pairs of reduction steps per pass
template <bool GATHER>
__global__ __launch_bounds__(64 * THIN_WAVES) void gemm_thin_tn_kernel(gemm_args a)
{
    constexpr int PAIRS = THIN_PAIRS;
    __shared__ __attribute__((aligned(16))) float red[4][128 * 32];
    const gemm_tile tb_ = tile_of_block(a);
    if (!tb_.valid) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 31, kh = lane >> 5;
    const int64_t m0 = (int64_t)tb_.bx * 128;
    const int64_t kbeg = (int64_t)tb_.bz * a.k_per_split;
    const int64_t kend = min(a.K, kbeg + a.k_per_split);
    const int64_t kw = a.k_per_split / THIN_WAVES;          // a multiple of 2
    const int64_t k0 = kbeg + wave * kw, k1 = min(kend, k0 + kw);
    const int64_t mcol = m0 + 4 * li;
    const bool mok = mcol < a.M, nok = li < a.N;
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    float cs = 0.f;
    for (int64_t k = k0; k < k1; k += 2 * PAIRS) {
        // Every load is issued unconditionally at a clamped (valid) address and zeroed afterwards where it is
        // out of range (a load under a branch would be waited for before the next one is issued), and all
        // loads of a pass are requested before its first multiply (the scheduling barrier keeps them there).
        // A second register set that prefetches the next pass measured slower: the other wavefront of the
        // SIMD already multiplies while this one waits.
        f32x4 av[PAIRS];
        float bv[PAIRS];
        int64_t ar[PAIRS];
#pragma unroll
        for (int s = 0; s < PAIRS; ++s) {
            const int64_t kc = min(k + 2 * s + kh, k1 - 1);
            ar[s] = GATHER ? (int64_t)a.a_row_index[kc] : kc;
        }
#pragma unroll
        for (int s = 0; s < PAIRS; ++s) {
            av[s] = *reinterpret_cast<const f32x4 *>(a.A + ar[s] * a.lda + (mok ? mcol : 0));
            bv[s] = a.B[min(k + 2 * s + kh, k1 - 1) * a.ldb + (nok ? li : 0)];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < PAIRS; ++s) {
            const bool ok = k + 2 * s + kh < k1;
            const float y = (ok && nok) ? bv[s] : 0.f;
            cs += y;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x = (ok && mok) ? av[s][j] : 0.f;
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[j], 0, 0, 0);
            }
        }
    }
    // acc[j][r] is the element (row 4 rho + j of the 128, column li); tree sum over the wavefronts in LDS:
    // (w, w + 4) -> w, then (w, w + 2) -> w, then (0, 1) -> 0, each a fixed order of additions
#pragma unroll
    for (int half = THIN_WAVES / 2; half >= 1; half >>= 1) {
        if (wave >= half && wave < 2 * half) {
            float *dst = red[wave - half];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(4 * (8 * (r / 4) + 4 * kh + (r % 4)) + j) * 32 + li] = acc[j][r];
        }
        __syncthreads();
        if (wave < half) {
            const float *src = red[wave];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] += src[(4 * (8 * (r / 4) + 4 * kh + (r % 4)) + j) * 32 + li];
        }
        __syncthreads();
    }
    cs += __shfl_xor(cs, 32);
    if (a.colsum && tb_.bx == 0) {
        float *cs_red = red[0];       // free again: the tree sum ended with a barrier
        if (kh == 0) cs_red[wave * 32 + li] = cs;
        __syncthreads();
        if (wave == 0 && kh == 0 && nok) {
            float t = 0.f;
#pragma unroll
            for (int w = 0; w < THIN_WAVES; ++w) t += cs_red[w * 32 + li];
            a.colsum[(int64_t)tb_.bz * a.N + li] = t;
        }
    }
    if (wave == 0 && nok) {
        float *out = a.partial + (int64_t)tb_.bz * a.M * a.N;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + 4 * (8 * (r / 4) + 4 * kh + (r % 4)) + j;
                if (row < a.M) out[row * a.N + li] = acc[j][r];
            }
    }
}

// gemm_smallk_nt_kernel: C = epilogue(A B^T), A given M x K, B given N x K, K <= 64 a multiple of 4
// (the gradient with respect to the input of a narrow layer, Eq. 22).  A wavefront computes 32 rows
// by 32 columns (eight wavefronts per SIMD in flight: with 32 x 64 the registers allowed three, and the
// last of 1 1/3 rounds of wavefronts ran on a nearly empty chip); the four wavefronts of a workgroup
// share the rows.  The reduction index is dealt to the two halves of the wavefront in two contiguous
// runs (lanes kh = 0 take k < 4 Q, the others the rest: any pairing of reduction steps gives the same
// sum up to rounding order), so that a lane reads its operand rows 16 bytes at a time with no element
// unused.  Q = 16-byte chunks per lane and row.
constexpr int SMALLK_TW = 1;    // 32-column tiles per wavefront
template <int Q>
__global__ __launch_bounds__(256) void gemm_smallk_nt_kernel(gemm_args a)
{
    constexpr int TW = SMALLK_TW;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 31, kh = lane >> 5;
    const int64_t r0 = (int64_t)blockIdx.x * 32;
    const int64_t n0 = (int64_t)blockIdx.y * (128 * TW) + 32 * TW * wave;
    if (n0 >= a.N) return;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // every load is issued unconditionally at a clamped (valid) address and zeroed afterwards where it is out of
    // range: a load under a branch would be waited for before the next one is issued
    f32x4 av[Q], bv[TW][Q];
    const int64_t arow = min(r0 + li, a.M - 1);
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int64_t k = 4 * (Q * kh + q);
        const bool kok = k < a.K;
        const int64_t kc = kok ? k : 0;
        const f32x4 x = *reinterpret_cast<const f32x4 *>(a.A + arow * a.lda + kc);
        av[q] = kok ? x : zero4;           // rows beyond M compute values that are never stored
#pragma unroll
        for (int t = 0; t < TW; ++t) {
            const int64_t n = min(n0 + 32 * t + li, a.N - 1);
            const f32x4 y = *reinterpret_cast<const f32x4 *>(a.B + n * a.ldb + kc);
            bv[t][q] = kok ? y : zero4;    // as are columns beyond N
        }
    }
    // the mask values of the lane's results, requested before the multiplies
    float mk[TW][16];
    if (a.mask) {
#pragma unroll
        for (int t = 0; t < TW; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = min(r0 + 8 * (r / 4) + 4 * kh + (r % 4), a.M - 1), col = min(n0 + 32 * t + li, a.N - 1);
                mk[t][r] = a.mask[row * a.ldm + col];
            }
    }
    f32x16 acc[TW];
#pragma unroll
    for (int t = 0; t < TW; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < TW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][e], bv[t][q][e], acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const int64_t col = n0 + 32 * t + li;
        if (col >= a.N) continue;
        const float bj = a.bias ? a.bias[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = r0 + 8 * (r / 4) + 4 * kh + (r % 4);
            if (row >= a.M) continue;
            float z = acc[t][r] + bj;
            if (a.relu) z = fmaxf(z, 0.f);
            if (a.mask && !(mk[t][r] > 0.f)) z = 0.f;
            a.C[row * a.ldc + col] = z;
        }
    }
}

// Sum of the split-K partial products in a fixed order (bit-reproducible).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int splits, int64_t MN,
                                                            int64_t N, float *__restrict__ C, int64_t ldc,
                                                            const float *__restrict__ cs_partial, float *__restrict__ cs_out)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) {
        // the threads behind the matrix add up the column sums of B, split by split
        const int64_t col = i - MN;
        if (cs_partial && col < N) {
            // eight loads in flight, the same fixed order of additions every time
            float t = 0.f;
            int z = 0;
            for (; z + 8 <= splits; z += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = cs_partial[(int64_t)(z + u) * N + col];
#pragma unroll
                for (int u = 0; u < 8; ++u) t += x[u];
            }
            for (; z < splits; ++z) t += cs_partial[(int64_t)z * N + col];
            cs_out[col] = t;
        }
        return;
    }
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
int launch_cfg(sgnn_ctx *ctx, int ta, int tb, int bf16, gemm_args a, int splits, hipStream_t st)
{
    a.mtiles = (uint32_t)cdiv(a.M, BM);
    a.ntiles = (uint32_t)cdiv(a.N, BN);
    a.splits = (uint32_t)splits;
    const uint64_t members = splits > 1 ? (uint64_t)a.mtiles * a.ntiles : a.ntiles;
    const uint64_t groups = splits > 1 ? (uint64_t)splits : a.mtiles;
    const uint64_t nblocks = cdiv(groups, 8) * 8 * members;
    if (nblocks > 0x7fffffffull) return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gemm: more than 2^31 tiles");
    dim3 grid((unsigned)nblocks), block(256);
    char tag[56];
    // fast path: every 16-byte chunk wholly inside or outside the operands
    const int64_t a_contig = ta ? a.M : a.K, b_contig = tb ? a.K : a.N;
    const bool fast = a.alignedA && a.alignedB && a_contig % 4 == 0 && b_contig % 4 == 0 && a_contig >= 4 && b_contig >= 4 &&
                      a.K >= 1 && a.M >= 1 && a.N >= 1;
    if (fast && !(ta && tb)) {
        snprintf(tag, sizeof(tag), "%c%c %dx%d %lldx%lldx%lld %s%s", ta ? 'T' : 'N', tb ? 'T' : 'N', BM, BN, (long long)a.M,
                 (long long)a.N, (long long)a.K, bf16 ? "bf16" : "f32", a.a_bf16 ? (a.b_bf16 ? " a=2 b=2" : " a=2") : (a.b_bf16 ? " b=2" : ""));
#define SGNN_GEMM_FAST(TA_, TB_, BF_)                                                                              \
    if (ta == TA_ && tb == TB_ && bf16 == BF_) {                                                                   \
        SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, TA_, TB_, BF_>), grid, block, 0, st, a); \
        return SGNN_OK;                                                                                            \
    }
        if (a.a_bf16 || a.b_bf16) {      // the launcher sends only A^T B with bf16 operands here in this storage
            if (a.a_bf16 && a.b_bf16)
                SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, true, false, true, true, true>), grid, block, 0, st, a);
            else if (a.a_bf16)
                SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, true, false, true, true, false>), grid, block, 0, st, a);
            else
                SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, (gemm_fast_kernel<BM, BN, WM, WN, true, false, true, false, true>), grid, block, 0, st, a);
            return SGNN_OK;
        }
        SGNN_GEMM_FAST(false, false, false)
        SGNN_GEMM_FAST(false, true, false)
        SGNN_GEMM_FAST(true, false, false)
        SGNN_GEMM_FAST(false, false, true)
        SGNN_GEMM_FAST(false, true, true)
        SGNN_GEMM_FAST(true, false, true)
#undef SGNN_GEMM_FAST
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


// bfloat16 <-> fp32 copies of a matrix (rows x cols), for the products whose kernel does not read or write the
// 16-bit storage itself; src rows optionally gathered through ridx.
__global__ __launch_bounds__(256) void widen_bf16_kernel(const u16 *__restrict__ src, int64_t lds_, const int32_t *__restrict__ ridx,
                                                         int64_t rows, int64_t cols, float *__restrict__ dst, int64_t ldd)
{
    const int64_t n = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / cols, c = i % cols;
        const int64_t sr = ridx ? (int64_t)ridx[r] : r;
        dst[r * ldd + c] = __builtin_bit_cast(float, (uint32_t)src[sr * lds_ + c] << 16);
    }
}

__global__ __launch_bounds__(256) void narrow_bf16_kernel(const float *__restrict__ src, int64_t lds_, int64_t rows, int64_t cols,
                                                          u16 *__restrict__ dst, int64_t ldd)
{
    const int64_t n = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / cols, c = i % cols;
        dst[r * ldd + c] = to_bf16_bits(src[r * lds_ + c]);
    }
}

} // namespace

size_t sgnn_gemm_ws_bytes(uint32_t d_max) { return (size_t)256 * d_max * d_max * 4 + (size_t)256 * d_max * 4 + 512; }

static inline int64_t gemm_pad4(int64_t d) { return (d + 3) & ~int64_t(3); }

// C = sum of `splits` partial products [splits][M][N] in a fixed order; cs_out = the same for [splits][N] column sums.
int sgnn_launch_splitk_reduce(sgnn_ctx *ctx, const float *partial, int splits, int64_t M, int64_t N, float *C, int64_t ldc,
                              const float *cs_partial, float *cs_out, hipStream_t st)
{
    SGNN_LAUNCH(ctx, st, "splitk_reduce_kernel", SGNN_TAG, splitk_reduce_kernel, dim3(cdiv(M * N + (cs_partial ? N : 0), 256)), dim3(256),
                0, st, partial, splits, M * N, N, C, ldc, cs_partial, cs_out);
    return SGNN_OK;
}

int sgnn_launch_gemm(sgnn_ctx *ctx, int ta, int tb, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                     const int32_t *a_row_index, const float *B, int64_t ldb, const float *bias, int flags, float *C,
                     int64_t ldc, const float *mask, int64_t ldm, float *b_colsum, ws_alloc *ws, hipStream_t st)
{
    return sgnn_launch_gemm_x(ctx, ta, tb, M, N, K, A, 0, lda, a_row_index, B, 0, ldb, bias, flags, C, 0, ldc, mask, 0, ldm, b_colsum, ws,
                              st);
}

int sgnn_launch_gemm_x(sgnn_ctx *ctx, int ta, int tb, int64_t M, int64_t N, int64_t K, const void *Av, int a_bf16, int64_t lda,
                       const int32_t *a_row_index, const void *Bv, int b_bf16, int64_t ldb, const float *bias, int flags, void *Cv,
                       int c_bf16, int64_t ldc, const void *maskv, int m_bf16, int64_t ldm, float *b_colsum, ws_alloc *ws,
                       hipStream_t st)
{
    const int bf16 = (flags & SGNN_BF16_MFMA) ? 1 : 0;
    if ((a_bf16 || b_bf16 || c_bf16) && !bf16)
        return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_gemm: bfloat16 storage of A or C goes with SGNN_BF16_MFMA only");
    if (!maskv) m_bf16 = 0;
    // Which kernel reads or writes the 16-bit storage itself: the tall-operand kernel (A, C, the mask) and the chunked
    // tile kernel for A^T B (A and B).  For everything else the operand is widened into scratch
    // first (exact), or the result narrowed from scratch afterwards (the same rounding the kernel would apply).
    const bool a_al16 = (reinterpret_cast<uintptr_t>(Av) & 7) == 0 && lda % 4 == 0;
    const bool skinny_shape = bf16 && !ta && K >= 1 && K <= 256 && N >= 1 && N <= 256 && M >= 4096;
    const bool a_al = a_bf16 ? a_al16 : ((reinterpret_cast<uintptr_t>(Av) & 15) == 0 && lda % 4 == 0);
    const bool b_al = (reinterpret_cast<uintptr_t>(Bv) & (b_bf16 ? 7 : 15)) == 0 && ldb % 4 == 0;
    const bool tn_fast16 = bf16 && ta && !tb && a_al && b_al && M % 4 == 0 && N % 4 == 0 && M >= 4 && N >= 4 && K >= 1;
    const bool a_native = a_bf16 && ((skinny_shape && a_al16) || tn_fast16);
    // A^T B with both operands stored as bfloat16 and a result of up to 256 x 256 (the weight gradients of a stack whose
    // activations and hand-down gradients are 16-bit): the streaming kernel, when it takes the shape (any M and N,
    // odd ones included, which the chunked tile kernel would only take after widening both operands)
    if (bf16 && ta && !tb && a_bf16 && b_bf16 && !c_bf16 && !a_row_index && !bias && !(flags & SGNN_RELU) && !maskv) {
        const int rc = sgnn_launch_gemm_tn_stream(ctx, M, N, K, Av, lda, Bv, ldb, static_cast<float *>(Cv), ldc, b_colsum, ws, st);
        if (rc != SGNN_ERR_UNSUPPORTED) return rc;
    }
    const float *B = static_cast<const float *>(Bv);
    if (b_bf16 && !tn_fast16) {
        const int64_t rows = tb ? N : K, cols = tb ? K : N, ldw = gemm_pad4(cols);
        float *Bw = ws->get<float>((size_t)rows * ldw);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small to widen a bfloat16 operand: call sgnn_ctx_reserve");
        if (rows * cols > 0)
            SGNN_LAUNCH(ctx, st, "widen_bf16_kernel", SGNN_TAG, widen_bf16_kernel, dim3((unsigned)std::min<int64_t>(cdiv(rows * cols, 256), 65536)),
                        dim3(256), 0, st, static_cast<const u16 *>(Bv), ldb, (const int32_t *)nullptr, rows, cols, Bw, ldw);
        B = Bw; ldb = ldw; b_bf16 = 0;
    }
    const bool cm_native = skinny_shape && (a_bf16 ? a_native : ((reinterpret_cast<uintptr_t>(Av) & 15) == 0 && lda % 4 == 0));
    const float *A = static_cast<const float *>(Av);
    if (a_bf16 && !a_native) {
        const int64_t rows = ta ? K : M, cols = ta ? M : K, ldw = gemm_pad4(cols);
        float *Aw = ws->get<float>((size_t)rows * ldw);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small to widen a bfloat16 operand: call sgnn_ctx_reserve");
        if (rows * cols > 0)
            SGNN_LAUNCH(ctx, st, "widen_bf16_kernel", SGNN_TAG, widen_bf16_kernel, dim3((unsigned)std::min<int64_t>(cdiv(rows * cols, 256), 65536)),
                        dim3(256), 0, st, static_cast<const u16 *>(Av), lda, a_row_index, rows, cols, Aw, ldw);
        A = Aw; lda = ldw; a_row_index = nullptr; a_bf16 = 0;
    }
    const float *mask = static_cast<const float *>(maskv);
    if (m_bf16 && !cm_native) {
        const int64_t ldw = gemm_pad4(N);
        float *Mw = ws->get<float>((size_t)M * ldw);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small to widen a bfloat16 mask: call sgnn_ctx_reserve");
        if (M * N > 0)
            SGNN_LAUNCH(ctx, st, "widen_bf16_kernel", SGNN_TAG, widen_bf16_kernel, dim3((unsigned)std::min<int64_t>(cdiv(M * N, 256), 65536)),
                        dim3(256), 0, st, static_cast<const u16 *>(maskv), ldm, (const int32_t *)nullptr, M, N, Mw, ldw);
        mask = Mw; ldm = ldw; m_bf16 = 0;
    }
    float *C = static_cast<float *>(Cv);
    if (c_bf16 && !cm_native) {
        const int64_t ldw = gemm_pad4(N);
        float *Cw = ws->get<float>((size_t)M * ldw);
        if (!ws->ok) return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small for a bfloat16 result: call sgnn_ctx_reserve");
        int rc = sgnn_launch_gemm_x(ctx, ta, tb, M, N, K, A, a_bf16, lda, a_row_index, B, b_bf16, ldb, bias, flags, Cw, 0, ldw, mask, m_bf16,
                                    ldm, b_colsum, ws, st);
        if (rc) return rc;
        if (M * N > 0)
            SGNN_LAUNCH(ctx, st, "narrow_bf16_kernel", SGNN_TAG, narrow_bf16_kernel, dim3((unsigned)std::min<int64_t>(cdiv(M * N, 256), 65536)),
                        dim3(256), 0, st, Cw, ldw, M, N, static_cast<u16 *>(Cv), ldc);
        return SGNN_OK;
    }

    gemm_args a = {};      // every field the call does not set is zero (fp32 storage, no mask, no row gather)
    a.mask = mask; a.ldm = ldm;
    a.colsum = nullptr;
    a.a_row_index = a_row_index;
    a.M = M; a.N = N; a.K = K;
    a.A = A; a.lda = lda; a.B = B; a.ldb = ldb; a.bias = bias; a.C = C; a.ldc = ldc;
    a.a_bf16 = a_bf16; a.b_bf16 = b_bf16; a.c_bf16 = c_bf16; a.m_bf16 = m_bf16;
    a.relu = (flags & SGNN_RELU) ? 1 : 0;
    a.alignedA = a_bf16 ? (a_al16 ? 1 : 0) : (((reinterpret_cast<uintptr_t>(A) & 15) == 0 && lda % 4 == 0) ? 1 : 0);
    a.alignedB = b_bf16 ? 1 : (((reinterpret_cast<uintptr_t>(B) & 15) == 0 && ldb % 4 == 0) ? 1 : 0);     // a bfloat16 B got here through tn_fast16 only
    a.vecM = (mask && N % 4 == 0 && ldm % 4 == 0 && (reinterpret_cast<uintptr_t>(mask) & (m_bf16 ? 7 : 15)) == 0) ? 1 : 0;
    a.c_pair = (c_bf16 && N % 2 == 0 && ldc % 2 == 0 && (reinterpret_cast<uintptr_t>(C) & 3) == 0) ? 1 : 0;
    a.vecC = (!c_bf16 && !m_bf16 && (reinterpret_cast<uintptr_t>(C) & 15) == 0 && ldc % 4 == 0 && N % 4 == 0 &&
              (!mask || ((reinterpret_cast<uintptr_t>(mask) & 15) == 0 && ldm % 4 == 0)) &&
              (!bias || (reinterpret_cast<uintptr_t>(bias) & 15) == 0)) ? 1 : 0;
    a.k_per_split = K;
    a.partial = nullptr;
    const int BK = bf16 ? 32 : SGNN_GEMM_BK_F32;

    // tall A times a small B on the bf16 path: stream A once with B resident in LDS
    if (skinny_shape && a.alignedA) {
        if (b_colsum) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: column sums of B go with A^T B only");
        return launch_skinny(ctx, a, tb, st);
    }

    // classifier-width products, fp32: straight from global memory into the MFMA operand layout
    if (!bf16 && !ta && tb && !a_row_index && K >= 4 && K <= 64 && K % 4 == 0 && a.alignedA && a.alignedB && M >= 1 && N >= 1 &&
        M <= (int64_t)0x7fffffff * 32 && N <= (int64_t)65535 * 128) {
        if (b_colsum) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: column sums of B go with A^T B only");
        char tag[56];
        snprintf(tag, sizeof(tag), "NT smallk %lldx%lldx%lld f32", (long long)M, (long long)N, (long long)K);
        dim3 grid((unsigned)cdiv(M, 32), (unsigned)cdiv(N, 128 * SMALLK_TW)), block(256);
        const int q = (int)cdiv(K, 8);
        if (q <= 1)      { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_smallk_nt_kernel<1>, grid, block, 0, st, a); }
        else if (q <= 2) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_smallk_nt_kernel<2>, grid, block, 0, st, a); }
        else if (q <= 4) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_smallk_nt_kernel<4>, grid, block, 0, st, a); }
        else             { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_smallk_nt_kernel<8>, grid, block, 0, st, a); }
        return SGNN_OK;
    }
    // long reductions onto a result of classifier width (that layer's weight gradient): 128 x 32 tiles, as many
    // reduction ranges as give every compute unit a workgroup.  (A variant with 128 x 64 tiles ran the wide weight
    // gradients as fast as the LDS-tiled kernel below, no faster: both wait for operands.)
    if (!bf16 && ta && !tb && N >= 1 && N <= 32 && cdiv(M, 128) <= 64 && K >= 4096 && M >= 4 && M % 4 == 0 && a.alignedA && !bias &&
        !(flags & SGNN_RELU) && !mask) {
        constexpr int PAIRS = THIN_PAIRS;
        a.mtiles = cdiv(M, 128); a.ntiles = 1;
        const int64_t tiles = a.mtiles;
        int64_t splits = std::max<int64_t>(1, 256 / tiles);
        splits = std::min<int64_t>(splits, cdiv(K, (int64_t)2 * PAIRS * THIN_WAVES));
        const int64_t unit = 2 * THIN_WAVES;
        const int64_t kps = cdiv(cdiv(K, splits), unit) * unit;
        splits = cdiv(K, kps);
        a.k_per_split = kps;
        a.splits = (uint32_t)splits;
        a.partial = ws->get<float>((size_t)splits * M * N);
        float *cs_part = b_colsum ? ws->get<float>((size_t)splits * N) : nullptr;
        if (!ws->ok)
            return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small for the split reduction: call sgnn_ctx_reserve");
        a.colsum = cs_part;
        char tag[56];
        snprintf(tag, sizeof(tag), "TN thin32 %lldx%lldx%lld f32", (long long)M, (long long)N, (long long)K);
        // at most 64 tiles and K >= 4096: always several reduction ranges, which tile_of_block() keeps together
        // on an XCD (all tiles of a range read the same rows of B)
        const dim3 grid((unsigned)(cdiv(splits, 8) * 8 * tiles)), block(64 * THIN_WAVES);
        if (a_row_index) { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_thin_tn_kernel<true>, grid, block, 0, st, a); }
        else             { SGNN_LAUNCH(ctx, st, "gemm_kernel", tag, gemm_thin_tn_kernel<false>, grid, block, 0, st, a); }
        SGNN_LAUNCH(ctx, st, "splitk_reduce_kernel", SGNN_TAG, splitk_reduce_kernel, dim3(cdiv(M * N + (cs_part ? N : 0), 256)),
                    dim3(256), 0, st, a.partial, (int)splits, M * N, N, C, ldc, cs_part, b_colsum);
        return SGNN_OK;
    }

    // wide fp32 results with whole chunks and whole slices: the direct-to-LDS kernel, 256 x 128 tiles.  Not for
    // the long reductions onto a small result (T^T dZ): with two 256 x 128 tiles the split would have to be
    // twice as fine, and the partial products it writes cost more than the kernel gains (those take the
    // kernel's 128 x 128 form, direct128 below).
    const int64_t a_contig = ta ? M : K, b_contig = tb ? K : N;
    const bool direct = !bf16 && !ta && a.alignedA && a.alignedB && a_contig % 4 == 0 && b_contig % 4 == 0 &&
                        a_contig >= 4 && b_contig >= 4 && K % 32 == 0 && K >= 128 && N > 64 && M > 128;

    // the weight gradients of the wide layers (A^T B, long reduction onto a result of a few 128 x 128 tiles): the same
    // kernel with 128-row tiles, one workgroup per reduction range and tile, two slices in flight behind the one
    // being multiplied (the register-staged tile kernel has one, and its wavefronts wait for it half of the time) and
    // eight wavefronts, two per SIMD (with four, one per SIMD, it was no faster than the tile kernel: nothing
    // multiplies while the only wavefront of a SIMD issues loads, reads LDS or stands at the barrier)
    const bool direct128 = !bf16 && ta && !tb && a.alignedA && a.alignedB && M % 4 == 0 && N % 4 == 0 &&
                           M > 64 && N > 64 && K % 32 == 0 && K >= 4096 && !bias && !(flags & SGNN_RELU) && !mask &&
                           (int64_t)cdiv(M, 128) * cdiv(N, 128) <= 64;

    // tile shape by the width of C
    const int bn = N > 64 ? 128 : (N > 32 ? 64 : 32);
    // narrow results: 256-row tiles, or 128-row ones when those would leave compute units without a tile
    const bool narrow128 = bn == 32 && K < 4096 && cdiv(M, 256) < 256;
    const int bm = direct ? DIRECT_BM : (bn == 32 ? (narrow128 ? 128 : 256) : 128);
    int splits = 1;
    const int64_t tiles = (int64_t)cdiv(M, bm) * cdiv(N, bn);
    if (tiles < 256 && K >= 4096 && !bias && !(flags & SGNN_RELU) && !mask) {
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
    // column sums of B next to A^T B: inside the tile kernel when it is the chunked (fast) one, else a pass of its own
    float *cs_partial = nullptr;
    bool cs_fused = false;
    if (b_colsum) {
        if (!ta || tb) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm: column sums of B go with A^T B only");
        cs_fused = !direct && a.alignedA && a.alignedB && M % 4 == 0 && N % 4 == 0 && M >= 4 && N >= 4 && K >= 1;   // direct128 included
        if (cs_fused) {
            if (splits > 1) {
                cs_partial = ws->get<float>((size_t)splits * N);
                if (!ws->ok)
                    return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_gemm: scratch too small for the split reduction: call sgnn_ctx_reserve");
                a.colsum = cs_partial;
            } else a.colsum = b_colsum;
        }
    }
    int rc;
    if (direct) rc = launch_direct(ctx, ta, tb, a, splits, false, st);
    else if (direct128 && splits > 1) rc = launch_direct(ctx, ta, tb, a, splits, true, st);
    else if (bn == 128) rc = launch_cfg<128, 128, 64, 64>(ctx, ta, tb, bf16, a, splits, st);
    else if (bn == 64) rc = launch_cfg<128, 64, 64, 32>(ctx, ta, tb, bf16, a, splits, st);
    else if (narrow128) rc = launch_cfg<128, 32, 32, 32>(ctx, ta, tb, bf16, a, splits, st);
    else rc = launch_cfg<256, 32, 64, 32>(ctx, ta, tb, bf16, a, splits, st);
    if (rc) return rc;
    if (splits > 1) {
        SGNN_LAUNCH(ctx, st, "splitk_reduce_kernel", SGNN_TAG, splitk_reduce_kernel, dim3(cdiv(M * N + (cs_partial ? N : 0), 256)),
                    dim3(256), 0, st, a.partial, splits, M * N, N, C, ldc, cs_partial, b_colsum);
    }
    if (b_colsum && !cs_fused)
        return sgnn_launch_relu_bwd_bias(ctx, nullptr, 0, 0, B, ldb, 0, K, N, nullptr, 0, b_colsum, ws, st);
    return SGNN_OK;
}

// Z = A W with the layer tail fused into the epilogue (bf16 operands, the tall-operand kernel).  Returns
// SGNN_ERR_UNSUPPORTED without launching when the shape is outside that kernel's range: the caller then runs
// the product and the tail as two launches.
int sgnn_launch_gemm_tail(sgnn_ctx *ctx, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *W,
                          int64_t ldw, const float *gamma, float eps, const float *R, int64_t ldr, float q, uint64_t seed,
                          uint32_t layer, uint64_t step, float *Z, int64_t ldz, float *Y, int64_t ldy, float *inv_rms,
                          hipStream_t st)
{
    if (!(q >= 0.f) || !(q < 1.f)) return sgnn_fail(ctx, SGNN_ERR_INVALID_ARG, "sgnn_gemm_tail_fwd: need 0 <= drop_q < 1");
    const bool alignedA = (reinterpret_cast<uintptr_t>(A) & 15) == 0 && lda % 4 == 0;
    if (!(K >= 1 && K <= 256 && N >= 1 && N <= 256 && N % 4 == 0 && M >= 4096 && alignedA)) return SGNN_ERR_UNSUPPORTED;
    gemm_args a = {};      // every field the call does not set is zero (fp32 storage, no mask, no row gather)
    a.a_row_index = nullptr;
    a.M = M; a.N = N; a.K = K;
    a.A = A; a.lda = lda; a.B = W; a.ldb = ldw; a.bias = nullptr; a.C = Z; a.ldc = ldz;
    a.relu = 0; a.mask = nullptr; a.ldm = 0;
    a.alignedA = 1;
    a.alignedB = ((reinterpret_cast<uintptr_t>(W) & 15) == 0 && ldw % 4 == 0) ? 1 : 0;
    a.k_per_split = K; a.partial = nullptr; a.mtiles = a.ntiles = a.splits = 0; a.colsum = nullptr;
    skinny_tail tl;
    tl.gamma = gamma; tl.eps = eps; tl.R = R; tl.ldr = ldr; tl.Y = Y; tl.ldy = ldy; tl.inv_rms = inv_rms;
    tl.thr = (uint32_t)floor((double)q * 4294967296.0);
    tl.scale = q > 0.f ? (float)(1.0 / (1.0 - (double)q)) : 1.f;
    tl.k0 = (uint32_t)seed; tl.k1 = (uint32_t)(seed >> 32); tl.c2 = (uint32_t)step; tl.c3 = 0x80000000u + layer;
    return launch_skinny_t<true>(ctx, a, 0, tl, st);
}
