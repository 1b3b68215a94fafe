// Weight gradient of a wide mini-batch (Sec. III-C: dW = H_agg^T dZ) with both operands stored as bfloat16:
//   C [M x N] = A^T B,   A given [K x M], B given [K x N], M, N <= 256, K = the number of sampled vertices (10^5 .. 10^6).
//
// The product reads 2 K (M + N) bytes and computes 2 K M N flop: with M = N = 256 that is 128 flop per byte, far below
// the machine's bf16 ridge, so the kernel is built as a stream over K and nothing else:
//  - a workgroup owns a range of K and the WHOLE M x N result (accumulators in registers: 8 wavefronts, each a
//    128 x 64 part as 4 x 2 MFMA tiles of 32 x 32), so every row of A and of B is fetched from HBM once, by one workgroup;
//  - 32 consecutive rows of A (and of B) are one contiguous block of memory, copied as it is into LDS with direct
//    global -> LDS loads (16 bytes a lane, no registers in between), four slices deep: three slices are in flight
//    behind the one being multiplied, one barrier per slice;
//  - v_mfma_f32_32x32x16_bf16 wants, per lane, eight consecutive reduction steps of ONE column of A, which in this
//    storage are eight rows apart.  A lane reads four adjacent columns of one row at a time (8 bytes; two for B) and
//    the wavefront's tiles are interleaved - tile i takes columns 4 l + i - so the eight reads of a 16-step block serve
//    all four tiles, and a v_perm puts two reduction steps into one operand register;
//  - the column sums of B (the bias gradient that rides along) come from the matrix pipe too: one more MFMA per B
//    tile with an A operand that is 1 in result row 0 and 0 elsewhere;
//  - every workgroup writes one partial product; they are added in a fixed order by the split reduction of gemm.hip.
// Columns of the 256 x 256 frame beyond M or N read whatever follows in LDS (finite or not): they only feed result
// rows and columns that are never stored.
#include <algorithm>

#include "common.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16;

constexpr int TNS_BK = 32;          // rows of a slice
constexpr int TNS_STAGES = 4;
constexpr int TNS_WAVES = 8;
constexpr int TNS_LOADS = 4;        // wave-loads (1 KB each) a wavefront issues per slice: 8 x 4 KB = 32 KB >= 32 x (256 + 256) x 2
constexpr int TNS_STAGE_BYTES = TNS_BK * 512 * 2;                 // room for 32 rows of up to 256 + 256 elements
constexpr int TNS_SLACK = 4096;     // head-room behind the last stage (reads of the frame's unused columns end exactly at a stage's end when ld = 256)

#define TNS_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define TNS_LPTR(p) ((__attribute__((address_space(3))) void *)(p))
// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left at their maxima), gfx9 encoding
#define TNS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

struct tns_args {
    const u16 *A; int64_t lda;      // [K x M] bfloat16, lda a multiple of 8
    const u16 *B; int64_t ldb;      // [K x N] bfloat16, ldb a multiple of 8
    int M, N;
    int64_t K, k_per_split;         // multiples of 32
    float *partial;                 // [splits][M][N]
    float *cs_partial;              // [splits][N] or NULL
    int interleave;
};

__global__ __launch_bounds__(64 * TNS_WAVES) void gemm_tn_stream_kernel(tns_args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char tns_smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kh = lane >> 5;
    const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
    // interleave: workgroup w takes slices w, w + splits, ... (the workgroups read one region together, as a copy kernel
    // does); else a contiguous range of k_per_split rows
    const int64_t kbeg = a.interleave ? (int64_t)blockIdx.x * TNS_BK : (int64_t)blockIdx.x * a.k_per_split;
    const int64_t kend = min(a.K, kbeg + a.k_per_split);
    const int64_t kstep = a.interleave ? (int64_t)gridDim.x * TNS_BK : TNS_BK;
    const int64_t total_slices = a.K / TNS_BK;
    const int nslices = a.interleave ? (int)((total_slices - blockIdx.x + gridDim.x - 1) / gridDim.x) : (int)((kend - kbeg) / TNS_BK);
    // one slice in LDS: the 32 rows of A as in memory (32 lda elements), then the 32 rows of B
    const int a_bytes = (int)(64 * a.lda), b_bytes = (int)(64 * a.ldb);     // 32 rows x ld x 2 bytes
    const int a_chunks = a_bytes / 16, chunks = (a_bytes + b_bytes) / 16;
    // the last row of a matrix need not be allocated beyond its last element: chunks of a block that hold nothing but the
    // padding behind the block's last row are not fetched (the chunk with the row's last element is fetched in their place)
    const int a_valid = (int)((2 * (31 * a.lda + a.M) + 15) / 16), b_valid = (int)((2 * (31 * a.ldb + a.N) + 15) / 16);

    // the wavefront's TNS_LOADS wave-loads of a slice: chunk (wave + 8 j) 64 + lane of [A block | B block]; a chunk past
    // the end repeats the last one (the same bytes to the same place), so that every wavefront has the same number of
    // loads in flight and the waits below count exactly
    auto issue = [&](int s) {
        const int sl = min(s, nslices - 1);          // past the end: the last slice again, into a stage nobody reads
        unsigned char *stage = tns_smem + (s % TNS_STAGES) * TNS_STAGE_BYTES;
        const unsigned char *ga = reinterpret_cast<const unsigned char *>(a.A + (kbeg + (int64_t)sl * kstep) * a.lda);
        const unsigned char *gb = reinterpret_cast<const unsigned char *>(a.B + (kbeg + (int64_t)sl * kstep) * a.ldb);
#pragma unroll
        for (int j = 0; j < TNS_LOADS; ++j) {
            const int q = wave + TNS_WAVES * j;
            const int c = min(64 * q + lane, chunks - 1);
            const unsigned char *g = c < a_chunks ? ga + 16 * min(c, a_valid - 1) : gb + 16 * min(c - a_chunks, b_valid - 1);
            // the LDS address of a direct load is wave-uniform base + 16 lane: chunk 64 q + lane lands at 16 (64 q + lane),
            // the clamped lanes' copies of the last chunk behind the slice's data, still inside the 32 KB of the stage
            __builtin_amdgcn_global_load_lds(TNS_GPTR(g), TNS_LPTR(stage + 1024 * q), 16, 0, 0);
        }
    };

    f32x16 acc[4][2], cs[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { acc[i][0][r] = 0.f; acc[i][1][r] = 0.f; }
        cs[0][r] = 0.f; cs[1][r] = 0.f;
    }
    // A operand of the column sums: 1.0 for result row 0 (lanes with li == 0), 0 elsewhere
    bf16x8 ones;
#pragma unroll
    for (int t = 0; t < 8; ++t) ones[t] = (__bf16)(li == 0 ? 1.0f : 0.0f);
    const bool wave_live = wm0 < a.M && wn0 < a.N;       // its part of the frame holds something of the result
    const bool do_cs = a.cs_partial && wm0 == 0 && wn0 < a.N;

    issue(0);
    issue(1);
    issue(2);
    for (int s = 0; s < nslices; ++s) {
        TNS_WAIT_VMCNT(2 * TNS_LOADS);           // slice s has landed (this wavefront's part); s + 1 and s + 2 may be in flight
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();            // everybody's part has; and everybody is through slice s - 1
        asm volatile("" ::: "memory");
        issue(s + 3);                            // into the stage slice s - 1 was read from
        if (wave_live) {
            const unsigned char *stage = tns_smem + (s % TNS_STAGES) * TNS_STAGE_BYTES;
            const unsigned char *LA = stage + 2 * (wm0 + 4 * li);
            const unsigned char *LB = stage + a_bytes + 2 * (wn0 + 2 * li);
            const int rowA = (int)(2 * a.lda), rowB = (int)(2 * a.ldb);
#pragma unroll
            for (int h = 0; h < 2; ++h) {          // the two 16-step blocks of the slice
                uint2 ra[8];
                uint32_t rb[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int k = 16 * h + 8 * kh + t;
                    ra[t] = *reinterpret_cast<const uint2 *>(LA + k * rowA);
                    rb[t] = *reinterpret_cast<const uint32_t *>(LB + k * rowB);
                }
                // tile i of A: column 4 li + i = half (i & 1) of word (i >> 1) of every read; two steps a register
                bf16x8 fa[4], fb[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t w[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const uint32_t x0 = (i >> 1) ? ra[2 * p].y : ra[2 * p].x, x1 = (i >> 1) ? ra[2 * p + 1].y : ra[2 * p + 1].x;
                        // bytes of the result, low to high: the chosen half of x0, then the chosen half of x1
                        w[p] = (i & 1) ? __builtin_amdgcn_perm(x1, x0, 0x07060302u) : __builtin_amdgcn_perm(x1, x0, 0x05040100u);
                    }
                    fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(w));
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    uint32_t w[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p)
                        w[p] = j ? __builtin_amdgcn_perm(rb[2 * p + 1], rb[2 * p], 0x07060302u)
                                 : __builtin_amdgcn_perm(rb[2 * p + 1], rb[2 * p], 0x05040100u);
                    fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(w));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                if (do_cs) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) cs[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, fb[j], cs[j], 0, 0, 0);
                }
            }
        }
    }
    TNS_WAIT_VMCNT(0);       // the repeated loads past the end are still in flight: nothing may leave before they land

    // result: register r of lane (li, kh) of tile (i, j) is row wm0 + 4 rho + i, rho = 8 (r / 4) + 4 kh + r % 4,
    // column wn0 + 2 li + j: the lane's two tiles j are adjacent columns, one 8-byte store
    if (wave_live) {
        float *P = a.partial + (int64_t)blockIdx.x * a.M * a.N;
        const int n = wn0 + 2 * li;
        const bool n_even = (a.N & 1) == 0;   // odd N: rows of the partial result start on odd words, one store per value
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = wm0 + 4 * (8 * (r / 4) + 4 * kh + (r % 4)) + i;
                if (m < a.M && n < a.N) {
                    float *p = P + (int64_t)m * a.N + n;
                    if (n_even) *reinterpret_cast<float2 *>(p) = make_float2(acc[i][0][r], acc[i][1][r]);   // wholly inside
                    else {
                        p[0] = acc[i][0][r];
                        if (n + 1 < a.N) p[1] = acc[i][1][r];
                    }
                }
            }
        if (do_cs && kh == 0 && n < a.N) {           // result row 0: register 0 of the lanes with kh == 0
            float *p = a.cs_partial + (int64_t)blockIdx.x * a.N + n;
            p[0] = cs[0][0];
            if (n + 1 < a.N) p[1] = cs[1][0];
        }
    }
}

} // namespace

// Returns SGNN_ERR_UNSUPPORTED without launching anything when the shape or the storage is outside what the kernel
// handles (the caller then takes the tile kernel); otherwise launches the product and the split reduction.
int sgnn_launch_gemm_tn_stream(sgnn_ctx *ctx, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               float *C, int64_t ldc, float *b_colsum, ws_alloc *ws, hipStream_t st)
{
    if (M < 1 || N < 2 || M > 256 || N > 256 || K < 8192 || K % TNS_BK || lda % 8 || ldb % 8 || lda > 256 || ldb > 256 ||
        lda < M || ldb < N || (reinterpret_cast<uintptr_t>(A) & 15) || (reinterpret_cast<uintptr_t>(B) & 15))
        return SGNN_ERR_UNSUPPORTED;
    // one workgroup a compute unit; every workgroup at least 16 slices
    int64_t splits = std::min<int64_t>(256, K / (16 * TNS_BK));
    int64_t kps = (K / splits + TNS_BK - 1) / TNS_BK * TNS_BK;
    splits = (K + kps - 1) / kps;
    tns_args a;
    a.A = static_cast<const u16 *>(A); a.lda = lda; a.B = static_cast<const u16 *>(B); a.ldb = ldb;
    a.M = (int)M; a.N = (int)N; a.K = K; a.k_per_split = kps;
    a.interleave = 1;       // measured 4-6 % faster at K = 2^20 than contiguous ranges (256 separate streams through memory)
    // not enough scratch for one partial product per workgroup: the tile kernel needs less
    const size_t need = (((size_t)splits * M * N * 4 + 255) & ~size_t(255)) + (((size_t)splits * N * 4 + 255) & ~size_t(255));
    if (!ws->base || ws->off + need > ws->cap) return SGNN_ERR_UNSUPPORTED;
    a.partial = ws->get<float>((size_t)splits * M * N);
    a.cs_partial = b_colsum ? ws->get<float>((size_t)splits * N) : nullptr;
    const size_t lds = (size_t)TNS_STAGES * TNS_STAGE_BYTES + TNS_SLACK;
    static bool attr_set = false;
    if (!attr_set) {
        SGNN_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tn_stream_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    char tag[56];
    snprintf(tag, sizeof(tag), "TN stream %lldx%lldx%lld bf16 a=2 b=2", (long long)M, (long long)N, (long long)K);
    SGNN_LAUNCH(ctx, st, "gemm_tn_stream_kernel", tag, gemm_tn_stream_kernel, dim3((unsigned)splits), dim3(64 * TNS_WAVES), lds, st, a);
    return sgnn_launch_splitk_reduce(ctx, a.partial, (int)splits, M, N, C, ldc, a.cs_partial, b_colsum, st);
}
