// Sparse aggregation of the GCN layer (Sec. III-B Eq. 5 and the transposed SpMM of Sec. III-C):
// out = A X with A in CSR.
//
// Row-split with a side path for long rows.  A wavefront owns a block of consecutive output rows
// and walks their entries as one stream: the CSR entries of the block are contiguous, so they are
// fetched 64 at a time with one coalesced load, and several gathered feature rows are in flight
// however short the rows are.  The 64 lanes cover the columns (VEC*CH of them per lane), so every
// feature row is read with coalesced vector loads and every output row is written once.  Rows
// much longer than the mean (power-law graphs have them) would leave one wavefront walking
// alone long after the others are done, so a plan built once per matrix cuts them into pieces of
// 64 entries (longer pieces for hub rows, so that no row has more than 256 of them):
//   spmm_plan_kernel    (once per matrix) piece descriptors of the long rows, one ticket per long row
//   spmm_main_kernel    the first wavefronts take pieces (one partial row per piece), the others take
//                       blocks of rows; both kinds run side by side.  A piece wavefront that has
//                       stored its partial row draws a ticket of its row; the one that draws the last
//                       ticket adds the partial rows of the row up, in piece order, and writes the row.
// No atomics touch floating-point data and the order of every sum is fixed: results are
// bit-reproducible.  Nothing waits on another wavefront.  Two products that use the same plan must
// not run at the same time (they would share the tickets).
#include <stdlib.h>

#include <algorithm>

#include "block_prims.h"
#include <type_traits>

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

// A feature row stored as bfloat16 (16-bit patterns: the upper half of an fp32): widened while it is read.
struct bf16_bits { uint16_t v; };

template <int VEC> __device__ __forceinline__ void vload(float (&dst)[VEC], const bf16_bits *p)
{
    if constexpr (VEC == 1) dst[0] = __builtin_bit_cast(float, (uint32_t)p->v << 16);
    else if constexpr (VEC == 2) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
        dst[0] = __builtin_bit_cast(float, w << 16);
        dst[1] = __builtin_bit_cast(float, w & 0xffff0000u);
    } else {
        static_assert(VEC == 4, "vector width");
        const uint2 w = *reinterpret_cast<const uint2 *>(p);
        dst[0] = __builtin_bit_cast(float, w.x << 16);
        dst[1] = __builtin_bit_cast(float, w.x & 0xffff0000u);
        dst[2] = __builtin_bit_cast(float, w.y << 16);
        dst[3] = __builtin_bit_cast(float, w.y & 0xffff0000u);
    }
}

// A gathered chunk as the load instruction returns it (fp32 values, or packed bfloat16 pairs), and its i-th value.
// Widening a bfloat16 chunk right behind its load would make every gather wait for the one before it; kept raw, all
// gathers of a round are in flight together and the widening happens where the value is multiplied.
template <int VEC, typename XT> struct raw_chunk { float v[VEC]; };
template <int VEC> struct raw_chunk<VEC, bf16_bits> { uint32_t w[(VEC + 1) / 2]; };

template <int VEC> __device__ __forceinline__ void raw_load(raw_chunk<VEC, float> &r, const float *p) { vload<VEC>(r.v, p); }
template <int VEC> __device__ __forceinline__ void raw_load(raw_chunk<VEC, bf16_bits> &r, const bf16_bits *p)
{
    if constexpr (VEC == 1) r.w[0] = p->v;
    else if constexpr (VEC == 2) r.w[0] = *reinterpret_cast<const uint32_t *>(p);
    else {
        const uint2 q = *reinterpret_cast<const uint2 *>(p);
        r.w[0] = q.x; r.w[1] = q.y;
    }
}
template <int VEC> __device__ __forceinline__ float raw_get(const raw_chunk<VEC, float> &r, int i) { return r.v[i]; }
template <int VEC> __device__ __forceinline__ float raw_get(const raw_chunk<VEC, bf16_bits> &r, int i)
{
    const uint32_t w = r.w[i >> 1];
    return __builtin_bit_cast(float, (i & 1) ? (w & 0xffff0000u) : (w << 16));
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

// A finished output row segment: fp32 as it is, or rounded to bfloat16 (nearest even) and packed.
template <int VEC> __device__ __forceinline__ void vstore_out(float *out, int64_t elem, const float (&src)[VEC], int out_bf16)
{
    if (!out_bf16) { vstore<VEC>(out + elem, src); return; }
    uint16_t *p = reinterpret_cast<uint16_t *>(out) + elem;
    uint16_t h[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) h[i] = __builtin_bit_cast(uint16_t, (__bf16)src[i]);
    if constexpr (VEC == 1) *p = h[0];
    else if constexpr (VEC == 2) *reinterpret_cast<uint32_t *>(p) = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
    else *reinterpret_cast<uint2 *>(p) = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
}

// Device-scope stores and loads (relaxed atomics, one word each): the store goes through to the
// level of the memory system that all compute dies share and the load reads from there, so data
// handed from one wavefront to another inside a kernel needs no write-back or invalidation of a
// whole cache.  p points at the lane's first word; the VEC words of a lane are 64 words apart, so
// that every store or load instruction of the wavefront covers 256 contiguous bytes.
template <int VEC> __device__ __forceinline__ void vstore_device(float *p, const float (&src)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) __hip_atomic_store(p + i * 64, src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int VEC> __device__ __forceinline__ void vload_device(float (&dst)[VEC], const float *p)
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) dst[i] = __hip_atomic_load(p + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Row offsets are int32 (mini-batch matrices) or int64 (a full graph with 2^31 entries or more).
__device__ __forceinline__ int64_t rp_load(const void *__restrict__ rowptr, int rp64, uint64_t i)
{
    return rp64 ? static_cast<const int64_t *>(rowptr)[i] : (int64_t) static_cast<const int32_t *>(rowptr)[i];
}

__device__ __forceinline__ int64_t readlane64(int64_t v, int lane)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

constexpr int SPMM_NT = 256;       // threads of a workgroup
#ifndef SPMM_SHORT_LEN
#define SPMM_SHORT_LEN 8
#endif
constexpr int SPMM_SHORT = SPMM_SHORT_LEN;      // smallest length from which a row counts as long
constexpr int SPMM_CHUNK = 64;     // entries per piece of a long row: what one wavefront fetches at once
constexpr int SPMM_MAX_PIECES = 256;   // pieces per row: longer rows get longer pieces

// Entries per piece of a row with `len` entries: 64, doubled until the row has at most
// SPMM_MAX_PIECES pieces, so that the wavefront that adds the partial rows of a hub row up has a
// bounded number of them to read.
__host__ __device__ inline int64_t spmm_piece_len(int64_t len)
{
    int64_t c = SPMM_CHUNK;
    while (len > c * SPMM_MAX_PIECES) c *= 2;
    return c;
}
constexpr unsigned SPMM_PIECE_WAVES = 2048;
constexpr int SPMM_PLAN_NT = 1024;  // rows per workgroup of the plan kernel

// Plan of a matrix (device memory): header, first chunk number per row, chunk descriptors.
struct spmm_plan_view {
    uint32_t *n_chunks;     // header word 0
    uint32_t *part_base;    // [rows], defined for long rows only
    uint2 *desc;            // [max_chunks] (row, chunk index inside the row)
    uint32_t *ticket;       // [max_chunks], used at the first chunk number of a long row; zero between products
};

// Rows longer than this count as long: four times the mean row length of the matrix, and at least
// 1/65536 of its entries (a full graph with 10^9 entries has long rows in the hundreds that one
// wavefront walks without holding anything up; what must be cut are its hubs).  Evaluated on the
// device from the true entry count when the plan is built (header word 1 of the plan).
__host__ __device__ inline int spmm_long_len(uint32_t rows, uint64_t entries)
{
    const uint64_t mean = rows ? entries / rows : 0;
    uint64_t t = 4 * mean;
    if (t < SPMM_SHORT) t = SPMM_SHORT;
    if (t < (entries >> 16)) t = entries >> 16;      // never more than 65536 long rows, however large the matrix
    if (t > (1u << 20)) t = 1u << 20;
    return (int)t;
}

// Rows that one wavefront walks as a block: about 128 entries, at most 32 rows, and no fewer than 4096 wavefronts while
// the rows last.  Measured: 16 entries / 8 rows -> 32 / 16: 7 % faster on a 2^20-row matrix with 1.3 entries a row;
// 32 / 16 -> 128 / 32: the five products of a 2^18-row step with 6.3 entries a row 6-9 % faster each (steps/s + 3.4 %),
// those of the 2^20-row step 1-4 %, dense-degree and small mini-batches unchanged; more gathers in flight per
// wavefront, 16 instead of 8, were slower at every size.  The plan holds the figure for the true entry count (header
// word 2); the host sizes the grid with the capacity in its place, which can only give fewer rows.
#ifndef SPMM_BLOCK_ENTRIES
#define SPMM_BLOCK_ENTRIES 128
#endif
#ifndef SPMM_BLOCK_ROWS
#define SPMM_BLOCK_ROWS 32
#endif
#ifndef SPMM_U4
#define SPMM_U4 8
#endif
__host__ __device__ inline int spmm_rows_per_wave(uint32_t rows, uint64_t entries)
{
    const uint64_t mean = rows && entries >= rows ? entries / rows : 1;
    uint64_t r = SPMM_BLOCK_ENTRIES / (mean < SPMM_BLOCK_ENTRIES ? mean : SPMM_BLOCK_ENTRIES);
    if (r > SPMM_BLOCK_ROWS) r = SPMM_BLOCK_ROWS;
    if (r > rows / 4096) r = rows / 4096;
    return r < 1 ? 1 : (int)r;
}

inline uint32_t spmm_max_chunks(uint32_t rows, uint64_t capacity)
{
    // a long row has more than SPMM_SHORT entries whatever the mean is, and more than four times the
    // mean (rounded down, so at least twice the exact mean once there is an entry per row): at most
    // capacity / SPMM_SHORT of them and at most half the rows, each with at most one partly filled
    // chunk, plus the full chunks
    const uint64_t n = std::min<uint64_t>(capacity / SPMM_SHORT, (uint64_t)rows / 2 + 1) + capacity / SPMM_CHUNK + 2;
    // and no more than 65536 long rows (spmm_long_len) of at most SPMM_MAX_PIECES pieces each
    return (uint32_t)std::min<uint64_t>(n, (uint64_t)65536 * SPMM_MAX_PIECES + 2);
}

inline spmm_plan_view plan_view(void *plan, uint32_t rows, uint32_t max_chunks)
{
    uint8_t *p = static_cast<uint8_t *>(plan);
    spmm_plan_view v;
    v.n_chunks = reinterpret_cast<uint32_t *>(p);
    v.part_base = reinterpret_cast<uint32_t *>(p + 256);
    v.desc = reinterpret_cast<uint2 *>(p + 256 + (((size_t)rows * 4 + 255) & ~size_t(255)));
    v.ticket = reinterpret_cast<uint32_t *>(v.desc + max_chunks);
    return v;
}

__global__ void spmm_plan_clear_kernel(uint32_t *n_chunks) { *n_chunks = 0; }

// One thread per row: the long rows of a wavefront reserve their chunk numbers with one atomic add,
// each records its first one in part_base[row] and writes one (row, chunk) descriptor per chunk.  The chunk
// numbering depends on timing; the values computed from it do not.
__global__ __launch_bounds__(SPMM_PLAN_NT) void spmm_plan_kernel(uint32_t rows, const void *__restrict__ rowptr, int rp64, uint64_t capacity,
                                                        uint32_t *__restrict__ n_chunks,
                                                        uint32_t max_chunks, uint32_t *__restrict__ part_base,
                                                        uint2 *__restrict__ desc, uint32_t *__restrict__ ticket)
{
    __shared__ uint32_t scan_lds[SPMM_PLAN_NT / 64 + 1];
    __shared__ uint32_t wg_base;
    const uint32_t row = blockIdx.x * SPMM_PLAN_NT + threadIdx.x;
    const uint64_t entries = min((uint64_t)rp_load(rowptr, rp64, rows), capacity);
    const int long_len = spmm_long_len(rows, entries);
    if (row == 0) {
        n_chunks[1] = (uint32_t)long_len;
        n_chunks[2] = (uint32_t)spmm_rows_per_wave(rows, entries);
    }
    int64_t len = 0;
    if (row < rows) len = min(rp_load(rowptr, rp64, (uint64_t)row + 1), (int64_t)capacity) - min(rp_load(rowptr, rp64, row), (int64_t)capacity);
    const int64_t plen = spmm_piece_len(len);
    const uint32_t nch = len > long_len ? (uint32_t)((len + plen - 1) / plen) : 0u;
    // one atomic per workgroup of 1024 rows (atomics on one address cost about 10 ns each, whoever issues
    // them): the long rows of the workgroup take consecutive piece numbers
    uint32_t wg_total;
    const uint32_t excl = block_excl_scan<uint32_t, SPMM_PLAN_NT>(nch, &wg_total, scan_lds);
    if (threadIdx.x == 0) wg_base = wg_total ? atomicAdd(n_chunks, wg_total) : 0u;
    __syncthreads();
    if (nch == 0) return;
    const uint32_t base = wg_base + excl;
    part_base[row] = base;
    if (base < max_chunks) ticket[base] = 0;
    for (uint32_t c = 0; c < nch && base + c < max_chunks; ++c) desc[base + c] = make_uint2(row, c);
}

// What happens to a finished output row: out = act(acc + bias), then (optionally) zero where the
// mask matrix is not positive - the ReLU backward of the layer below, fused into this product.
struct spmm_epi {
    const float *bias;
    int relu;
    const float *mask;
    int64_t ldm;
    const float *add;   // optional matrix added to the result last (the skip path of a residual layer)
    int64_t ldadd;
    int out_bf16;       // the result is stored as bfloat16 (rounded to nearest even; `out` then points at 16-bit elements)
    int mask_bf16;      // the mask matrix is stored as bfloat16
    // softmax cross-entropy of the finished rows (kernels instantiated with XENT; bias is the only other epilogue then)
    const int32_t *labels;      // class of every output row
    void *dO;                   // gradient rows (softmax - onehot) * inv_rows, or null
    int dO_bf16;
    int64_t lddo;
    float inv_rows;
    float *loss_partial;        // one partial sum of -log p_label per workgroup
    float *cs_partial;          // [workgroups][d] column sums of the stored gradient, or null
    int write_out;              // the logits are written to `out` as well
    // A long row is finished by whichever of its piece wavefronts comes last, so its share of the sums cannot go into
    // that wavefront's running sums (the result would depend on the race).  It is added, as 64-bit fixed-point
    // integers, to one of XENT_SLOTS rows of d + 1 counters chosen by the row number: integer addition is exact in
    // any order, and the final kernel adds the slots up.  [slot][d + 1], column d holds the loss terms.
    unsigned long long *fix;
};
constexpr int XENT_SLOTS = 256;
constexpr double XENT_FIX_CS = 1152921504606846976.0;      // 2^60: a gradient entry is at most 1 in magnitude, their sum too
constexpr double XENT_FIX_LOSS = 1073741824.0;             // 2^30: loss terms are below 2^10, at most 2^20 long rows

// per-wavefront running sums of the cross-entropy epilogue
template <int VEC, int CH> struct spmm_xent_sums {
    float loss;
    float cs[CH][VEC];
};

// Wavefront-wide sum / maximum for the row epilogue: four DPP steps make every lane of a 16-lane row hold the row's
// result (quad swaps, half mirror, mirror: register-to-register, no LDS round trips as with the shuffle built-ins, of
// which a reduction needs six in a dependent chain), four lane reads combine the rows.  The order of the additions is fixed.
template <int CTRL> __device__ __forceinline__ float dpp_f32(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
template <bool MAX> __device__ __forceinline__ float wave_reduce_rows(float x)
{
    auto op = [](float a, float b) { return MAX ? fmaxf(a, b) : a + b; };
    x = op(x, dpp_f32<0xB1>(x));      // quad_perm [1, 0, 3, 2]
    x = op(x, dpp_f32<0x4E>(x));      // quad_perm [2, 3, 0, 1]
    x = op(x, dpp_f32<0x141>(x));     // row_half_mirror
    x = op(x, dpp_f32<0x140>(x));     // row_mirror
    const int xi = __builtin_bit_cast(int, x);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0)), r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16)),
                r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 32)), r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 48));
    return op(op(r0, r1), op(r2, r3));
}

// Cross-entropy of one finished row of logits v (bias already added), held by the wavefront as chunk (m, lane) =
// columns (m * 64 + lane) * VEC ..: the row's softmax from one maximum and one sum across the wavefront, the
// gradient row written where the logits would be read back from otherwise.  Probabilities are exp(x - max) / sum,
// as in the stand-alone loss kernel.  A label outside [0, d) contributes the log-sum-exp alone.
template <int VEC, int CH, bool SHARED_ROW = false>
__device__ __forceinline__ void spmm_row_xent(const float (&v)[CH][VEC], const spmm_epi &ep, int64_t row, int32_t y, int d, int lane,
                                              spmm_xent_sums<VEC, CH> &xs)
{
    unsigned long long *fix = SHARED_ROW ? ep.fix + (uint64_t)(row % XENT_SLOTS) * (uint64_t)(d + 1) : nullptr;
    auto add_loss = [&](float t) {
        if constexpr (SHARED_ROW) atomicAdd(fix + d, (unsigned long long)(long long)llrint((double)t * XENT_FIX_LOSS));
        else xs.loss += t;
    };
    // d is a multiple of VEC (the launcher's condition for this instantiation): a lane's VEC columns of a chunk are
    // inside the row or outside it together
    float mx = -INFINITY;
#pragma unroll
    for (int m = 0; m < CH; ++m)
        if ((m * 64 + lane) * VEC < d) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) mx = fmaxf(mx, v[m][i]);
        }
    mx = wave_reduce_rows<true>(mx);
    float e[CH][VEC], s = 0.f;
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const bool in = (m * 64 + lane) * VEC < d;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            e[m][i] = in ? exp_neg(v[m][i] - mx) : 0.f;
            s += e[m][i];
        }
    }
    s = wave_reduce_rows<false>(s);
    const float inv = __builtin_amdgcn_rcpf(s), lse = log_ge1(s);       // 1 ulp each
    if ((uint32_t)y >= (uint32_t)d && lane == 0) add_loss(mx + lse);
#pragma unroll
    for (int m = 0; m < CH; ++m) {
        const int col = (m * 64 + lane) * VEC;
        if (col < d) {
            // the label's column, if it is one of this lane's: one test and one loss term per chunk, not one per column
            const uint32_t rel = (uint32_t)(y - col);
            if (rel < (uint32_t)VEC) {
                float vy = v[m][0];
#pragma unroll
                for (int i = 1; i < VEC; ++i) vy = rel == (uint32_t)i ? v[m][i] : vy;
                add_loss(lse - (vy - mx));
            }
            float g[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const bool hit = rel == (uint32_t)i;
                g[i] = (e[m][i] * inv - (hit ? 1.f : 0.f)) * ep.inv_rows;
                if (ep.dO_bf16) g[i] = (float)(__bf16)g[i];       // the column sums add what is stored
                if constexpr (SHARED_ROW) {
                    if (ep.cs_partial) atomicAdd(fix + col + i, (unsigned long long)(long long)llrint((double)g[i] * XENT_FIX_CS));
                } else xs.cs[m][i] += g[i];
            }
            if (ep.dO) vstore_out<VEC>(static_cast<float *>(ep.dO), row * ep.lddo + col, g, ep.dO_bf16);
        }
    }
}

// bias: the lane's VEC bias values (zeros without a bias), loaded once per wavefront: a lane's columns never change,
// and a load of them in front of every row's store cost a third of the kernel on a 2^20-row matrix
template <int VEC>
__device__ __forceinline__ void spmm_epilogue(float (&v)[VEC], const spmm_epi &ep, int64_t row, int col, const float (&bias)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        v[i] += bias[i];
        if (ep.relu) v[i] = fmaxf(v[i], 0.f);
    }
    if (ep.mask) {
        float m[VEC];
        if (ep.mask_bf16) vload<VEC>(m, reinterpret_cast<const bf16_bits *>(ep.mask) + row * ep.ldm + col);
        else vload<VEC>(m, ep.mask + row * ep.ldm + col);
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = m[i] > 0.f ? v[i] : 0.f;
    }
    if (ep.add) {
        float a[VEC];
        vload<VEC>(a, ep.add + row * ep.ldadd + col);
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] += a[i];
    }
}

// One wavefront walks `rows_per_wave` consecutive rows as one stream of entries.  The entries of
// consecutive rows are contiguous in the CSR arrays, so 64 of them are fetched with one coalesced
// load (lane l keeps entry e + l) and handed out by lane index; U gathered feature rows are in
// flight at a time whatever the lengths of the rows, the 64 lanes covering the columns.  Every
// value that steers the walk (row number, row bounds, entry number) is the same in all lanes.
// A row longer than long_len is left out: its chunks and the fix-up write it.
template <int VEC, int CH, typename XT, bool XENT>
__device__ __forceinline__ void spmm_wave_rows(uint32_t rows, const void *__restrict__ rowptr, int rp64,
                                               const int32_t *__restrict__ colidx, const float *__restrict__ val,
                                               uint64_t capacity, const XT *__restrict__ X, int64_t ldx,
                                               const int32_t *__restrict__ row_index, int d, uint64_t wave, int rows_per_wave,
                                               int long_len, float *__restrict__ out, int64_t ldo,
                                               const spmm_epi &ep, const float (&bias)[CH][VEC], spmm_xent_sums<VEC, CH> &xs)
{
    constexpr int U = CH * VEC <= 4 ? SPMM_U4 : (CH * VEC <= 8 ? 4 : 2);
    const int lane = threadIdx.x & 63;
    const uint64_t r0 = wave * (uint64_t)rows_per_wave;
    if (r0 >= rows) return;
    const int nr = (int)min((uint64_t)rows_per_wave, rows - r0);
    // lane k: start of row r0 + k, as an offset from the start of the block's first row (a block of
    // rows holds far fewer than 2^31 entries, so everything behind this line is 32-bit)
    int64_t rpl = 0;
    if (lane <= nr) rpl = min(rp_load(rowptr, rp64, r0 + lane), (int64_t)min(capacity, (uint64_t)0x7fffffffffffffffull));
    const int64_t block_base = readlane64(rpl, 0);
    const int32_t rp = lane <= nr ? (int32_t)(rpl - block_base) : 0;
    int32_t ylane = 0;      // XENT: lane k holds the label of row r0 + k
    if constexpr (XENT) ylane = lane < nr ? ep.labels[r0 + lane] : 0;
    colidx += block_base;
    val += block_base;
    const int e_end = __builtin_amdgcn_readlane(rp, nr);
    int e = __builtin_amdgcn_readlane(rp, 0);
    int row = 0, row_end = __builtin_amdgcn_readlane(rp, 1);
    bool row_long = row_end - e > long_len;
    float acc[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;

    // the current row is complete: write it (unless it is a long one) and move to the next
    auto next_row = [&]() {
        if (!row_long) {
            const int64_t o = (int64_t)(r0 + row) * ldo;
            if constexpr (XENT) {
#pragma unroll
                for (int m = 0; m < CH; ++m)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[m][i] += bias[m][i];
                spmm_row_xent<VEC, CH>(acc, ep, (int64_t)(r0 + row), __builtin_amdgcn_readlane(ylane, __builtin_amdgcn_readfirstlane(row)),
                                       d, lane, xs);
            }
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * 64 + lane) * VEC;
                if (col < d) {
                    if constexpr (XENT) {
                        if (ep.write_out) vstore_out<VEC>(out, o + col, acc[m], 0);
                    } else {
                        spmm_epilogue<VEC>(acc[m], ep, (int64_t)(r0 + row), col, bias[m]);
                        vstore_out<VEC>(out, o + col, acc[m], ep.out_bf16);
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < CH; ++m)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
        ++row;
        if (row < nr) {
            const int rs = row_end;
            row_end = __builtin_amdgcn_readlane(rp, __builtin_amdgcn_readfirstlane(row + 1));
            row_long = row_end - rs > long_len;
        }
    };

    for (;;) {
        while (row < nr && (e >= row_end || row_long)) {
            if (row_long) e = max(e, row_end);
            next_row();
        }
        if (row >= nr) break;
        // e is an entry of a row this wavefront sums: fetch up to 64 entries from there
        const int n = min(64, e_end - e);
        int32_t src = 0;
        float a = 0.f;
        if (lane < n) {
            const int32_t c = colidx[e + lane];
            a = val[e + lane];
            src = row_index ? row_index[c] : c;
        }
        int used = n;
        for (int j0 = 0; j0 < n && used == n; j0 += U) {
            raw_chunk<VEC, XT> v[U][CH];
            float av[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
                const int jj = __builtin_amdgcn_readfirstlane(min(j0 + t, n - 1));
                const XT *x = X + (int64_t)__builtin_amdgcn_readlane(src, jj) * ldx;
                av[t] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), jj));
#pragma unroll
                for (int m = 0; m < CH; ++m) {
                    const int col = (m * 64 + lane) * VEC;
                    if (col < d) raw_load<VEC>(v[t][m], x + col);
                }
            }
#pragma unroll
            for (int t = 0; t < U; ++t) {
                if (j0 + t < n && used == n) {
                    const int ee = e + j0 + t;
                    while (ee >= row_end) next_row();     // ee < e_end: a later row of this block holds it
                    if (row_long) used = j0 + t;          // stop in front of the long row
                    else {
#pragma unroll
                        for (int m = 0; m < CH; ++m) {
                            const int col = (m * 64 + lane) * VEC;
                            if (col < d) {
#pragma unroll
                                for (int i = 0; i < VEC; ++i) acc[m][i] = fmaf(av[t], raw_get<VEC>(v[t][m], i), acc[m][i]);
                            }
                        }
                    }
                }
            }
        }
        e += used;
    }
}

// acc += sum over the n <= 64 entries starting at e, which lane l < n holds as (src, a): U feature
// rows in flight at a time, handed out by lane index.  keep(j) tells whether entry j still counts
// and may move the caller's row state; it is called in entry order.
template <int VEC, int CH, int U, typename XT, typename Keep>
__device__ __forceinline__ void spmm_wave_entries(float (&acc)[CH][VEC], int32_t src, float a, int n, const XT *__restrict__ X,
                                                  int64_t ldx, int d, int lane, Keep keep)
{
    bool go = true;
    for (int j0 = 0; j0 < n && go; j0 += U) {
        raw_chunk<VEC, XT> v[U][CH];
        float av[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const int jj = __builtin_amdgcn_readfirstlane(min(j0 + t, n - 1));
            const XT *x = X + (int64_t)__builtin_amdgcn_readlane(src, jj) * ldx;
            av[t] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), jj));
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * 64 + lane) * VEC;
                if (col < d) raw_load<VEC>(v[t][m], x + col);
            }
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
            if (j0 + t < n && go) {
                go = keep(j0 + t);
                if (go) {
#pragma unroll
                    for (int m = 0; m < CH; ++m) {
                        const int col = (m * 64 + lane) * VEC;
                        if (col < d) {
#pragma unroll
                            for (int i = 0; i < VEC; ++i) acc[m][i] = fmaf(av[t], raw_get<VEC>(v[t][m], i), acc[m][i]);
                        }
                    }
                }
            }
        }
    }
}

template <int VEC, int CH> struct spmm_unroll { static constexpr int U = CH * VEC <= 1 ? 16 : (CH * VEC <= 4 ? 8 : (CH * VEC <= 8 ? 4 : 2)); };

// Wavefronts [0, n_piece_waves) take pieces of long rows (grid-stride over the pieces the plan
// lists) and write one partial row per piece; the others take blocks of rows_per_wave rows.
// A long row is finished by whichever of its piece wavefronts stores its partial row last: the
// partial row is written with device-scope stores, the wavefront waits for them to complete and
// draws a ticket of the row, and the holder of the last ticket reads all partial rows back with
// device-scope loads and adds them up in piece order - the same sum whoever does it.  That wavefront also puts the ticket counter
// back to zero for the next product with this plan.
template <int VEC, int CH, typename XT, bool XENT = false>
__global__ __launch_bounds__(SPMM_NT) void spmm_main_kernel(uint32_t rows, const void *__restrict__ rowptr, int rp64,
                                                            const int32_t *__restrict__ colidx,
                                                            const float *__restrict__ val, uint64_t capacity,
                                                            const XT *__restrict__ X, int64_t ldx,
                                                            const int32_t *__restrict__ row_index, int d,
                                                            unsigned n_piece_waves, const uint32_t *__restrict__ n_chunks,
                                                            uint32_t max_chunks, const uint2 *__restrict__ desc,
                                                            uint32_t *__restrict__ ticket, float *part, float *__restrict__ out,
                                                            int64_t ldo, spmm_epi ep, int rows_per_wave)
{
    constexpr int U = spmm_unroll<VEC, CH>::U;
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * (uint32_t)(SPMM_NT / 64) + (threadIdx.x >> 6);
    float bias[CH][VEC];
#pragma unroll
    for (int m = 0; m < CH; ++m)
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const int col = (m * 64 + lane) * VEC + i;
            bias[m][i] = (ep.bias && col < d) ? ep.bias[col] : 0.f;
        }
    const int64_t cap = (int64_t)min(capacity, (uint64_t)0x7fffffffffffffffull);
    spmm_xent_sums<VEC, CH> xs;
    xs.loss = 0.f;
#pragma unroll
    for (int m = 0; m < CH; ++m)
#pragma unroll
        for (int i = 0; i < VEC; ++i) xs.cs[m][i] = 0.f;
    // a finished row held as sum (bias not yet added): written, or with XENT turned into its loss and gradient row
    auto finish = [&](float (&sum)[CH][VEC], int64_t row, auto shared_row) {
        const int64_t orow = row * ldo;
        if constexpr (XENT) {
#pragma unroll
            for (int m = 0; m < CH; ++m)
#pragma unroll
                for (int i = 0; i < VEC; ++i) sum[m][i] += bias[m][i];
            spmm_row_xent<VEC, CH, decltype(shared_row)::value>(sum, ep, row, ep.labels[row], d, lane, xs);
        }
#pragma unroll
        for (int m = 0; m < CH; ++m) {
            const int col = (m * 64 + lane) * VEC;
            if (col < d) {
                if constexpr (XENT) {
                    if (ep.write_out) vstore_out<VEC>(out, orow + col, sum[m], 0);
                } else {
                    spmm_epilogue<VEC>(sum[m], ep, row, col, bias[m]);
                    vstore_out<VEC>(out, orow + col, sum[m], ep.out_bf16);
                }
            }
        }
    };
    if (wave < n_piece_waves) {
        const uint32_t total = min(*n_chunks, max_chunks);
        constexpr int PSTRIDE = CH * VEC * 64;
        // The partial row of a piece goes out with device-scope stores; once they have completed it is
        // visible to every wavefront of the device, and only then may the ticket be drawn.  Neither wait
        // is taken on the spot: the stores of piece k are waited for, and its ticket drawn, after piece
        // k+1 has been summed, and the number drawn is looked at after piece k+2 (the gathers of the
        // pieces in between hide both latencies).  `owed`: stored, ticket not drawn; `drawn`: ticket
        // requested, number not looked at yet.
        uint32_t owed_first = 0, owed_nch = 0, owed_row = 0;
        uint32_t drawn_first = 0, drawn_nch = 0, drawn_row = 0, drawn_t = 0;
        bool owed = false, drawn = false;
        auto draw_ticket = [&]() {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            drawn_t = 0;
            if (lane == 0) drawn_t = atomicAdd(&ticket[owed_first], 1u);
            drawn_first = owed_first; drawn_nch = owed_nch; drawn_row = owed_row;
            drawn = true; owed = false;
        };
        auto finish_row = [&]() {
            drawn = false;
            const uint32_t t = (uint32_t)__builtin_amdgcn_readfirstlane((int)drawn_t);
            if (t + 1 != drawn_nch) return;
            // last ticket: all partial rows of the row are complete; they are read with device-scope loads
            float sum[CH][VEC];
#pragma unroll
            for (int m = 0; m < CH; ++m)
#pragma unroll
                for (int i = 0; i < VEC; ++i) sum[m][i] = 0.f;
            const float *pr = part + (int64_t)drawn_first * PSTRIDE + lane;
            uint32_t c = 0;
            for (; c + U <= drawn_nch; c += U) {
                float v[U][CH][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int m = 0; m < CH; ++m) {
                        const int col = (m * 64 + lane) * VEC;
                        if (col < d) vload_device<VEC>(v[u][m], pr + (int64_t)(c + u) * PSTRIDE + m * VEC * 64);
                    }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int m = 0; m < CH; ++m) {
                        const int col = (m * 64 + lane) * VEC;
                        if (col < d) {
#pragma unroll
                            for (int i = 0; i < VEC; ++i) sum[m][i] += v[u][m][i];
                        }
                    }
            }
            for (; c < drawn_nch; ++c) {
#pragma unroll
                for (int m = 0; m < CH; ++m) {
                    const int col = (m * 64 + lane) * VEC;
                    if (col < d) {
                        float v[VEC];
                        vload_device<VEC>(v, pr + (int64_t)c * PSTRIDE + m * VEC * 64);
#pragma unroll
                        for (int i = 0; i < VEC; ++i) sum[m][i] += v[i];
                    }
                }
            }
            finish(sum, (int64_t)drawn_row, std::true_type{});      // finished by whoever came last: sums through the slots
            if (lane == 0) ticket[drawn_first] = 0;
        };
        for (uint32_t pc = wave; pc < total; pc += n_piece_waves) {
            const uint2 rc = desc[pc];
            const int64_t re = min(rp_load(rowptr, rp64, (uint64_t)rc.x + 1), cap);
            const int64_t rs = min(rp_load(rowptr, rp64, rc.x), re);
            const int64_t plen = spmm_piece_len(re - rs);
            const int64_t c0 = rs + (int64_t)rc.y * plen;
            const int64_t c1 = min(re, c0 + plen);
            float acc[CH][VEC];
#pragma unroll
            for (int m = 0; m < CH; ++m)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[m][i] = 0.f;
            for (int64_t cb = c0; cb < c1; cb += SPMM_CHUNK) {      // 64 entries at a time
                const int n = (int)min(c1 - cb, (int64_t)SPMM_CHUNK);
                int32_t src = 0;
                float a = 0.f;
                if (lane < n) {
                    const int32_t c = colidx[cb + lane];
                    a = val[cb + lane];
                    src = row_index ? row_index[c] : c;
                }
                spmm_wave_entries<VEC, CH, U, XT>(acc, src, a, n, X, ldx, d, lane, [](int) { return true; });
            }
            if (re - rs <= plen) {
                // the row's only piece: it is the row, written as the row-block wavefronts write theirs
                // With the loss epilogue its sums go the way of the rows shared between wavefronts (integer adds): the
                // numbering of the pieces depends on the timing of the plan kernel, so which wavefront gets this row does
                // too, and a float sum per wavefront would not come out the same bits twice.
                finish(acc, (int64_t)rc.x, std::integral_constant<bool, XENT>{});
                continue;
            }
            if (drawn) finish_row();
            if (owed) draw_ticket();
            // a partial row holds the words of the wavefront's registers in register order: word (m, i)
            // of lane l at (m * VEC + i) * 64 + l
            float *o = part + (int64_t)pc * PSTRIDE + lane;
#pragma unroll
            for (int m = 0; m < CH; ++m) {
                const int col = (m * 64 + lane) * VEC;
                if (col < d) vstore_device<VEC>(o + m * VEC * 64, acc[m]);
            }
            // pieces of this row that exist (the list may have been cut short at max_chunks)
            owed_first = pc - rc.y;
            owed_nch = min((uint32_t)((re - rs + plen - 1) / plen), total - owed_first);
            owed_row = rc.x;
            owed = true;
        }
        if (drawn) finish_row();
        if (owed) { draw_ticket(); finish_row(); }
    } else {
        // blocks of rows, grid-stride: the grid is capped (a launch holds fewer than 2^32 threads), a full graph
        // of 10^8 rows has more blocks than that
        const int rpw = n_chunks ? (int)n_chunks[2] : rows_per_wave;
        const int long_len = n_chunks ? (int)n_chunks[1] : 0x7fffffff;
        const uint64_t n_row_waves = (uint64_t)gridDim.x * (SPMM_NT / 64) - n_piece_waves;
        for (uint64_t w = wave - n_piece_waves; w * (uint64_t)rpw < rows; w += n_row_waves)
            spmm_wave_rows<VEC, CH, XT, XENT>(rows, rowptr, rp64, colidx, val, capacity, X, ldx, row_index, d, w, rpw, long_len, out,
                                              ldo, ep, bias, xs);
    }
    if constexpr (XENT) {
        // every wavefront of the workgroup arrives here (a workgroup is all pieces or all row blocks): its sums are
        // added in a fixed order and leave as the workgroup's partial loss and partial column sums
        __shared__ float xl[SPMM_NT / 64];
        __shared__ float xc[SPMM_NT / 64][CH * VEC * 64];
        const int wv = threadIdx.x >> 6;
        const float l = wave_sum(xs.loss);
        if (lane == 0) xl[wv] = l;
#pragma unroll
        for (int m = 0; m < CH; ++m)
#pragma unroll
            for (int i = 0; i < VEC; ++i) xc[wv][(m * VEC + i) * 64 + lane] = xs.cs[m][i];
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int w = 0; w < SPMM_NT / 64; ++w) t += xl[w];
            ep.loss_partial[blockIdx.x] = t;
        }
        if (ep.cs_partial) {
            for (int idx = threadIdx.x; idx < CH * VEC * 64; idx += SPMM_NT) {
                const int l2 = idx & 63, mi = idx >> 6, m = mi / VEC, i = mi % VEC;
                const int col = (m * 64 + l2) * VEC + i;
                if (col < d) {
                    float t = 0.f;
                    for (int w = 0; w < SPMM_NT / 64; ++w) t += xc[w][idx];
                    ep.cs_partial[(int64_t)blockIdx.x * d + col] = t;
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void spmm_xent_clear_kernel(unsigned long long *__restrict__ p, unsigned n)
{
    const unsigned i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

int build_plan(sgnn_ctx *ctx, const sgnn_csr *A, void *plan, hipStream_t st)
{
    const uint32_t max_chunks = spmm_max_chunks(A->rows, A->capacity);
    const spmm_plan_view pv = plan_view(plan, A->rows, max_chunks);
    SGNN_LAUNCH(ctx, st, "spmm_plan_clear_kernel", SGNN_TAG, spmm_plan_clear_kernel, dim3(1), dim3(1), 0, st, pv.n_chunks);
    SGNN_LAUNCH(ctx, st, "spmm_plan_kernel", SGNN_TAG, spmm_plan_kernel, dim3(cdiv(A->rows, SPMM_PLAN_NT)), dim3(SPMM_PLAN_NT), 0, st, A->rows,
                A->rowptr, A->rowptr_is_i64, A->capacity, pv.n_chunks, max_chunks, pv.part_base, pv.desc, pv.ticket);
    return SGNN_OK;
}

// XENT: the cross-entropy epilogue; loss_out / colsum_out receive the mean loss and the column sums of the gradient
template <int VEC, int CH, typename XT, bool XENT = false>
int launch_vc(sgnn_ctx *ctx, const sgnn_csr *A, const XT *X, int64_t ldx, const int32_t *row_index, int d, float *out,
              int64_t ldo, const spmm_epi &ep_in, ws_alloc *ws, hipStream_t st, float *loss_out = nullptr, float *colsum_out = nullptr)
{
    spmm_epi ep = ep_in;
    const int rows_per_wave = spmm_rows_per_wave(A->rows, A->capacity);   // lower bound of the plan's figure
    const unsigned rows_per_block = (unsigned)(SPMM_NT / 64) * (unsigned)rows_per_wave;
    char tag[56];
    if (XENT)
        snprintf(tag, sizeof(tag), "%ux%u d=%d <%d,%d> in=%d out=%d xent dO=%d", A->rows, A->cols, d, VEC, CH, (int)sizeof(XT),
                 ep.write_out ? 4 : 0, ep.dO ? (ep.dO_bf16 ? 2 : 4) : 0);
    else
        snprintf(tag, sizeof(tag), "%ux%u d=%d <%d,%d> in=%d out=%d%s", A->rows, A->cols, d, VEC, CH, (int)sizeof(XT), ep.out_bf16 ? 2 : 4,
                 ep.mask ? (ep.mask_bf16 ? " m=2" : " m=4") : "");
    const bool may_have_long = A->capacity > (uint64_t)SPMM_SHORT;
    spmm_plan_view pv = {nullptr, nullptr, nullptr, nullptr};
    float *part = nullptr;
    uint32_t max_chunks = 0;
    unsigned n_piece_waves = 0;
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
        pv = plan_view(plan, A->rows, max_chunks);
        part = ws->get<float>((size_t)max_chunks * (CH * VEC * 64));
        if (!ws->ok)
            return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_spmm: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                             ws->off);
        // wavefronts that take pieces: 2048, more for matrices with many entries (about 32 pieces of 64 entries
        // each if every entry sat in a long row); those that find no piece leave at once
        const uint64_t want = std::min<uint64_t>(std::max<uint64_t>(A->capacity / 2048, SPMM_PIECE_WAVES), 65536);
        n_piece_waves = cdiv(std::min<uint64_t>(max_chunks, want), SPMM_NT / 64) * (SPMM_NT / 64);
    }
    // The host sizes the grid from the capacity (the entry count is on the device), which for a sparse mini-batch is many
    // times the true count: most of the workgroups of such a launch would find no block of rows and leave at once, and
    // dispatching a quarter of a million of them cost a third of the kernel's time.  16384 workgroups fill the machine
    // several times over; the wavefronts stride over whatever is left.
    // (with the cross-entropy epilogue every workgroup leaves a row of partial sums for the final kernel: a quarter of that)
    const unsigned row_blocks = std::min<unsigned>(cdiv(A->rows, rows_per_block), XENT ? 4096u : 16384u);
    const unsigned grid = n_piece_waves / (SPMM_NT / 64) + row_blocks;
    if (XENT) {
        ep.loss_partial = ws->get<float>(grid);
        ep.cs_partial = colsum_out ? ws->get<float>((size_t)grid * d) : nullptr;
        ep.fix = ws->get<unsigned long long>((size_t)XENT_SLOTS * (d + 1));
        if (!ws->ok)
            return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_spmm_xent: scratch too small (%zu bytes needed): call sgnn_ctx_reserve", ws->off);
        const unsigned nfix = (unsigned)(XENT_SLOTS * (d + 1));
        SGNN_LAUNCH(ctx, st, "spmm_xent_clear_kernel", SGNN_TAG, spmm_xent_clear_kernel, dim3(cdiv(nfix, 256)), dim3(256), 0, st, ep.fix, nfix);
    }
    SGNN_LAUNCH(ctx, st, "spmm_main_kernel", tag, (spmm_main_kernel<VEC, CH, XT, XENT>), dim3(grid),
                dim3(SPMM_NT), 0, st, A->rows, A->rowptr, A->rowptr_is_i64, A->colidx, A->val, A->capacity, X, ldx, row_index, d,
                n_piece_waves, pv.n_chunks, max_chunks, pv.desc, pv.ticket, part, out, ldo, ep, rows_per_wave);
    if (XENT && (loss_out || colsum_out))
        return sgnn_launch_xent_final(ctx, ep.loss_partial, (int)grid, ep.inv_rows, loss_out, ep.cs_partial, d, colsum_out, ep.fix, XENT_SLOTS,
                                      1.0 / XENT_FIX_CS, 1.0 / XENT_FIX_LOSS, st);
    return SGNN_OK;
}

template <int VEC, typename XT>
int launch_v(sgnn_ctx *ctx, const sgnn_csr *A, const XT *X, int64_t ldx, const int32_t *row_index, int d, float *out,
             int64_t ldo, const spmm_epi &ep, ws_alloc *ws, hipStream_t st)
{
    const int per = (d + VEC - 1) / VEC;   // lanes needed for one pass over the row
    const int ch = (per + 63) / 64;
    switch (ch) {
    case 1: return launch_vc<VEC, 1, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 2: return launch_vc<VEC, 2, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 3: return launch_vc<VEC, 3, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 4: return launch_vc<VEC, 4, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 5: return launch_vc<VEC, 5, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 6: return launch_vc<VEC, 6, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 7: return launch_vc<VEC, 7, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    case 8: return launch_vc<VEC, 8, XT>(ctx, A, X, ldx, row_index, d, out, ldo, ep, ws, st);
    default: break;
    }
    return sgnn_fail(ctx, SGNN_ERR_UNSUPPORTED, "sgnn_spmm: feature width %d is beyond %d columns", d, 64 * 8 * VEC);
}

} // namespace

size_t sgnn_spmm_ws_bytes(uint64_t max_entries, uint32_t B, uint32_t d_max)
{
    // a plan built on the fly plus the partial rows, for the smallest long-row threshold
    const size_t max_chunks = spmm_max_chunks(B, max_entries);
    return max_chunks * (((size_t)d_max + 255) * sizeof(float) + 12) + (size_t)B * 4 + 5 * 256;
}

extern "C" uint64_t sgnn_csr_plan_bytes(uint32_t rows, uint64_t capacity)
{
    return 256 + (((uint64_t)rows * 4 + 255) & ~uint64_t(255)) + (uint64_t)spmm_max_chunks(rows, capacity) * 12 + 512;
}

int sgnn_launch_spmm_plan(sgnn_ctx *ctx, const sgnn_csr *A, hipStream_t st)
{
    if (!A->plan || A->rows == 0) return SGNN_OK;
    return build_plan(ctx, A, A->plan, st);
}

template <typename XT>
static int launch_x(sgnn_ctx *ctx, const sgnn_csr *A, const XT *X, int64_t ldx, const int32_t *row_index, int64_t d, float *out,
                    int64_t ldo, const spmm_epi &ep, ws_alloc *ws, hipStream_t st)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(ep.mask) |
                           reinterpret_cast<uintptr_t>(ep.add);
    // the narrowest vector with which one wavefront still covers the row
    const int64_t lds_ = ldx | ldo | (ep.mask ? ep.ldm : 0) | (ep.add ? ep.ldadd : 0);
    const bool ok4 = d % 4 == 0 && lds_ % 4 == 0 && (bits & 15) == 0;
    const bool ok2 = d % 2 == 0 && lds_ % 2 == 0 && (bits & 7) == 0;
    if (d <= 64) return launch_v<1, XT>(ctx, A, X, ldx, row_index, (int)d, out, ldo, ep, ws, st);
    if (d <= 128 && ok2) return launch_v<2, XT>(ctx, A, X, ldx, row_index, (int)d, out, ldo, ep, ws, st);
    if (ok4) return launch_v<4, XT>(ctx, A, X, ldx, row_index, (int)d, out, ldo, ep, ws, st);
    if (ok2) return launch_v<2, XT>(ctx, A, X, ldx, row_index, (int)d, out, ldo, ep, ws, st);
    return launch_v<1, XT>(ctx, A, X, ldx, row_index, (int)d, out, ldo, ep, ws, st);
}

// O = A X + bias with the softmax cross-entropy of O's rows in the epilogue (see spmm_row_xent).  Returns
// SGNN_ERR_UNSUPPORTED without launching anything for widths or alignments the fused kernels are not built for
// (more than 512 columns, rows that do not allow the vector width the column count asks for): the caller then
// runs the product and the loss kernel one after the other.
template <typename XT>
static int launch_xent_x(sgnn_ctx *ctx, const sgnn_csr *A, const XT *X, int64_t ldx, int64_t d, float *out, int64_t ldo,
                         const spmm_epi &ep, float *loss, float *colsum, ws_alloc *ws, hipStream_t st)
{
    // a lane moves VEC consecutive elements of X, of the logits (fp32) and of the gradient at once
    auto fits = [](const void *ptr, int64_t ld, int elem_bytes, int vec) {
        return !ptr || ((reinterpret_cast<uintptr_t>(ptr) % (uintptr_t)(vec * elem_bytes)) == 0 && ld % vec == 0);
    };
    auto ok = [&](int vec) {
        return d % vec == 0 && fits(X, ldx, (int)sizeof(XT), vec) && fits(ep.write_out ? out : nullptr, ldo, 4, vec) &&
               fits(ep.dO, ep.lddo, ep.dO_bf16 ? 2 : 4, vec);
    };
    const bool ok4 = ok(4), ok2 = ok(2);
    if (d <= 64) return launch_vc<1, 1, XT, true>(ctx, A, X, ldx, nullptr, (int)d, out, ldo, ep, ws, st, loss, colsum);
    if (d <= 128 && ok2) return launch_vc<2, 1, XT, true>(ctx, A, X, ldx, nullptr, (int)d, out, ldo, ep, ws, st, loss, colsum);
    if (d <= 256 && ok4) return launch_vc<4, 1, XT, true>(ctx, A, X, ldx, nullptr, (int)d, out, ldo, ep, ws, st, loss, colsum);
    if (d <= 512 && ok4) return launch_vc<4, 2, XT, true>(ctx, A, X, ldx, nullptr, (int)d, out, ldo, ep, ws, st, loss, colsum);
    return SGNN_ERR_UNSUPPORTED;
}

int sgnn_launch_spmm_xent(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, int64_t d, const float *bias,
                          const int32_t *labels, float *out, int64_t ldo, float *loss, void *dO, int dO_bf16, int64_t lddo,
                          float *dO_colsum, ws_alloc *ws, hipStream_t st)
{
    spmm_epi ep = {};
    ep.bias = bias;
    ep.labels = labels;
    ep.dO = dO; ep.dO_bf16 = dO_bf16 ? 1 : 0; ep.lddo = lddo;
    ep.inv_rows = 1.f / (float)A->rows;
    ep.write_out = out ? 1 : 0;
    if (x_bf16) return launch_xent_x(ctx, A, static_cast<const bf16_bits *>(X), ldx, d, out, ldo, ep, loss, dO_colsum, ws, st);
    return launch_xent_x(ctx, A, static_cast<const float *>(X), ldx, d, out, ldo, ep, loss, dO_colsum, ws, st);
}

// X: cols x d, fp32 or (x_bf16) bfloat16 bit patterns, leading dimension ldx in elements
int sgnn_launch_spmm(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, const int32_t *row_index, int64_t d,
                     float *out, int64_t ldo, const float *bias, int relu, const float *mask, int64_t ldm, const float *add,
                     int64_t ldadd, ws_alloc *ws, hipStream_t st)
{
    return sgnn_launch_spmm_x(ctx, A, X, x_bf16, ldx, row_index, d, out, 0, ldo, bias, relu, mask, 0, ldm, add, ldadd, ws, st);
}

// The same with the result (out_bf16) and the mask (mask_bf16) optionally stored as bfloat16; their leading
// dimensions are in elements.
int sgnn_launch_spmm_x(sgnn_ctx *ctx, const sgnn_csr *A, const void *X, int x_bf16, int64_t ldx, const int32_t *row_index, int64_t d,
                       void *out, int out_bf16, int64_t ldo, const float *bias, int relu, const void *mask, int mask_bf16,
                       int64_t ldm, const float *add, int64_t ldadd, ws_alloc *ws, hipStream_t st)
{
    const spmm_epi ep = {bias, relu, static_cast<const float *>(mask), ldm, add, ldadd, out_bf16 ? 1 : 0, (mask && mask_bf16) ? 1 : 0};
    if (A->rows == 0 || d == 0) return SGNN_OK;
    if (x_bf16) return launch_x(ctx, A, static_cast<const bf16_bits *>(X), ldx, row_index, d, static_cast<float *>(out), ldo, ep, ws, st);
    return launch_x(ctx, A, static_cast<const float *>(X), ldx, row_index, d, static_cast<float *>(out), ldo, ep, ws, st);
}
