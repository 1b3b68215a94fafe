// Induced, normalised, rescaled mini-batch subgraph as CSR (Sec. III-D, Eqs. 21-24; the full-range
// case of Algorithm 2).
//
// The sampled rows of the full CSR are treated as one flat edge sequence of length
// F = sum_{v in S} deg(v), cut into tiles of 2048 edges, one workgroup per tile, so the work per
// workgroup does not depend on the degree distribution (a hub row of 10^5 edges is spread over
// many workgroups; thousands of short rows share one).  Membership of a column in S is one bit
// test in the sampler's bitmap; its compact id is the sampler's rank prefix plus a popcount.
// Because the output CSR is in the same order as the flat sequence, the output position of a
// surviving edge is (survivors in earlier tiles) + (survivors before it inside the tile):
//
//   1. induced_deg_kernel      row length of every sampled row and per-workgroup sums
//   2. induced_offsets_kernel  flat offsets P[B+1] (exclusive prefix of the row lengths)
//   3. induced_count_kernel    survivors per tile (wave ballots / popcounts)
//   4. prefix sum              survivors in earlier tiles, for every tile
//   5. induced_fill_kernel     survivors only (keep words of pass 3): ordered compaction, colidx, val, rowptr
//   6. induced_renorm_kernel   only for norm_mode 1: weights from the degrees of the induced graph
// A tile stages the starts of the rows it touches in LDS, so finding the row of an edge is a
// binary search in LDS, and the whole tile needs one barrier for its ordered compaction.
#include <algorithm>

#include "block_prims.h"
#include "common.h"

namespace {

constexpr int IND_NT = 256;
constexpr int IND_ITEMS = 8;
constexpr int IND_TILE = IND_NT * IND_ITEMS;      // 2048 flat edges per workgroup (4096 and 8192 with 512 threads measured slower)
constexpr int IND_WORDS = IND_ITEMS * (IND_NT / 64);   // 64-bit keep words of a tile: one per slab and wavefront
constexpr int IND_ROWS = 512;                     // rows a tile's LDS table holds (more only when rows average under 4 edges): 6 KB, so LDS does not limit occupancy
#ifndef IND_FILL_SLOTS
#define IND_FILL_SLOTS 2                          // survivors a thread of the fill pass works on at a time
#endif
constexpr unsigned IND_MAX_GRID = 8192;
constexpr int DEG_TILE = 2048;                    // sampled rows per workgroup in the offset kernels

// Row and column range of a shard (Algorithm 2: [R0, R1) x [C0, C1) in global vertex ids); the whole graph by default.
struct shard_range { int64_t r0, r1, c0, c1; };

template <class RP>
__global__ __launch_bounds__(256) void induced_deg_kernel(const RP *__restrict__ rowptr, const int32_t *__restrict__ S,
                                                          uint32_t B, shard_range rg, uint32_t *__restrict__ deg,
                                                          int64_t *__restrict__ rowstart, uint64_t *__restrict__ wg_sum,
                                                          unsigned long long *__restrict__ total64)
{
    __shared__ uint64_t lds[256 / 64];
    if (blockIdx.x == 0 && threadIdx.x == 0) *total64 = 0ull;     // survivors of the whole mini-batch, summed by the count pass
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < DEG_TILE / 256; ++k) {
        const uint32_t i = blockIdx.x * DEG_TILE + k * 256 + threadIdx.x;
        if (i < B) {
            const int64_t v = S[i];
            // a sampled row outside the shard's row range contributes no edge: it comes out as an empty row
            const int64_t rs = (int64_t)rowptr[v];
            const uint32_t dgr = (v >= rg.r0 && v < rg.r1) ? (uint32_t)((int64_t)rowptr[v + 1] - rs) : 0u;
            deg[i] = dgr;
            rowstart[i] = rs;      // kept for the tile kernels: no second gather through S
            s += dgr;
        }
    }
    const uint64_t t = block_sum<uint64_t, 256>(s, lds);
    if (threadIdx.x == 0) wg_sum[blockIdx.x] = t;
}

// Also tells every tile of IND_TILE flat edges which row its first edge belongs to: the row that covers the
// flat offset c * IND_TILE writes its number to tile_row[c] (a hub row covers many tile starts, most rows
// none), so that the tile kernels need no search for their first row.
__global__ __launch_bounds__(256) void induced_offsets_kernel(const uint32_t *__restrict__ deg, uint32_t B,
                                                              const uint64_t *__restrict__ wg_sum,
                                                              uint64_t *__restrict__ P, uint32_t *__restrict__ tile_row)
{
    __shared__ uint64_t lds[256 / 64 + 1];
    uint64_t part = 0;
    for (unsigned i = threadIdx.x; i < blockIdx.x; i += 256) part += wg_sum[i];
    const uint64_t base = block_sum<uint64_t, 256>(part, lds);
    // blocked arrangement: thread t owns rows i0 .. i0+7
    const uint32_t i0 = blockIdx.x * DEG_TILE + threadIdx.x * (DEG_TILE / 256);
    uint32_t d[DEG_TILE / 256];
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < DEG_TILE / 256; ++k) {
        d[k] = (i0 + k < B) ? deg[i0 + k] : 0u;
        s += d[k];
    }
    uint64_t total;
    uint64_t ex = block_excl_scan<uint64_t, 256>(s, &total, lds) + base;
#pragma unroll
    for (int k = 0; k < DEG_TILE / 256; ++k) {
        if (i0 + k < B) {
            P[i0 + k] = ex;
            for (uint64_t c = (ex + IND_TILE - 1) / IND_TILE; c * IND_TILE < ex + d[k]; ++c) tile_row[c] = i0 + k;
        }
        ex += d[k];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) P[B] = base + total;
}

// Coarse membership filter for sparse samples of large graphs: one byte per bitmap word, bit b set iff byte b of the
// word holds a sampled vertex (1 bit per 8 vertices).  With a sample of 1 % of 10^8 vertices the 14 MB bitmap does not
// stay in a 4 MB L2 and every edge's probe is a cache-line fetch from further away; the filter (N / 64 bytes) does stay,
// and turns away the 93 % of the edges whose eight-vertex group holds no sampled vertex at all.
__global__ __launch_bounds__(256) void induced_coarse_kernel(const uint64_t *__restrict__ bitmap, uint64_t W,
                                                             uint8_t *__restrict__ coarse)
{
    for (uint64_t w = (uint64_t)blockIdx.x * 256 + threadIdx.x; w < W; w += (uint64_t)gridDim.x * 256) {
        const uint64_t x = bitmap[w];
        uint32_t c = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) c |= ((x >> (8 * b)) & 0xffull) ? (1u << b) : 0u;
        coarse[w] = (uint8_t)c;
    }
}

// largest r in [lo, hi] with P[r] <= f   (P[lo] <= f is guaranteed by the caller)
__device__ __forceinline__ uint32_t find_row(const uint64_t *__restrict__ P, uint32_t lo, uint32_t hi, uint64_t f)
{
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (P[mid] <= f) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Per-tile row table in LDS.  Rows r_lo .. r_lo+nr-1 intersect the tile [f0, f1).
//   relP[k]  = P[r_lo+k] - f0, clamped to -1 when the row starts before the tile
//   ebase[k] = rowptr[S[r]] - P[r]: the position in colidx of flat edge f of that row is ebase + f
// staged == false (more rows than the table holds: rows averaging under four edges, or the run of empty
// rows behind the last tile of a shard) falls back to searching P in global memory.
struct tile_table {
    int32_t relP[IND_ROWS + 1];
    int64_t ebase[IND_ROWS + 1];
};

// Rows r_lo .. r_lo + nr - 1 of a tile: from the row of its first edge to the row of the first edge of the next
// tile (which holds the tile's last edge, or starts right behind it and is then never found by the search);
// the last tile takes every row up to the last one.
__device__ __forceinline__ void tile_rows(const uint32_t *__restrict__ tile_row, uint64_t c, uint64_t n_tiles, uint32_t B,
                                          uint32_t &r_lo, uint32_t &nr)
{
    r_lo = c ? tile_row[c] : 0;        // the first tile also takes the empty rows in front of the first edge
    const uint32_t r_hi = c + 1 < n_tiles ? tile_row[c + 1] : B - 1;
    nr = r_hi - r_lo + 1;
}

// Staging of a tile's row table.  The first IND_NT rows arrive in registers: (p, rs) of row r_lo + threadIdx.x, requested
// while the tile before this one was being worked on (tile_prefetch), so that the two round trips that fetch a
// tile's rows - tile_row, then P / row starts - are off its critical path.
struct tile_pref {
    uint64_t p;
    int64_t rs;
};

__device__ __forceinline__ tile_pref tile_prefetch(const int64_t *__restrict__ rowstart, const uint64_t *__restrict__ P,
                                                   bool valid, uint32_t r_lo, uint32_t nr)
{
    tile_pref t = {0, 0};
    if (valid && threadIdx.x < nr && nr <= (uint32_t)IND_ROWS + 1) {
        t.p = P[r_lo + threadIdx.x];
        t.rs = rowstart[r_lo + threadIdx.x];
    }
    return t;
}

__device__ __forceinline__ bool stage_tile_prefetched(tile_table &tt, const tile_pref &pf, const int64_t *__restrict__ rowstart,
                                                      const uint64_t *__restrict__ P, uint64_t f0, uint32_t r_lo, uint32_t nr)
{
    const bool staged = nr <= (uint32_t)IND_ROWS + 1;
    if (staged) {
        for (uint32_t k = threadIdx.x; k < nr; k += IND_NT) {
            const uint64_t p = k < IND_NT ? pf.p : P[r_lo + k];
            const int64_t rs = k < IND_NT ? pf.rs : rowstart[r_lo + k];
            const int64_t rel = (int64_t)p - (int64_t)f0;      // signed on purpose: the row may start in front of the tile
            tt.relP[k] = rel < 0 ? -1 : (rel > IND_TILE ? IND_TILE : (int32_t)rel);
            tt.ebase[k] = rs - (int64_t)p;
        }
    }
    __syncthreads();
    return staged;
}

// index k of the row of flat offset x = f - f0 >= 0: largest k < nr with relP[k] <= x
__device__ __forceinline__ uint32_t find_row_lds(const tile_table &tt, uint32_t nr, int32_t x)
{
    uint32_t lo = 0, hi = nr - 1;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (tt.relP[mid] <= x) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// The same search for the edges of a thread at once, in lock step with a fixed number of rounds,
// so that the LDS reads of the slabs are in flight together (x[k] < 0: no edge, the result is unused).
template <int ITEMS>
__device__ __forceinline__ void find_rows_lds(const tile_table &tt, uint32_t nr, const int32_t (&x)[ITEMS], uint32_t (&rk)[ITEMS])
{
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) rk[k] = 0;
    for (uint32_t step = 1u << (31 - __clz((int)nr)); step; step >>= 1) {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            // the read is unconditional (of the last row where t is beyond it), so that the compiler issues the reads
            // of a round together instead of branching round each one and waiting for it
            const uint32_t t = rk[k] + step;
            const int32_t start = tt.relP[min(t, nr - 1)];
            rk[k] = (t < nr && start <= x[k]) ? t : rk[k];
        }
    }
}

__global__ __launch_bounds__(IND_NT) void induced_count_kernel(const int64_t *__restrict__ rowstart,
                                                               const int32_t *__restrict__ colidx, uint32_t B,
                                                               const uint64_t *__restrict__ bitmap,
                                                               const uint8_t *__restrict__ coarse, shard_range rg,
                                                               const uint64_t *__restrict__ P,
                                                               const uint32_t *__restrict__ tile_row,
                                                               uint32_t *__restrict__ tile_total,
                                                               uint64_t *__restrict__ keepbits,
                                                               uint64_t *__restrict__ n_tiles_out,
                                                               unsigned long long *__restrict__ total64)
{
    __shared__ tile_table tt;
    __shared__ uint32_t lds[IND_NT / 64];
    const unsigned lane = lane_id(), wave = threadIdx.x >> 6;
    const uint64_t F = P[B];
    const uint64_t n_tiles = (F + IND_TILE - 1) / IND_TILE;
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_tiles_out = n_tiles;
    unsigned long long wg_total = 0;      // 64 bits: the 32-bit prefix over the tile counts wraps beyond 2^32 survivors
    // software pipeline over the workgroup's tiles: the rows of the tile after next and the table of the next tile are
    // requested before the current tile's edges are gathered
    const uint64_t g = gridDim.x;
    uint32_t r_lo = 0, nr = 0, r_lo1 = 0, nr1 = 0;
    if (blockIdx.x < n_tiles) tile_rows(tile_row, blockIdx.x, n_tiles, B, r_lo, nr);
    if (blockIdx.x + g < n_tiles) tile_rows(tile_row, blockIdx.x + g, n_tiles, B, r_lo1, nr1);
    tile_pref pf = tile_prefetch(rowstart, P, blockIdx.x < n_tiles, r_lo, nr);
    for (uint64_t c = blockIdx.x; c < n_tiles; c += g) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const bool staged = stage_tile_prefetched(tt, pf, rowstart, P, f0, r_lo, nr);
        uint32_t r_lo2 = 0, nr2 = 0;
        if (c + 2 * g < n_tiles) tile_rows(tile_row, c + 2 * g, n_tiles, B, r_lo2, nr2);
        pf = tile_prefetch(rowstart, P, c + g < n_tiles, r_lo1, nr1);
        int32_t x[IND_ITEMS], u[IND_ITEMS];
        uint32_t rk[IND_ITEMS];
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t f = f0 + (uint64_t)k * IND_NT + threadIdx.x;
            x[k] = f < f1 ? (int32_t)(f - f0) : -1;
        }
        if (staged) {
            // Branch-free, one step for all eight edges at a time: the eight gathers of colidx are then in flight together
            // (with a branch round each edge the compiler waits for every load before it issues the next: eight round
            // trips per tile instead of one).  An offset behind the end of the last tile reads the tile's first edge.
            find_rows_lds(tt, nr, x, rk);
            int64_t e[IND_ITEMS];
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k) e[k] = tt.ebase[rk[k]] + (int64_t)(f0 + (uint64_t)max(x[k], 0));
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k) u[k] = colidx[e[k]];
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k)
                if (x[k] < 0 || u[k] < rg.c0 || u[k] >= rg.c1) u[k] = -1;   // no edge, or a column outside the shard
        } else {
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k) {
                u[k] = -1;
                if (x[k] >= 0) {
                    const uint64_t f = f0 + (uint64_t)x[k];
                    const uint32_t r = find_row(P, r_lo, r_lo + nr - 1, f);
                    u[k] = colidx[rowstart[r] + (int64_t)(f - P[r])];
                    if (u[k] < rg.c0 || u[k] >= rg.c1) u[k] = -1;   // a column outside the shard
                }
            }
        }
        uint64_t word[IND_ITEMS];
        if (coarse) {
            // the filter first (all eight probes in flight), the bitmap only for the edges it lets through
            uint8_t cf[IND_ITEMS];
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k) cf[k] = u[k] >= 0 ? coarse[(uint32_t)u[k] >> 6] : (uint8_t)0;
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k)
                word[k] = ((cf[k] >> (((uint32_t)u[k] >> 3) & 7)) & 1) ? bitmap[(uint32_t)u[k] >> 6] : 0ull;
        } else {
#pragma unroll
            for (int k = 0; k < IND_ITEMS; ++k) word[k] = u[k] >= 0 ? bitmap[(uint32_t)u[k] >> 6] : 0ull;
        }
        // one keep word per slab and wavefront, kept for the fill pass; the count is their popcount
        uint32_t cnt = 0;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t bal = __ballot(u[k] >= 0 && ((word[k] >> (u[k] & 63)) & 1ull));
            if (lane == 0) {
                keepbits[c * IND_WORDS + k * (IND_NT / 64) + wave] = bal;
                cnt += (uint32_t)__popcll(bal);
            }
        }
        const uint32_t t = block_sum<uint32_t, IND_NT>(cnt, lds);   // ends with a barrier: tt may be reused
        if (threadIdx.x == 0) { tile_total[c] = t; wg_total += t; }
        r_lo = r_lo1; nr = nr1; r_lo1 = r_lo2; nr1 = nr2;
    }
    if (threadIdx.x == 0 && wg_total) atomicAdd(total64, wg_total);     // integer: the sum does not depend on the order
}

// Fill pass.  The keep words of the count pass say which edges survive, so only survivors are looked at again:
// position = survivors in earlier tiles + survivors before the edge in the tile (prefix over the popcounts of
// the tile's keep words).  Row offsets come from the row side: every row that starts inside the tile gets the
// position of the first survivor at or behind its start, which also covers rows without any stored entry.
template <class RP>
__global__ __launch_bounds__(IND_NT) __attribute__((amdgpu_waves_per_eu(8, 8))) void induced_fill_kernel(
    const RP *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *__restrict__ gval,
    const int32_t *__restrict__ S, const int64_t *__restrict__ rowstart, const uint32_t *__restrict__ deg, uint32_t B,
    const uint64_t *__restrict__ bitmap, const uint32_t *__restrict__ rank, const uint64_t *__restrict__ P,
    const uint32_t *__restrict__ tile_row, const uint32_t *__restrict__ tile_off_all, const uint64_t *__restrict__ n_tiles_p, const uint64_t *__restrict__ keepbits, float inv_p, int write_val,
    int32_t *__restrict__ rowptr_S, int32_t *__restrict__ colidx_S, float *__restrict__ val_S, uint64_t capacity,
    uint32_t *__restrict__ nnz_dev, uint32_t *__restrict__ status, const unsigned long long *__restrict__ total64,
    int sticky_capacity, int deg_by_rank)
{
    __shared__ tile_table tt;
    __shared__ uint64_t balw[IND_WORDS];
    __shared__ uint32_t pre[IND_WORDS + 1];
    __shared__ uint16_t xs[IND_TILE];
    const uint64_t F = P[B];
    const uint64_t n_tiles = *n_tiles_p;
    const unsigned lane = lane_id(), wave = threadIdx.x >> 6;
    if (blockIdx.x == 0) {
        const uint32_t total = tile_off_all[n_tiles];
        if (threadIdx.x == 0) {
            const unsigned long long t64 = *total64;
            if (t64 > 0x7fffffffull) atomicOr(status, SGNN_ST_NNZ_OVERFLOW);
            // entries beyond the capacity are dropped below: without a host read-back of the count the caller learns
            // of it through the sticky status word (sgnn_ctx_status)
            if (sticky_capacity && t64 > capacity) atomicOr(status, SGNN_ST_CAPACITY_OVERFLOW);
            rowptr_S[B] = (int32_t)total;
            if (nnz_dev) *nnz_dev = total;
        }
        if (n_tiles == 0)       // not a single edge: every row is empty
            for (uint32_t r = threadIdx.x; r < B; r += IND_NT) rowptr_S[r] = 0;
    }
    // software pipeline over the workgroup's tiles, as in the count pass: the next tile's keep words, offset and row
    // table are requested while the current tile's survivors are gathered
    const uint64_t g = gridDim.x;
    uint32_t r_lo = 0, nr = 0, r_lo1 = 0, nr1 = 0;
    if (blockIdx.x < n_tiles) tile_rows(tile_row, blockIdx.x, n_tiles, B, r_lo, nr);
    if (blockIdx.x + g < n_tiles) tile_rows(tile_row, blockIdx.x + g, n_tiles, B, r_lo1, nr1);
    tile_pref pf = tile_prefetch(rowstart, P, blockIdx.x < n_tiles, r_lo, nr);
    uint64_t kw = 0;               // wavefront 0: keep word `lane` of the tile
    uint32_t tile_off = 0;         // survivors in earlier tiles (exclusive prefix of the tile counts)
    if (blockIdx.x < n_tiles) {
        if (wave == 0 && lane < IND_WORDS) kw = keepbits[(uint64_t)blockIdx.x * IND_WORDS + lane];
        tile_off = tile_off_all[blockIdx.x];
    }
    for (uint64_t c = blockIdx.x; c < n_tiles; c += g) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const uint32_t tile_len = (uint32_t)(f1 - f0);
        const bool last = c + 1 == n_tiles;
        if (wave == 0) {
            const uint64_t w = lane < IND_WORDS ? kw : 0ull;
            if (lane < IND_WORDS) balw[lane] = w;
            const uint32_t pc = (uint32_t)__popcll(w);
            const uint32_t inc = wave_incl_scan(pc);
            if (lane < IND_WORDS) pre[lane] = inc - pc;
            if (lane == IND_WORDS - 1) pre[IND_WORDS] = inc;
        }
        const bool staged = stage_tile_prefetched(tt, pf, rowstart, P, f0, r_lo, nr);     // ends with a barrier
        const uint32_t tile_off_cur = tile_off;
        uint32_t r_lo2 = 0, nr2 = 0;
        if (c + 2 * g < n_tiles) tile_rows(tile_row, c + 2 * g, n_tiles, B, r_lo2, nr2);
        pf = tile_prefetch(rowstart, P, c + g < n_tiles, r_lo1, nr1);
        if (c + g < n_tiles) {
            if (wave == 0 && lane < IND_WORDS) kw = keepbits[(c + g) * IND_WORDS + lane];
            tile_off = tile_off_all[c + g];
        }

        // row offsets.  A row that starts right at the end of the tile is empty if it is not the row the next
        // tile begins with (that tile writes that one); behind the last tile every such row is empty.
        for (uint32_t k = threadIdx.x; k < nr; k += IND_NT) {
            int64_t x;
            if (staged) x = tt.relP[k];
            else {
                const int64_t rel = (int64_t)P[r_lo + k] - (int64_t)f0;
                x = rel < 0 ? -1 : (rel > IND_TILE ? IND_TILE : rel);
            }
            if (x < 0) continue;
            if (x < (int64_t)tile_len) {
                const uint32_t wd = ((uint32_t)x / IND_NT) * (IND_NT / 64) + (((uint32_t)x % IND_NT) >> 6);
                rowptr_S[r_lo + k] = (int32_t)(tile_off_cur + pre[wd] + (uint32_t)__popcll(balw[wd] & ((1ull << (x & 63)) - 1ull)));
            } else if (x == (int64_t)tile_len && (last || k + 1 < nr)) rowptr_S[r_lo + k] = (int32_t)(tile_off_cur + pre[IND_WORDS]);
        }

        // Survivors, in their order: the flat offsets of the set bits of the keep words are written to a list in LDS, and
        // thread i takes survivor i, i + 256, ... (IND_FILL_SLOTS of them at a time).  A thread then holds the state of a few
        // survivors instead of one slot for each of its eight edges, of which one in eight survives on a typical
        // mini-batch: half the registers, twice the tiles in flight on a compute unit.
        const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint32_t wd = k * (IND_NT / 64) + wave;
            const uint64_t w = balw[wd];
            if ((w >> lane) & 1ull) xs[pre[wd] + (uint32_t)__popcll(w & below)] = (uint16_t)(k * IND_NT + threadIdx.x);
        }
        __syncthreads();
        const uint32_t n_surv = pre[IND_WORDS];
        for (uint32_t i0 = 0; i0 < n_surv; i0 += IND_FILL_SLOTS * IND_NT) {
            int32_t x[IND_FILL_SLOTS], u[IND_FILL_SLOTS];
            uint32_t rk[IND_FILL_SLOTS];
#pragma unroll
            for (int k = 0; k < IND_FILL_SLOTS; ++k) {
                const uint32_t i = i0 + k * IND_NT + threadIdx.x;
                x[k] = i < n_surv ? (int32_t)xs[i] : -1;
            }
            if (staged) find_rows_lds(tt, nr, x, rk);
            int64_t eidx[IND_FILL_SLOTS];
#pragma unroll
            for (int k = 0; k < IND_FILL_SLOTS; ++k) {
                u[k] = -1; eidx[k] = 0;
                if (x[k] >= 0) {
                    const uint64_t f = f0 + (uint64_t)x[k];
                    if (staged) eidx[k] = tt.ebase[rk[k]] + (int64_t)f;
                    else {
                        const uint32_t r = find_row(P, r_lo, r_lo + nr - 1, f);
                        rk[k] = r - r_lo;
                        eidx[k] = rowstart[r] + (int64_t)(f - P[r]);
                    }
                    u[k] = colidx[eidx[k]];
                }
            }
            uint64_t word[IND_FILL_SLOTS];
            uint32_t rnk[IND_FILL_SLOTS];
            int64_t du[IND_FILL_SLOTS];
#pragma unroll
            for (int k = 0; k < IND_FILL_SLOTS; ++k) {
                word[k] = 0; rnk[k] = 0; du[k] = 1;
                if (u[k] >= 0) {
                    word[k] = bitmap[(uint32_t)u[k] >> 6];
                    rnk[k] = rank[(uint32_t)u[k] >> 6];
                    if (write_val && !gval && !deg_by_rank) du[k] = (int64_t)rowptr[(int64_t)u[k] + 1] - (int64_t)rowptr[u[k]];
                }
            }
            // compact column ids; a surviving column is itself a sampled vertex, so with every sampled row inside the row
            // range its degree is already in deg[] (B entries, cache resident) and need not be gathered from rowptr
            uint32_t cid[IND_FILL_SLOTS];
#pragma unroll
            for (int k = 0; k < IND_FILL_SLOTS; ++k) {
                cid[k] = rnk[k] + (uint32_t)__popcll(word[k] & ((1ull << (u[k] & 63)) - 1ull));
                if (u[k] >= 0 && write_val && !gval && deg_by_rank) du[k] = (int64_t)deg[min(cid[k], B - 1)];
            }
#pragma unroll
            for (int k = 0; k < IND_FILL_SLOTS; ++k) {
                if (u[k] < 0) continue;
                const uint32_t pos = tile_off_cur + i0 + k * IND_NT + threadIdx.x;
                if (pos >= capacity) continue;
                colidx_S[pos] = (int32_t)cid[k];
                if (write_val) {
                    const uint32_t r = r_lo + rk[k];
                    const int64_t v = S[r];
                    float a;
                    if (gval) a = gval[eidx[k]];
                    else {
                        // 1 / sqrt(deg(v) deg(u)) in single precision: product, reciprocal square root, one Newton step.
                        // Against the double-precision formula rounded once: a few 1e-7 relative (two roundings of
                        // 2^-24 here, one for 1/p, the Newton step leaves under one more), inside the 1e-6 the weights are held to.
                        // A row that holds an edge lies inside the row range: deg is its full length.
                        const float xx = (float)deg[r] * (float)du[k];
                        float y = __frsqrt_rn(xx);
                        const float err = fmaf(-xx * y, y, 1.0f);
                        a = fmaf(0.5f * y, err, y);
                    }
                    if ((int64_t)u[k] != v) a *= inv_p;
                    val_S[pos] = a;
                }
            }
        }
        __syncthreads();   // the keep words and the row table are reused by the next tile
        r_lo = r_lo1; nr = nr1; r_lo1 = r_lo2; nr1 = nr2;
    }
}

// norm_mode 1: a_ij = 1/sqrt(c_i c_j) with c = entry counts of the induced rows, off-diagonal / p.
__global__ __launch_bounds__(256) void induced_renorm_kernel(const int32_t *__restrict__ rowptr_S,
                                                             const int32_t *__restrict__ colidx_S,
                                                             float *__restrict__ val_S, uint32_t B, uint64_t capacity,
                                                             double p)
{
    // a wavefront per row
    const uint32_t row = (blockIdx.x * 256 + threadIdx.x) >> 6;
    if (row >= B) return;
    const int64_t rs = rowptr_S[row], re = min((int64_t)rowptr_S[row + 1], (int64_t)capacity);
    const double ci = (double)(rowptr_S[row + 1] - rowptr_S[row]);
    for (int64_t e = rs + lane_id(); e < re; e += 64) {
        const int32_t j = colidx_S[e];
        const double cj = (double)(rowptr_S[j + 1] - rowptr_S[j]);
        double a = 1.0 / sqrt(ci * cj);
        if ((uint32_t)j != row) a /= p;
        val_S[e] = (float)a;
    }
}

template <class RP>
int launch_typed(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                 const uint32_t *rank, int norm_mode, int rescale, shard_range rg, sgnn_csr *out, int sticky_capacity,
                 hipStream_t st)
{
    const RP *rowptr = static_cast<const RP *>(g->rowptr);
    ws_alloc ws(ctx);
    const uint64_t max_tiles = g->E / IND_TILE + 2;
    const unsigned n_deg_wg = cdiv(B, DEG_TILE);
    uint32_t *deg = ws.get<uint32_t>(B);
    int64_t *rowstart = ws.get<int64_t>(B);
    uint64_t *deg_sum = ws.get<uint64_t>(n_deg_wg);
    uint64_t *P = ws.get<uint64_t>((size_t)B + 1);
    uint32_t *tile_total = ws.get<uint32_t>(max_tiles);
    uint32_t *tile_row = ws.get<uint32_t>(max_tiles + 1);
    uint64_t *keepbits = ws.get<uint64_t>(max_tiles * IND_WORDS);
    uint32_t *tile_off = ws.get<uint32_t>(max_tiles + 1);
    uint32_t *scan_tmp = ws.get<uint32_t>(sgnn_scan_tmp_elems(max_tiles));
    uint64_t *n_tiles = ws.get<uint64_t>(1);
    unsigned long long *total64 = ws.get<unsigned long long>(1);
    // the coarse filter pays when the bitmap is far larger than an L2 and the sample is sparse
    const uint64_t W = (g->N + 63) / 64;
    const bool use_coarse = g->N >= (1ull << 24) && (uint64_t)B * 32 < g->N;
    uint8_t *coarse = use_coarse ? ws.get<uint8_t>(W) : nullptr;
    if (!ws.ok)
        return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_induced_csr: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                         ws.off);

    SGNN_LAUNCH(ctx, st, "induced_deg_kernel", SGNN_TAG, induced_deg_kernel<RP>, dim3(n_deg_wg), dim3(256), 0, st, rowptr, S, B,
                rg, deg, rowstart, deg_sum, total64);
    SGNN_LAUNCH(ctx, st, "induced_offsets_kernel", SGNN_TAG, induced_offsets_kernel, dim3(n_deg_wg), dim3(256), 0, st, deg, B,
                deg_sum, P, tile_row);
    // Workgroups walk their tiles in a software pipeline (the next tile's row table is requested while the current
    // tile's edges are gathered).  Where the expected number of tiles, E B / N / 2048, is a few times the 2048
    // workgroups of the count pass that are resident at once, exactly those are launched (large graph: 94 -> 78 us);
    // with more tiles the larger grid measured better (the chip is then full anyway), as it does for the fill pass.
    const uint64_t expected_tiles = (uint64_t)((double)g->E * (double)B / (double)std::max<uint64_t>(g->N, 1) / IND_TILE);
    const unsigned grid_fill = (unsigned)std::min<uint64_t>(max_tiles, IND_MAX_GRID);
    const unsigned grid = (expected_tiles >= 2048 && expected_tiles < IND_MAX_GRID) ? 2048u : grid_fill;
    if (use_coarse)
        SGNN_LAUNCH(ctx, st, "induced_coarse_kernel", SGNN_TAG, induced_coarse_kernel, dim3((unsigned)std::min<uint64_t>(cdiv(W, 256), 4096)),
                    dim3(256), 0, st, bitmap, W, coarse);
    SGNN_LAUNCH(ctx, st, "induced_count_kernel", SGNN_TAG, induced_count_kernel, dim3(grid), dim3(IND_NT), 0, st, rowstart,
                g->colidx, B, bitmap, coarse, rg, P, tile_row, tile_total, keepbits, n_tiles, total64);
    int rc = sgnn_scan_u32_devn(ctx, tile_total, tile_off, n_tiles, max_tiles, scan_tmp, st);
    if (rc) return rc;
    double p = 1.0;
    if (rescale && B > 1) p = ((double)B - 1.0) / ((double)g->N - 1.0);
    SGNN_LAUNCH(ctx, st, "induced_fill_kernel", SGNN_TAG, induced_fill_kernel<RP>, dim3(grid_fill), dim3(IND_NT), 0, st, rowptr,
                g->colidx, norm_mode == 0 ? g->val : nullptr, S, rowstart, deg, B, bitmap, rank, P, tile_row, tile_off,
                n_tiles, keepbits, (float)(1.0 / p), norm_mode == 0 ? 1 : 0, out->rowptr, out->colidx, out->val,
                out->capacity, out->nnz_dev, ctx->status, total64, sticky_capacity,
                (rg.r0 <= 0 && rg.r1 >= (int64_t)g->N) ? 1 : 0);
    if (norm_mode == 1)
        SGNN_LAUNCH(ctx, st, "induced_renorm_kernel", SGNN_TAG, induced_renorm_kernel, dim3(cdiv((uint64_t)B * 64, 256)),
                    dim3(256), 0, st, out->rowptr, out->colidx, out->val, B, out->capacity, p);
    return SGNN_OK;
}

// Full graph as a matrix for the evaluation forward (Sec. VI: full-graph inference): int32 row offsets and
// the weights of Eq. 3, a_vu = 1 / sqrt(deg(v) deg(u)), evaluated in double precision and rounded once
// (the same arithmetic as the mini-batch weights).  One wavefront per row, grid-stride; a set-up kernel.
template <typename RP>
__global__ __launch_bounds__(256) void graph_normalize_kernel(uint64_t N, const RP *__restrict__ rowptr,
                                                              const int32_t *__restrict__ colidx,
                                                              const float *__restrict__ val_in, int32_t *__restrict__ rowptr32,
                                                              float *__restrict__ val)
{
    const int lane = threadIdx.x & 63;
    const uint64_t wave = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (uint64_t)gridDim.x * 4;
    for (uint64_t v = wave; v < N; v += nwaves) {
        const int64_t rs = (int64_t)rowptr[v], re = (int64_t)rowptr[v + 1];
        if (lane == 0 && rowptr32) {
            rowptr32[v] = (int32_t)rs;
            if (v + 1 == N) rowptr32[N] = (int32_t)re;
        }
        const double dv = (double)(re - rs);
        for (int64_t e = rs + lane; e < re; e += 64) {
            if (val_in) val[e] = val_in[e];
            else {
                const int64_t u = colidx[e];
                const double du = (double)((int64_t)rowptr[u + 1] - (int64_t)rowptr[u]);
                val[e] = (float)(1.0 / sqrt(dv * du));
            }
        }
    }
}

} // namespace

size_t sgnn_induced_ws_bytes(uint64_t N, uint64_t E, uint32_t B)
{
    const uint64_t max_tiles = E / IND_TILE + 2;
    return (size_t)(N + 63) / 64 + 256 + (size_t)B * 12 + ((size_t)B + 1) * 8 + (size_t)cdiv(B, DEG_TILE) * 8 + max_tiles * 4 + (max_tiles + 1) * 4 +
           max_tiles * IND_WORDS * 8 + (max_tiles + 1) * 4 + sgnn_scan_tmp_elems(max_tiles) * 4 + 16 + 13 * 256;
}

int sgnn_launch_induced(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                        const uint32_t *rank, int norm_mode, int rescale, int64_t R0, int64_t R1, int64_t C0, int64_t C1,
                        sgnn_csr *out, int sticky_capacity, hipStream_t st)
{
    const shard_range rg = {R0, R1, C0, C1};
    if (g->rowptr_is_i64) return launch_typed<int64_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, rg, out, sticky_capacity, st);
    return launch_typed<int32_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, rg, out, sticky_capacity, st);
}

int sgnn_launch_graph_normalize(sgnn_ctx *ctx, const sgnn_graph *g, int32_t *rowptr32, float *val, hipStream_t st)
{
    if (g->N == 0) return SGNN_OK;
    const unsigned nwg = (unsigned)std::min<uint64_t>((g->N + 3) / 4, 1u << 16);
    if (g->rowptr_is_i64)
        SGNN_LAUNCH(ctx, st, "graph_normalize_kernel", SGNN_TAG, graph_normalize_kernel<int64_t>, dim3(nwg), dim3(256), 0, st, g->N,
                    static_cast<const int64_t *>(g->rowptr), g->colidx, g->val, rowptr32, val);
    else
        SGNN_LAUNCH(ctx, st, "graph_normalize_kernel", SGNN_TAG, graph_normalize_kernel<int32_t>, dim3(nwg), dim3(256), 0, st, g->N,
                    static_cast<const int32_t *>(g->rowptr), g->colidx, g->val, rowptr32, val);
    return SGNN_OK;
}
