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
//   4. induced_group_kernel    only beyond 2048 tiles: survivors per group of 2048 tiles
//   5. induced_fill_kernel     ordered compaction inside the tile; writes colidx, val, rowptr
//   6. induced_renorm_kernel   only for norm_mode 1: weights from the degrees of the induced graph
// A tile stages the starts of the rows it touches in LDS, so finding the row of an edge is a
// binary search in LDS, and the whole tile needs one barrier for its ordered compaction.
#include <algorithm>

#include "block_prims.h"
#include "common.h"

namespace {

constexpr int IND_NT = 256;
constexpr int IND_ITEMS = 8;
constexpr int IND_TILE = IND_NT * IND_ITEMS;      // 2048 flat edges per workgroup
constexpr int IND_GROUP = 2048;                   // tiles per group of the two-level tile offsets
constexpr unsigned IND_MAX_GRID = 8192;
constexpr int DEG_TILE = 2048;                    // sampled rows per workgroup in the offset kernels

// Row and column range of a shard (Algorithm 2: [R0, R1) x [C0, C1) in global vertex ids); the whole graph by default.
struct shard_range { int64_t r0, r1, c0, c1; };

template <class RP>
__global__ __launch_bounds__(256) void induced_deg_kernel(const RP *__restrict__ rowptr, const int32_t *__restrict__ S,
                                                          uint32_t B, shard_range rg, uint32_t *__restrict__ deg,
                                                          uint64_t *__restrict__ wg_sum)
{
    __shared__ uint64_t lds[256 / 64];
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < DEG_TILE / 256; ++k) {
        const uint32_t i = blockIdx.x * DEG_TILE + k * 256 + threadIdx.x;
        if (i < B) {
            const int64_t v = S[i];
            // a sampled row outside the shard's row range contributes no edge: it comes out as an empty row
            const uint32_t dgr = (v >= rg.r0 && v < rg.r1) ? (uint32_t)(rowptr[v + 1] - rowptr[v]) : 0u;
            deg[i] = dgr;
            s += dgr;
        }
    }
    const uint64_t t = block_sum<uint64_t, 256>(s, lds);
    if (threadIdx.x == 0) wg_sum[blockIdx.x] = t;
}

__global__ __launch_bounds__(256) void induced_offsets_kernel(const uint32_t *__restrict__ deg, uint32_t B,
                                                              const uint64_t *__restrict__ wg_sum,
                                                              uint64_t *__restrict__ P)
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
        if (i0 + k < B) P[i0 + k] = ex;
        ex += d[k];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) P[B] = base + total;
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
// staged == false (more rows than the table holds: only possible when the input has rows without
// any entry) falls back to searching P in global memory.
struct tile_table {
    int32_t relP[IND_TILE];
    int64_t ebase[IND_TILE];
    uint32_t r_lo, nr;
};

template <class RP>
__device__ __forceinline__ bool stage_tile(tile_table &tt, const RP *__restrict__ rowptr, const int32_t *__restrict__ S,
                                           uint32_t B, const uint64_t *__restrict__ P, uint64_t f0, uint64_t f1)
{
    if (threadIdx.x == 0) {
        tt.r_lo = find_row(P, 0, B - 1, f0);
        tt.nr = find_row(P, tt.r_lo, B - 1, f1 - 1) - tt.r_lo + 1;
    }
    __syncthreads();
    const uint32_t r_lo = tt.r_lo, nr = tt.nr;
    const bool staged = nr <= (uint32_t)IND_TILE;
    if (staged) {
        for (uint32_t k = threadIdx.x; k < nr; k += IND_NT) {
            const uint64_t p = P[r_lo + k];
            const int64_t v = S[r_lo + k];
            tt.relP[k] = p < f0 ? -1 : (int32_t)(p - f0);
            tt.ebase[k] = (int64_t)rowptr[v] - (int64_t)p;
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

template <class RP>
__global__ __launch_bounds__(IND_NT) void induced_count_kernel(const RP *__restrict__ rowptr,
                                                               const int32_t *__restrict__ colidx,
                                                               const int32_t *__restrict__ S, uint32_t B,
                                                               const uint64_t *__restrict__ bitmap, shard_range rg,
                                                               const uint64_t *__restrict__ P,
                                                               uint32_t *__restrict__ tile_total,
                                                               uint64_t *__restrict__ n_tiles_out)
{
    __shared__ tile_table tt;
    __shared__ uint32_t lds[IND_NT / 64];
    const uint64_t F = P[B];
    const uint64_t n_tiles = (F + IND_TILE - 1) / IND_TILE;
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_tiles_out = n_tiles;
    for (uint64_t c = blockIdx.x; c < n_tiles; c += gridDim.x) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const bool staged = stage_tile(tt, rowptr, S, B, P, f0, f1);
        const uint32_t nr = tt.nr, r_lo = tt.r_lo;
        int32_t u[IND_ITEMS];
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t f = f0 + (uint64_t)k * IND_NT + threadIdx.x;
            u[k] = -1;
            if (f < f1) {
                int64_t e;
                if (staged) e = tt.ebase[find_row_lds(tt, nr, (int32_t)(f - f0))] + (int64_t)f;
                else {
                    const uint32_t r = find_row(P, r_lo, r_lo + nr - 1, f);
                    e = (int64_t)rowptr[S[r]] + (int64_t)(f - P[r]);
                }
                u[k] = colidx[e];
                if (u[k] < rg.c0 || u[k] >= rg.c1) u[k] = -1;   // a column outside the shard
            }
        }
        uint32_t cnt = 0;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k)
            if (u[k] >= 0) cnt += (uint32_t)((bitmap[(uint32_t)u[k] >> 6] >> (u[k] & 63)) & 1ull);
        const uint32_t t = block_sum<uint32_t, IND_NT>(cnt, lds);   // ends with a barrier: tt may be reused
        if (threadIdx.x == 0) tile_total[c] = t;
    }
}

// survivors per group of IND_GROUP consecutive tiles
__global__ __launch_bounds__(256) void induced_group_kernel(const uint32_t *__restrict__ tile_total,
                                                            const uint64_t *__restrict__ n_tiles_p,
                                                            uint32_t *__restrict__ group_total)
{
    __shared__ uint32_t lds[256 / 64];
    const uint64_t n_tiles = *n_tiles_p;
    const uint64_t c0 = (uint64_t)blockIdx.x * IND_GROUP;
    uint32_t s = 0;
    for (uint64_t c = c0 + threadIdx.x; c < min(n_tiles, c0 + IND_GROUP); c += 256) s += tile_total[c];
    const uint32_t t = block_sum<uint32_t, 256>(s, lds);
    if (threadIdx.x == 0) group_total[blockIdx.x] = t;
}

// survivors in tiles [0, c): whole groups from group_total, the rest from tile_total
__device__ __forceinline__ uint32_t survivors_before(const uint32_t *__restrict__ tile_total,
                                                     const uint32_t *__restrict__ group_total, uint64_t c, uint32_t *lds)
{
    const uint64_t gq = group_total ? c / IND_GROUP : 0;
    uint32_t s = 0;
    for (uint64_t i = threadIdx.x; i < gq; i += IND_NT) s += group_total[i];
    for (uint64_t i = gq * IND_GROUP + threadIdx.x; i < c; i += IND_NT) s += tile_total[i];
    return block_sum<uint32_t, IND_NT>(s, lds);
}

template <class RP>
__global__ __launch_bounds__(IND_NT) void induced_fill_kernel(
    const RP *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *__restrict__ gval,
    const int32_t *__restrict__ S, uint32_t B, const uint64_t *__restrict__ bitmap, const uint32_t *__restrict__ rank,
    shard_range rg, const uint64_t *__restrict__ P, const uint32_t *__restrict__ tile_total, const uint32_t *__restrict__ group_total,
    const uint64_t *__restrict__ n_tiles_p, double p, int write_val, int32_t *__restrict__ rowptr_S,
    int32_t *__restrict__ colidx_S, float *__restrict__ val_S, uint64_t capacity, uint32_t *__restrict__ nnz_dev,
    uint32_t *__restrict__ status, int empty_rows_here)
{
    // empty_rows_here: rows without any stored entry get their offset from the thread that holds the first
    // entry of the next row, one after the other (fine for the odd isolated vertex); 0: a kernel of its own
    // does it afterwards (a shard leaves every sampled row outside its row range empty)
    __shared__ tile_table tt;
    __shared__ uint32_t lds[IND_NT / 64];
    __shared__ uint32_t wcnt[IND_ITEMS][IND_NT / 64];
    const uint64_t F = P[B];
    const uint64_t n_tiles = *n_tiles_p;
    const unsigned lane = lane_id(), wave = threadIdx.x >> 6;
    if (blockIdx.x == 0) {
        const uint32_t total = survivors_before(tile_total, group_total, n_tiles, lds);
        if (threadIdx.x == 0) {
            if (total > 0x7fffffffu) atomicOr(status, SGNN_ST_NNZ_OVERFLOW);
            rowptr_S[B] = (int32_t)total;
            // rows at the end that have no stored entry at all
            if (empty_rows_here)
                for (int64_t r = (int64_t)B - 1; r >= 0 && P[r] == F; --r) rowptr_S[r] = (int32_t)total;
            if (nnz_dev) *nnz_dev = total;
        }
    }
    for (uint64_t c = blockIdx.x; c < n_tiles; c += gridDim.x) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const uint32_t tile_off = survivors_before(tile_total, group_total, c, lds);
        const bool staged = stage_tile(tt, rowptr, S, B, P, f0, f1);
        const uint32_t nr = tt.nr, r_lo = tt.r_lo;

        int32_t u[IND_ITEMS];
        uint32_t rk[IND_ITEMS];      // row of the edge, relative to r_lo
        int64_t eidx[IND_ITEMS];
        bool first[IND_ITEMS];       // the edge is the first stored entry of its row
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t f = f0 + (uint64_t)k * IND_NT + threadIdx.x;
            u[k] = -1; rk[k] = 0; eidx[k] = 0; first[k] = false;
            if (f < f1) {
                if (staged) {
                    const int32_t x = (int32_t)(f - f0);
                    rk[k] = find_row_lds(tt, nr, x);
                    eidx[k] = tt.ebase[rk[k]] + (int64_t)f;
                    first[k] = tt.relP[rk[k]] == x;
                } else {
                    const uint32_t r = find_row(P, r_lo, r_lo + nr - 1, f);
                    rk[k] = r - r_lo;
                    eidx[k] = (int64_t)rowptr[S[r]] + (int64_t)(f - P[r]);
                    first[k] = P[r] == f;
                }
                u[k] = colidx[eidx[k]];
            }
        }
        uint64_t word[IND_ITEMS], bal[IND_ITEMS];
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) word[k] = u[k] >= 0 ? bitmap[(uint32_t)u[k] >> 6] : 0ull;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const bool keep = u[k] >= 0 && u[k] >= rg.c0 && u[k] < rg.c1 && ((word[k] >> (u[k] & 63)) & 1ull);
            bal[k] = __ballot(keep);
            if (lane == 0) wcnt[k][wave] = __popcll(bal[k]);
        }
        __syncthreads();
        uint32_t base = tile_off;
        const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            uint32_t before = 0, slab = 0;
#pragma unroll
            for (int w = 0; w < IND_NT / 64; ++w) {
                const uint32_t cw = wcnt[k][w];
                if (w < (int)wave) before += cw;
                slab += cw;
            }
            const uint32_t pos = base + before + __popcll(bal[k] & below);   // survivors ahead of this edge
            base += slab;
            if (u[k] < 0) continue;
            const uint32_t r = r_lo + rk[k];
            if (first[k]) {
                // everything before the first entry of row r belongs to earlier rows
                rowptr_S[r] = (int32_t)pos;
                if (empty_rows_here) {
                    const uint64_t Pr = P[r];
                    for (int64_t q = (int64_t)r - 1; q >= 0 && P[q] == Pr; --q) rowptr_S[q] = (int32_t)pos;
                }
            }
            if (((bal[k] >> lane) & 1ull) && pos < capacity) {
                colidx_S[pos] = (int32_t)(rank[(uint32_t)u[k] >> 6] + __popcll(word[k] & ((1ull << (u[k] & 63)) - 1ull)));
                if (write_val) {
                    const int64_t v = S[r];
                    double a;
                    if (gval) a = (double)gval[eidx[k]];
                    else {
                        const double dv = (double)(rowptr[v + 1] - rowptr[v]);
                        const double du = (double)(rowptr[(int64_t)u[k] + 1] - rowptr[u[k]]);
                        a = 1.0 / sqrt(dv * du);
                    }
                    if ((int64_t)u[k] != v) a /= p;
                    val_S[pos] = (float)a;
                }
            }
        }
        __syncthreads();   // wcnt and the row table are reused by the next tile
    }
}

// Offsets of the rows without any stored entry, one thread per row: such a row starts where the next
// row that has stored entries starts (found by binary search in the flat offsets), or at the end.
__global__ __launch_bounds__(256) void induced_empty_rows_kernel(const uint64_t *__restrict__ P, uint32_t B,
                                                                 int32_t *rowptr_S)
{
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B) return;
    const uint64_t Pi = P[i];
    if (P[i + 1] != Pi) return;
    // the last row whose flat offset is still Pi is the one that holds the entries (none does when Pi is the
    // end of the flat range); its offset was written by the fill kernel and no thread of this kernel touches it
    rowptr_S[i] = Pi == P[B] ? rowptr_S[B] : rowptr_S[find_row(P, i, B - 1, Pi)];
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
                 const uint32_t *rank, int norm_mode, int rescale, shard_range rg, sgnn_csr *out, hipStream_t st)
{
    const RP *rowptr = static_cast<const RP *>(g->rowptr);
    ws_alloc ws(ctx);
    const uint64_t max_tiles = g->E / IND_TILE + 2;
    const unsigned n_groups = cdiv(max_tiles, IND_GROUP);
    const unsigned n_deg_wg = cdiv(B, DEG_TILE);
    uint32_t *deg = ws.get<uint32_t>(B);
    uint64_t *deg_sum = ws.get<uint64_t>(n_deg_wg);
    uint64_t *P = ws.get<uint64_t>((size_t)B + 1);
    uint32_t *tile_total = ws.get<uint32_t>(max_tiles);
    uint32_t *group_total = ws.get<uint32_t>(n_groups);
    uint64_t *n_tiles = ws.get<uint64_t>(1);
    if (!ws.ok)
        return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_induced_csr: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                         ws.off);

    SGNN_LAUNCH(ctx, st, "induced_deg_kernel", SGNN_TAG, induced_deg_kernel<RP>, dim3(n_deg_wg), dim3(256), 0, st, rowptr, S, B,
                rg, deg, deg_sum);
    SGNN_LAUNCH(ctx, st, "induced_offsets_kernel", SGNN_TAG, induced_offsets_kernel, dim3(n_deg_wg), dim3(256), 0, st, deg, B,
                deg_sum, P);
    const unsigned grid = (unsigned)std::min<uint64_t>(max_tiles, IND_MAX_GRID);
    SGNN_LAUNCH(ctx, st, "induced_count_kernel", SGNN_TAG, induced_count_kernel<RP>, dim3(grid), dim3(IND_NT), 0, st, rowptr,
                g->colidx, S, B, bitmap, rg, P, tile_total, n_tiles);
    const bool grouped = max_tiles > IND_GROUP;
    if (grouped)
        SGNN_LAUNCH(ctx, st, "induced_group_kernel", SGNN_TAG, induced_group_kernel, dim3(n_groups), dim3(256), 0, st,
                    tile_total, n_tiles, group_total);
    double p = 1.0;
    if (rescale && B > 1) p = ((double)B - 1.0) / ((double)g->N - 1.0);
    const bool whole_rows = rg.r0 <= 0 && rg.r1 >= (int64_t)g->N;
    SGNN_LAUNCH(ctx, st, "induced_fill_kernel", SGNN_TAG, induced_fill_kernel<RP>, dim3(grid), dim3(IND_NT), 0, st, rowptr,
                g->colidx, norm_mode == 0 ? g->val : nullptr, S, B, bitmap, rank, rg, P, tile_total,
                grouped ? group_total : nullptr, n_tiles, p, norm_mode == 0 ? 1 : 0, out->rowptr, out->colidx, out->val,
                out->capacity, out->nnz_dev, ctx->status, whole_rows ? 1 : 0);
    if (!whole_rows)
        SGNN_LAUNCH(ctx, st, "induced_empty_rows_kernel", SGNN_TAG, induced_empty_rows_kernel, dim3(cdiv(B, 256)), dim3(256), 0,
                    st, P, B, out->rowptr);
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
        if (lane == 0) {
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

size_t sgnn_induced_ws_bytes(uint64_t E, uint32_t B)
{
    const uint64_t max_tiles = E / IND_TILE + 2;
    return (size_t)B * 4 + ((size_t)B + 1) * 8 + (size_t)cdiv(B, DEG_TILE) * 8 + max_tiles * 4 +
           (size_t)cdiv(max_tiles, IND_GROUP) * 4 + 8 + 8 * 256;
}

int sgnn_launch_induced(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                        const uint32_t *rank, int norm_mode, int rescale, int64_t R0, int64_t R1, int64_t C0, int64_t C1,
                        sgnn_csr *out, hipStream_t st)
{
    const shard_range rg = {R0, R1, C0, C1};
    if (g->rowptr_is_i64) return launch_typed<int64_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, rg, out, st);
    return launch_typed<int32_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, rg, out, st);
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
