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
//   1. induced_deg_kernel     row length of every sampled row; scan -> flat offsets P[B+1]
//   2. induced_count_kernel   survivors per tile (wave ballots / popcounts); scan -> tile offsets
//   3. induced_fill_kernel    ordered compaction inside the tile; writes colidx, val, rowptr
//   4. induced_renorm_kernel  only for norm_mode 1: weights from the degrees of the induced graph
#include "block_prims.h"
#include <algorithm>

#include "common.h"

namespace {

constexpr int IND_NT = 256;
constexpr int IND_ITEMS = 8;
constexpr int IND_TILE = IND_NT * IND_ITEMS;
constexpr unsigned IND_MAX_GRID = 8192;

template <class RP>
__global__ __launch_bounds__(256) void induced_deg_kernel(const RP *__restrict__ rowptr, const int32_t *__restrict__ S,
                                                          uint32_t B, uint32_t *__restrict__ deg)
{
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < B) {
        const int64_t v = S[i];
        deg[i] = (uint32_t)(rowptr[v + 1] - rowptr[v]);
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

struct tile_rows { uint32_t lo, hi; };

// Row range touched by the tile [f0, f1): computed by one thread, shared through LDS.
__device__ __forceinline__ tile_rows tile_row_range(const uint64_t *__restrict__ P, uint32_t B, uint64_t f0, uint64_t f1,
                                                    uint32_t *lds2)
{
    if (threadIdx.x == 0) {
        lds2[0] = find_row(P, 0, B - 1, f0);
        lds2[1] = find_row(P, lds2[0], B - 1, f1 - 1);
    }
    __syncthreads();
    tile_rows r = {lds2[0], lds2[1]};
    __syncthreads();
    return r;
}

template <class RP>
__global__ __launch_bounds__(IND_NT) void induced_count_kernel(const RP *__restrict__ rowptr,
                                                               const int32_t *__restrict__ colidx,
                                                               const int32_t *__restrict__ S, uint32_t B,
                                                               const uint64_t *__restrict__ bitmap,
                                                               const uint64_t *__restrict__ P,
                                                               uint32_t *__restrict__ tile_total,
                                                               uint64_t *__restrict__ n_tiles_out)
{
    __shared__ uint32_t lds[IND_NT / 64];
    __shared__ uint32_t lds2[2];
    const uint64_t F = P[B];
    const uint64_t n_tiles = (F + IND_TILE - 1) / IND_TILE;
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_tiles_out = n_tiles;
    for (uint64_t c = blockIdx.x; c < n_tiles; c += gridDim.x) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const tile_rows tr = tile_row_range(P, B, f0, f1, lds2);
        uint32_t cnt = 0;
#pragma unroll
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t f = f0 + (uint64_t)k * IND_NT + threadIdx.x;
            if (f < f1) {
                const uint32_t r = find_row(P, tr.lo, tr.hi, f);
                const int64_t v = S[r];
                const int32_t u = colidx[(int64_t)rowptr[v] + (int64_t)(f - P[r])];
                cnt += (uint32_t)((bitmap[(uint32_t)u >> 6] >> (u & 63)) & 1ull);
            }
        }
        const uint32_t t = block_sum<uint32_t, IND_NT>(cnt, lds);
        if (threadIdx.x == 0) tile_total[c] = t;
    }
}

template <class RP>
__global__ __launch_bounds__(IND_NT) void induced_fill_kernel(
    const RP *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *__restrict__ gval,
    const int32_t *__restrict__ S, uint32_t B, const uint64_t *__restrict__ bitmap, const uint32_t *__restrict__ rank,
    const uint64_t *__restrict__ P, const uint32_t *__restrict__ tile_off, const uint64_t *__restrict__ n_tiles_p,
    double p, int write_val, int32_t *__restrict__ rowptr_S, int32_t *__restrict__ colidx_S, float *__restrict__ val_S,
    uint64_t capacity, uint32_t *__restrict__ nnz_dev, uint32_t *__restrict__ status)
{
    __shared__ uint32_t lds[IND_NT / 64 + 1];
    __shared__ uint32_t lds2[2];
    const uint64_t F = P[B];
    const uint64_t n_tiles = *n_tiles_p;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const uint32_t total = tile_off[n_tiles];
        if (total > 0x7fffffffu) atomicOr(status, SGNN_ST_NNZ_OVERFLOW);
        rowptr_S[B] = (int32_t)total;
        // rows at the end that have no stored entry at all
        for (int64_t r = (int64_t)B - 1; r >= 0 && P[r] == F; --r) rowptr_S[r] = (int32_t)total;
        if (nnz_dev) *nnz_dev = total;
    }
    for (uint64_t c = blockIdx.x; c < n_tiles; c += gridDim.x) {
        const uint64_t f0 = c * IND_TILE, f1 = min(F, f0 + IND_TILE);
        const tile_rows tr = tile_row_range(P, B, f0, f1, lds2);
        uint32_t running = tile_off[c];
#pragma unroll 1
        for (int k = 0; k < IND_ITEMS; ++k) {
            const uint64_t f = f0 + (uint64_t)k * IND_NT + threadIdx.x;
            bool keep = false;
            uint32_t r = 0;
            int32_t u = 0;
            int64_t v = 0, e = 0;
            uint64_t Pr = 0, word = 0;
            if (f < f1) {
                r = find_row(P, tr.lo, tr.hi, f);
                Pr = P[r];
                v = S[r];
                e = (int64_t)rowptr[v] + (int64_t)(f - Pr);
                u = colidx[e];
                word = bitmap[(uint32_t)u >> 6];
                keep = (word >> (u & 63)) & 1ull;
            }
            uint32_t total;
            const uint32_t pos = block_excl_scan<uint32_t, IND_NT>(keep ? 1u : 0u, &total, lds) + running;
            if (f < f1) {
                if (f == Pr) {
                    // first stored entry of row r: everything before it belongs to earlier rows
                    rowptr_S[r] = (int32_t)pos;
                    for (int64_t q = (int64_t)r - 1; q >= 0 && P[q] == Pr; --q) rowptr_S[q] = (int32_t)pos;
                }
                if (keep && pos < capacity) {
                    colidx_S[pos] = (int32_t)(rank[(uint32_t)u >> 6] + __popcll(word & ((1ull << (u & 63)) - 1ull)));
                    if (write_val) {
                        double a;
                        if (gval) a = (double)gval[e];
                        else {
                            const double dv = (double)(P[r + 1] - Pr);
                            const double du = (double)(rowptr[(int64_t)u + 1] - rowptr[u]);
                            a = 1.0 / sqrt(dv * du);
                        }
                        if ((int64_t)u != v) a /= p;
                        val_S[pos] = (float)a;
                    }
                }
            }
            running += total;
        }
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
                 const uint32_t *rank, int norm_mode, int rescale, sgnn_csr *out, hipStream_t st)
{
    const RP *rowptr = static_cast<const RP *>(g->rowptr);
    ws_alloc ws(ctx);
    const uint64_t max_tiles = g->E / IND_TILE + 2;
    uint32_t *deg = ws.get<uint32_t>(B);
    uint64_t *P = ws.get<uint64_t>((size_t)B + 1);
    uint64_t *scan_tmp64 = ws.get<uint64_t>(sgnn_scan_tmp_elems(B));
    uint32_t *tile_total = ws.get<uint32_t>(max_tiles);
    uint32_t *tile_off = ws.get<uint32_t>(max_tiles + 1);
    uint32_t *scan_tmp32 = ws.get<uint32_t>(sgnn_scan_tmp_elems(max_tiles));
    uint64_t *n_tiles = ws.get<uint64_t>(1);
    if (!ws.ok)
        return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_induced_csr: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                         ws.off);

    SGNN_LAUNCH(ctx, st, "induced_deg_kernel", SGNN_TAG, induced_deg_kernel<RP>, dim3(cdiv(B, 256)), dim3(256), 0, st, rowptr, S, B, deg);
    int rc = sgnn_scan_u32_to_u64(ctx, deg, P, B, scan_tmp64, st);
    if (rc) return rc;
    const unsigned grid = (unsigned)std::min<uint64_t>(max_tiles, IND_MAX_GRID);
    SGNN_LAUNCH(ctx, st, "induced_count_kernel", SGNN_TAG, induced_count_kernel<RP>, dim3(grid), dim3(IND_NT), 0, st, rowptr, g->colidx, S, B, bitmap, P,
                       tile_total, n_tiles);
    rc = sgnn_scan_u32_devn(ctx, tile_total, tile_off, n_tiles, max_tiles, scan_tmp32, st);
    if (rc) return rc;
    double p = 1.0;
    if (rescale && B > 1) p = ((double)B - 1.0) / ((double)g->N - 1.0);
    SGNN_LAUNCH(ctx, st, "induced_fill_kernel", SGNN_TAG, induced_fill_kernel<RP>, dim3(grid), dim3(IND_NT), 0, st, rowptr, g->colidx,
                       norm_mode == 0 ? g->val : nullptr, S, B, bitmap, rank, P, tile_off, n_tiles, p,
                       norm_mode == 0 ? 1 : 0, out->rowptr, out->colidx, out->val, out->capacity, out->nnz_dev,
                       ctx->status);
    if (norm_mode == 1) {
        SGNN_LAUNCH(ctx, st, "induced_renorm_kernel", SGNN_TAG, induced_renorm_kernel, dim3(cdiv((uint64_t)B * 64, 256)), dim3(256), 0, st, out->rowptr,
                           out->colidx, out->val, B, out->capacity, p);
    }
    return SGNN_OK;
}

} // namespace

size_t sgnn_induced_ws_bytes(uint64_t E, uint32_t B)
{
    const uint64_t max_tiles = E / IND_TILE + 2;
    return (size_t)B * 4 + ((size_t)B + 1) * 8 + sgnn_scan_tmp_elems(B) * 8 + max_tiles * 8 + 4 +
           sgnn_scan_tmp_elems(max_tiles) * 4 + 8 + 8 * 256;
}

int sgnn_launch_induced(sgnn_ctx *ctx, const sgnn_graph *g, const int32_t *S, uint32_t B, const uint64_t *bitmap,
                        const uint32_t *rank, int norm_mode, int rescale, sgnn_csr *out, hipStream_t st)
{
    if (g->rowptr_is_i64) return launch_typed<int64_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, out, st);
    return launch_typed<int32_t>(ctx, g, S, B, bitmap, rank, norm_mode, rescale, out, st);
}
