// Transpose of a mini-batch CSR (Algorithm 2, last phase: the forward and the transposed matrix are
// both assembled; Sec. III-C uses the transposed one).  For the symmetric matrix of an undirected
// graph over the full ranges the matrix is its own transpose and none of this runs; a shard with
// different row and column ranges, or a directed graph, needs the real thing.
//
//   1. count    entries per column (integer atomics: the counts do not depend on timing)
//   2. scan     exclusive prefix sum -> row offsets of the transpose
//   3. scatter  every entry takes the next free slot of its column (atomic cursor; the order inside a
//               column depends on timing) into a scratch copy
//   4. order    every row of the transpose is put in ascending column order by ranking: an entry goes
//               to the position equal to the number of smaller keys in its row.  Keys are unique
//               (a CSR row holds a column once), so the result is the same whatever step 3 did.
// Ranking by comparison costs n^2 for a row of n entries, which is what the short rows of a
// mini-batch get; the hub columns of a power-law graph are ranked through a bitmap instead.
#include <algorithm>

#include "block_prims.h"
#include "common.h"

namespace {

__global__ __launch_bounds__(256) void transpose_clear_kernel(uint32_t *__restrict__ cnt, uint32_t *__restrict__ cursor,
                                                              uint32_t cols)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j < cols) { cnt[j] = 0; cursor[j] = 0; }
}

__global__ __launch_bounds__(256) void transpose_count_kernel(const int32_t *__restrict__ rowptr, uint32_t rows,
                                                              const int32_t *__restrict__ colidx, uint64_t capacity,
                                                              uint32_t cols, uint32_t *__restrict__ cnt)
{
    const int64_t nnz = min((int64_t)rowptr[rows], (int64_t)capacity);
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
        const uint32_t j = (uint32_t)colidx[e];
        if (j < cols) atomicAdd(&cnt[j], 1u);
    }
}

// a wavefront per source row
__global__ __launch_bounds__(256) void transpose_scatter_kernel(const int32_t *__restrict__ rowptr, uint32_t rows,
                                                                const int32_t *__restrict__ colidx,
                                                                const float *__restrict__ val, uint64_t capacity,
                                                                uint32_t cols, const uint32_t *__restrict__ rowptr_T,
                                                                uint32_t *__restrict__ cursor, int32_t *__restrict__ tmp_row,
                                                                float *__restrict__ tmp_val)
{
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
    for (uint32_t i = wave; i < rows; i += nwaves) {
        const int64_t rs = min((int64_t)rowptr[i], (int64_t)capacity), re = min((int64_t)rowptr[i + 1], (int64_t)capacity);
        for (int64_t e = rs + lane; e < re; e += 64) {
            const uint32_t j = (uint32_t)colidx[e];
            if (j >= cols) continue;
            const uint32_t pos = rowptr_T[j] + atomicAdd(&cursor[j], 1u);
            tmp_row[pos] = (int32_t)i;
            tmp_val[pos] = val[e];
        }
    }
}

// Ordering pass: a workgroup takes 256 rows of the transpose.
//   up to 16 entries      the row's own thread ranks them (n^2 comparisons, n tiny)
//   up to 512 entries     the wavefront takes such rows of its 64 one after the other, a lane per entry
//   longer (hub columns)  the workgroup takes them one after the other and ranks through a bitmap over
//                         the source rows: the keys of a window of ORDER_WINDOW source rows set their bits,
//                         a prefix sum over the popcounts of the bitmap words gives every key its rank
//                         (entries in earlier windows + bits below it): O(n + rows / 32) work per row
constexpr uint32_t ORDER_TINY = 16, ORDER_WAVE = 512;
constexpr uint32_t ORDER_WINDOW = 131072;                 // source rows per bitmap window: 16 KB of bits

__global__ __launch_bounds__(256) void transpose_order_kernel(const uint32_t *__restrict__ rowptr_T, uint32_t cols, uint32_t rows,
                                                              const int32_t *__restrict__ tmp_row,
                                                              const float *__restrict__ tmp_val, int32_t *__restrict__ colidx_T,
                                                              float *__restrict__ val_T)
{
    __shared__ uint32_t bits[ORDER_WINDOW / 32];
    __shared__ uint32_t pre[ORDER_WINDOW / 32];
    __shared__ __attribute__((aligned(16))) int32_t wkeys[256 / 64][ORDER_WAVE];     // keys of the row a wavefront is ranking
    __shared__ uint32_t red[256 / 64 + 1];
    __shared__ uint32_t hub[256];
    __shared__ uint32_t n_hub;
    // rows are dealt out to the workgroups in turn: the hub columns of a power-law graph have neighbouring
    // numbers and would otherwise all land in one workgroup
    const uint32_t j = threadIdx.x * gridDim.x + blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint32_t s = 0, n = 0;
    if (j < cols) { s = rowptr_T[j]; n = rowptr_T[j + 1] - s; }
    if (threadIdx.x == 0) n_hub = 0;
    __syncthreads();
    if (n <= ORDER_TINY) {
        // all keys of the row in registers (the loads go out together), ranked by comparison
        int32_t key[ORDER_TINY];
        float vv[ORDER_TINY];
#pragma unroll
        for (uint32_t k = 0; k < ORDER_TINY; ++k) {
            key[k] = 0x7fffffff; vv[k] = 0.f;
            if (k < n) { key[k] = tmp_row[s + k]; vv[k] = tmp_val[s + k]; }
        }
#pragma unroll
        for (uint32_t k = 0; k < ORDER_TINY; ++k) {
            if (k < n) {
                uint32_t rank = 0;
#pragma unroll
                for (uint32_t q = 0; q < ORDER_TINY; ++q) rank += key[q] < key[k] ? 1u : 0u;    // unused slots hold the largest int
                colidx_T[s + rank] = key[k];
                val_T[s + rank] = vv[k];
            }
        }
    } else if (n > ORDER_WAVE) hub[atomicAdd(&n_hub, 1u)] = threadIdx.x;     // any order: every hub row is done in full
    uint64_t mid = __ballot(n > ORDER_TINY && n <= ORDER_WAVE);
    while (mid) {
        const int src = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mid));
        mid &= mid - 1;
        const uint32_t ss = (uint32_t)__builtin_amdgcn_readlane((int)s, src), nn = (uint32_t)__builtin_amdgcn_readlane((int)n, src);
        // the keys of the row go to the wavefront's LDS slot, padded to a multiple of four with the largest int
        const uint32_t n4 = (nn + 3) & ~3u;
        for (uint32_t k = lane; k < n4; k += 64) wkeys[wv][k] = k < nn ? tmp_row[ss + k] : 0x7fffffff;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (uint32_t k = lane; k < nn; k += 64) {
            const int32_t key = wkeys[wv][k];
            uint32_t rank = 0;
            for (uint32_t q = 0; q < n4; q += 4) {
                const int4 kk = *reinterpret_cast<const int4 *>(&wkeys[wv][q]);
                rank += (kk.x < key ? 1u : 0u) + (kk.y < key ? 1u : 0u) + (kk.z < key ? 1u : 0u) + (kk.w < key ? 1u : 0u);
            }
            colidx_T[ss + rank] = key;
            val_T[ss + rank] = tmp_val[ss + k];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    __syncthreads();
    const uint32_t nh = n_hub;
    for (uint32_t h = 0; h < nh; ++h) {
        const uint32_t jj = hub[h] * gridDim.x + blockIdx.x;
        const uint32_t ss = rowptr_T[jj], nn = rowptr_T[jj + 1] - ss;
        uint32_t before = 0;                                  // entries of the row in earlier windows
        for (uint32_t w0 = 0; w0 < rows; w0 += ORDER_WINDOW) {
            const uint32_t wn = min(ORDER_WINDOW, rows - w0), words = (wn + 31) / 32;
            for (uint32_t i = threadIdx.x; i < words; i += 256) bits[i] = 0;
            __syncthreads();
            for (uint32_t k = threadIdx.x; k < nn; k += 256) {
                const uint32_t key = (uint32_t)tmp_row[ss + k] - w0;
                if (key < wn) atomicOr(&bits[key >> 5], 1u << (key & 31));
            }
            __syncthreads();
            // exclusive prefix of the popcounts: thread t owns the words [t * per, (t + 1) * per)
            const uint32_t per = (words + 255) / 256;
            const uint32_t i0 = min(threadIdx.x * per, words), i1 = min(i0 + per, words);
            uint32_t mine = 0;
            for (uint32_t i = i0; i < i1; ++i) mine += __popc(bits[i]);
            uint32_t total;
            uint32_t ex = block_excl_scan<uint32_t, 256>(mine, &total, red);
            for (uint32_t i = i0; i < i1; ++i) { pre[i] = ex; ex += __popc(bits[i]); }
            __syncthreads();
            for (uint32_t k = threadIdx.x; k < nn; k += 256) {
                const int32_t key32 = tmp_row[ss + k];
                const uint32_t key = (uint32_t)key32 - w0;
                if (key < wn) {
                    const uint32_t rank = before + pre[key >> 5] + __popc(bits[key >> 5] & ((1u << (key & 31)) - 1u));
                    colidx_T[ss + rank] = key32;
                    val_T[ss + rank] = tmp_val[ss + k];
                }
            }
            before += total;
            __syncthreads();
        }
    }
}

__global__ void transpose_finish_kernel(const uint32_t *__restrict__ rowptr_T, uint32_t cols, uint32_t *__restrict__ nnz_dev)
{
    if (nnz_dev) *nnz_dev = rowptr_T[cols];
}

} // namespace

size_t sgnn_transpose_ws_bytes(uint64_t max_entries, uint32_t B)
{
    return (size_t)max_entries * 8 + (size_t)B * 8 + sgnn_scan_tmp_elems(B) * 4 + 8 * 256;
}

int sgnn_launch_csr_transpose(sgnn_ctx *ctx, const sgnn_csr *A, sgnn_csr *out, ws_alloc *ws, hipStream_t st)
{
    const uint32_t rows = A->rows, cols = A->cols;
    uint32_t *cnt = ws->get<uint32_t>(cols + 1);
    uint32_t *cursor = ws->get<uint32_t>(cols + 1);
    uint32_t *scan_tmp = ws->get<uint32_t>(sgnn_scan_tmp_elems(cols));
    int32_t *tmp_row = ws->get<int32_t>(std::max<uint64_t>(A->capacity, 1));
    float *tmp_val = ws->get<float>(std::max<uint64_t>(A->capacity, 1));
    if (!ws->ok)
        return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_csr_transpose: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                         ws->off);
    uint32_t *rowptr_T = reinterpret_cast<uint32_t *>(out->rowptr);
    if (cols == 0) return SGNN_OK;
    SGNN_LAUNCH(ctx, st, "transpose_clear_kernel", SGNN_TAG, transpose_clear_kernel, dim3(cdiv(cols, 256)), dim3(256), 0, st, cnt,
                cursor, cols);
    const unsigned flat = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>(cdiv(A->capacity, 256), 4096));
    SGNN_LAUNCH(ctx, st, "transpose_count_kernel", SGNN_TAG, transpose_count_kernel, dim3(flat), dim3(256), 0, st, A->rowptr, rows,
                A->colidx, A->capacity, cols, cnt);
    int rc = sgnn_scan_u32_devn(ctx, cnt, rowptr_T, nullptr, cols, scan_tmp, st);
    if (rc) return rc;
    const unsigned rowgrid = (unsigned)std::max<uint32_t>(1, std::min<uint32_t>(cdiv(rows, 4), 8192));
    SGNN_LAUNCH(ctx, st, "transpose_scatter_kernel", SGNN_TAG, transpose_scatter_kernel, dim3(rowgrid), dim3(256), 0, st, A->rowptr,
                rows, A->colidx, A->val, A->capacity, cols, rowptr_T, cursor, tmp_row, tmp_val);
    SGNN_LAUNCH(ctx, st, "transpose_order_kernel", SGNN_TAG, transpose_order_kernel, dim3(cdiv(cols, 256)), dim3(256), 0, st, rowptr_T,
                cols, rows, tmp_row, tmp_val, out->colidx, out->val);
    SGNN_LAUNCH(ctx, st, "transpose_finish_kernel", SGNN_TAG, transpose_finish_kernel, dim3(1), dim3(1), 0, st, rowptr_T, cols,
                out->nnz_dev);
    return SGNN_OK;
}
