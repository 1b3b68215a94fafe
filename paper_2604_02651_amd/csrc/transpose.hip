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
// Ranking costs O(n^2) comparisons for a row of n entries; rows of a mini-batch are short and the
// few long ones are spread over a whole workgroup each.
#include <algorithm>

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

// Rows of the transpose with up to `short_len` entries: a wavefront per row.  Longer rows: a workgroup per
// row in a second launch of the same kernel (whole = 1).
__global__ __launch_bounds__(256) void transpose_order_kernel(const uint32_t *__restrict__ rowptr_T, uint32_t cols,
                                                              const int32_t *__restrict__ tmp_row,
                                                              const float *__restrict__ tmp_val, uint32_t short_len,
                                                              int whole, int32_t *__restrict__ colidx_T,
                                                              float *__restrict__ val_T)
{
    const uint32_t nthr = whole ? 256u : 64u;
    const uint32_t t = whole ? threadIdx.x : (threadIdx.x & 63);
    const uint32_t unit = whole ? blockIdx.x : blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t nunits = whole ? gridDim.x : gridDim.x * 4;
    for (uint32_t j = unit; j < cols; j += nunits) {
        const uint32_t s = rowptr_T[j], n = rowptr_T[j + 1] - s;
        if (whole ? n <= short_len : n > short_len) continue;
        for (uint32_t k = t; k < n; k += nthr) {
            const int32_t key = tmp_row[s + k];
            uint32_t rank = 0;
            for (uint32_t q = 0; q < n; ++q) rank += tmp_row[s + q] < key ? 1u : 0u;
            colidx_T[s + rank] = key;
            val_T[s + rank] = tmp_val[s + k];
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
    const uint32_t short_len = 256;
    const unsigned colgrid = (unsigned)std::max<uint32_t>(1, std::min<uint32_t>(cdiv(cols, 4), 8192));
    SGNN_LAUNCH(ctx, st, "transpose_order_kernel", SGNN_TAG, transpose_order_kernel, dim3(colgrid), dim3(256), 0, st, rowptr_T, cols,
                tmp_row, tmp_val, short_len, 0, out->colidx, out->val);
    SGNN_LAUNCH(ctx, st, "transpose_order_kernel", SGNN_TAG, transpose_order_kernel, dim3(std::min<uint32_t>(cols, 4096)), dim3(256),
                0, st, rowptr_T, cols, tmp_row, tmp_val, short_len, 1, out->colidx, out->val);
    SGNN_LAUNCH(ctx, st, "transpose_finish_kernel", SGNN_TAG, transpose_finish_kernel, dim3(1), dim3(1), 0, st, rowptr_T, cols,
                out->nnz_dev);
    return SGNN_OK;
}
