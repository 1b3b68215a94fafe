// Device-wide exclusive prefix sums of uint32 arrays (reduce / scan-of-partials / downsweep).
// Small inputs take a single-workgroup path so that latency-bound mini-batches pay one launch.
#include "block_prims.h"
#include "common.h"

namespace {

constexpr int SCAN_NT = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_NT * SCAN_ITEMS;   // 2048
constexpr uint64_t SCAN_SINGLE_MAX = 65536;

// One workgroup scans everything: 1024 threads, chunks of 1024*16 with a running carry; the loads of the
// next chunk are issued before the current one is scanned.
template <class OutT>
__global__ __launch_bounds__(1024) void scan_single_kernel(const uint32_t *__restrict__ in, OutT *__restrict__ out,
                                                           const uint64_t *n_dev, uint64_t n_host)
{
    constexpr int PER = 16;
    __shared__ OutT lds[1024 / 64 + 1];
    const uint64_t n = n_dev ? *n_dev : n_host;
    const bool vec = (reinterpret_cast<uintptr_t>(in) & 15) == 0;
    auto fetch = [&](uint64_t base, uint32_t (&v)[PER]) {
        const uint64_t i0 = base + (uint64_t)threadIdx.x * PER;
        if (vec && i0 + PER <= n) {
#pragma unroll
            for (int k = 0; k < PER / 4; ++k) {
                const uint4 q = *reinterpret_cast<const uint4 *>(in + i0 + 4 * k);
                v[4 * k] = q.x; v[4 * k + 1] = q.y; v[4 * k + 2] = q.z; v[4 * k + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < PER; ++k) v[k] = (i0 + k < n) ? in[i0 + k] : 0u;
        }
    };
    OutT carry = 0;
    uint32_t v[PER], nxt[PER] = {};
    fetch(0, v);
    for (uint64_t base = 0; base < n; base += 1024 * PER) {
        const uint64_t i0 = base + (uint64_t)threadIdx.x * PER;
        if (base + 1024 * PER < n) fetch(base + 1024 * PER, nxt);
        OutT s = 0;
#pragma unroll
        for (int k = 0; k < PER; ++k) s += v[k];
        OutT total;
        OutT ex = block_excl_scan<OutT, 1024>(s, &total, lds) + carry;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            if (i0 + k < n) out[i0 + k] = ex;
            ex += v[k];
        }
        carry += total;
#pragma unroll
        for (int k = 0; k < PER; ++k) v[k] = nxt[k];
    }
    if (threadIdx.x == 0) out[n] = carry;
}

template <class OutT>
__global__ __launch_bounds__(SCAN_NT) void scan_reduce_kernel(const uint32_t *__restrict__ in, OutT *__restrict__ partial,
                                                              const uint64_t *n_dev, uint64_t n_host)
{
    __shared__ OutT lds[SCAN_NT / 64];
    const uint64_t n = n_dev ? *n_dev : n_host;
    const uint64_t base = (uint64_t)blockIdx.x * SCAN_TILE;
    if (base >= n) return;
    OutT s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        uint64_t i = base + (uint64_t)k * SCAN_NT + threadIdx.x;
        if (i < n) s += in[i];
    }
    OutT t = block_sum<OutT, SCAN_NT>(s, lds);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

// Exclusive scan, in place, of the per-tile partial sums; the grand total goes to partial[nb].
template <class OutT>
__global__ __launch_bounds__(1024) void scan_partials_kernel(OutT *partial, const uint64_t *n_dev, uint64_t n_host)
{
    __shared__ OutT lds[1024 / 64 + 1];
    const uint64_t n = n_dev ? *n_dev : n_host;
    const uint64_t nb = (n + SCAN_TILE - 1) / SCAN_TILE;
    OutT carry = 0;
    for (uint64_t base = 0; base < nb; base += 1024) {
        uint64_t i = base + threadIdx.x;
        OutT v = i < nb ? partial[i] : OutT(0);
        OutT total;
        OutT ex = block_excl_scan<OutT, 1024>(v, &total, lds) + carry;
        if (i < nb) partial[i] = ex;
        carry += total;
    }
    if (threadIdx.x == 0) partial[nb] = carry;
}

template <class OutT>
__global__ __launch_bounds__(SCAN_NT) void scan_down_kernel(const uint32_t *__restrict__ in, OutT *__restrict__ out,
                                                            const OutT *__restrict__ partial, const uint64_t *n_dev,
                                                            uint64_t n_host)
{
    __shared__ OutT lds[SCAN_NT / 64 + 1];
    const uint64_t n = n_dev ? *n_dev : n_host;
    const uint64_t nb = (n + SCAN_TILE - 1) / SCAN_TILE;
    const uint64_t base = (uint64_t)blockIdx.x * SCAN_TILE;
    if (base >= n) {
        if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) out[0] = 0;
        return;
    }
    // blocked arrangement: thread t owns items base + t*8 .. +7
    const uint64_t i0 = base + (uint64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS];
    OutT s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = (i0 + k < n) ? in[i0 + k] : 0u;
        s += v[k];
    }
    OutT total;
    OutT ex = block_excl_scan<OutT, SCAN_NT>(s, &total, lds) + partial[blockIdx.x];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (i0 + k < n) out[i0 + k] = ex;
        ex += v[k];
    }
    if (blockIdx.x == nb - 1 && threadIdx.x == 0) out[n] = partial[nb];
}

template <class OutT>
int scan_impl(sgnn_ctx *ctx, const uint32_t *in, OutT *out, const uint64_t *n_dev, uint64_t n_max, OutT *tmp,
              hipStream_t st)
{
    if (n_max <= SCAN_SINGLE_MAX) {
        SGNN_LAUNCH(ctx, st, "scan_single_kernel", SGNN_TAG, scan_single_kernel<OutT>, dim3(1), dim3(1024), 0, st, in, out, n_dev, n_max);
        return SGNN_OK;
    }
    const unsigned nb = cdiv(n_max, SCAN_TILE);
    SGNN_LAUNCH(ctx, st, "scan_reduce_kernel", SGNN_TAG, scan_reduce_kernel<OutT>, dim3(nb), dim3(SCAN_NT), 0, st, in, tmp, n_dev, n_max);
    SGNN_LAUNCH(ctx, st, "scan_partials_kernel", SGNN_TAG, scan_partials_kernel<OutT>, dim3(1), dim3(1024), 0, st, tmp, n_dev, n_max);
    SGNN_LAUNCH(ctx, st, "scan_down_kernel", SGNN_TAG, scan_down_kernel<OutT>, dim3(nb), dim3(SCAN_NT), 0, st, in, out, tmp, n_dev, n_max);
    return SGNN_OK;
}

} // namespace

size_t sgnn_scan_tmp_elems(uint64_t n) { return (size_t)((n + SCAN_TILE - 1) / SCAN_TILE) + 1; }

int sgnn_scan_u32_to_u64(sgnn_ctx *ctx, const uint32_t *in, uint64_t *out, uint64_t n, uint64_t *tmp, hipStream_t st)
{
    return scan_impl<uint64_t>(ctx, in, out, nullptr, n, tmp, st);
}

int sgnn_scan_u32_devn(sgnn_ctx *ctx, const uint32_t *in, uint32_t *out, const uint64_t *n_dev, uint64_t n_max,
                       uint32_t *tmp, hipStream_t st)
{
    return scan_impl<uint32_t>(ctx, in, out, n_dev, n_max, tmp, st);
}
