// Uniform vertex sampling without replacement (Sec. III-D "Vertex Sampling", Eq. 20).
//
// The sample is the B vertices with the smallest (key(v), v), key(v) being 64 bits of
// Philox4x32-10 (Salmon et al., SC'11) counted by (v/2, step) and keyed by the seed.  Whole keys are
// never stored.  A pass that recomputes them is bound by the 20 quarter-rate 32 x 32 -> 64 multiplies
// of a Philox call (about 19 us per 2^23 calls, measured), three passes cost three times that; with
// scratch for two bytes per vertex the first pass also stores the top 16 bits of every key, and the
// later passes read those instead: they decide all but 2^-11 (candidates) and 2^-16 (ties with the
// threshold's prefix) of the vertices, and only for these is the key computed again.
//
// Sparse samples of large graphs take passes 1, 2, 4 and 6 only, pass 1 in the form of sampler_hist_window_kernel
// (which also appends the candidates and sets the bits of the vertices that are in for certain).
//
//   1. sampler_hist_kernel     histogram of the top 11 key bits (LDS histograms, one merge)
//   2. sampler_pick_bin_kernel the bin b* that holds the B-th smallest key and the rank r inside
//   3. sampler_collect_kernel  (key, v) of every vertex in bin b* -> candidate list (about N/2048)
//   4. sampler_threshold_kernel exact r-th smallest (key, v) of the candidates, by radix select
//   5. sampler_emit_kernel     bitmap word per 64 vertices from wave ballots + per-workgroup counts
//   6. sampler_rank_kernel     rank prefix per bitmap word and the ascending list S
#include "block_prims.h"
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>

#include "common.h"
#include "philox.h"

namespace {

constexpr int HIST_BITS = 11;
constexpr int HIST_BINS = 1 << HIST_BITS;
constexpr int SAMP_NT = 256;
constexpr int SCAN_NT = 1024;            // key passes: few large workgroups, so that few of them meet on one address
constexpr unsigned EMIT_MAX_WG = 1024;

struct sampler_state {
    uint32_t bin;       // histogram bin of the threshold key
    uint32_t r;         // 1-based rank of the threshold inside that bin
    uint32_t ncand;     // candidates appended by the collect pass
    uint32_t thr_v;     // threshold vertex
    uint64_t thr_key;   // threshold key
    uint32_t fallback;  // windowed call whose threshold bin fell outside the window: the recomputing passes run instead
    uint32_t nmark;     // candidates the threshold pass looked at (ncand is zero again when it ends)
};

// keys of vertices 2j (even) and 2j+1 (odd)
__device__ __forceinline__ void vertex_pair_keys(uint64_t j, uint64_t seed, uint64_t step, uint64_t &ke, uint64_t &ko)
{
    philox_out o = philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                                 (uint32_t)seed, (uint32_t)(seed >> 32));
    ke = ((uint64_t)o.w1 << 32) | o.w0;
    ko = ((uint64_t)o.w3 << 32) | o.w2;
}

__device__ __forceinline__ uint64_t spread_even(uint32_t x32)
{
    uint64_t x = x32;
    x = (x | (x << 16)) & 0x0000FFFF0000FFFFull;
    x = (x | (x << 8)) & 0x00FF00FF00FF00FFull;
    x = (x | (x << 4)) & 0x0F0F0F0F0F0F0F0Full;
    x = (x | (x << 2)) & 0x3333333333333333ull;
    x = (x | (x << 1)) & 0x5555555555555555ull;
    return x;
}

// The merge of the workgroups' histograms costs one device-wide atomic per bin and workgroup, and atomics on one
// address are taken one after the other (about 50 ns each, measured): with 2048 workgroups the merge took four
// times as long as the keys.  Hence at most a few hundred workgroups of 1024 threads.
// prefix (may be NULL): word j receives the top 16 bits of the keys of vertices 2j (low half) and 2j+1.
__global__ __launch_bounds__(SCAN_NT) void sampler_hist_kernel(uint64_t N, uint64_t seed, uint64_t step,
                                                               uint32_t *__restrict__ hist, uint32_t *__restrict__ prefix)
{
    __shared__ uint32_t lh[HIST_BINS];
    for (int i = threadIdx.x; i < HIST_BINS; i += SCAN_NT) lh[i] = 0;
    __syncthreads();
    const uint64_t J = (N + 1) >> 1;
    for (uint64_t j = (uint64_t)blockIdx.x * SCAN_NT + threadIdx.x; j < J; j += (uint64_t)gridDim.x * SCAN_NT) {
        uint64_t ke, ko;
        vertex_pair_keys(j, seed, step, ke, ko);
        atomicAdd(&lh[ke >> (64 - HIST_BITS)], 1u);
        if (2 * j + 1 < N) atomicAdd(&lh[ko >> (64 - HIST_BITS)], 1u);
        if (prefix) prefix[j] = (uint32_t)(ke >> 48) | ((uint32_t)(ko >> 48) << 16);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < HIST_BINS; i += SCAN_NT) {
        uint32_t c = lh[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// Workgroup-local candidate list: matches are rare, so a workgroup gathers its own in LDS and reserves room in the
// global list with ONE atomic add, instead of one add per match on a single hot address.
template <uint32_t LCAP> struct cand_lds {
    uint64_t key[LCAP];
    uint32_t v[LCAP];
    uint32_t n, base, fail;
};

template <uint32_t LCAP>
__device__ __forceinline__ void cand_append(cand_lds<LCAP> &l, bool me, bool mo, uint64_t ke, uint64_t ko, uint64_t j,
                                            sampler_state *__restrict__ state, uint64_t *__restrict__ cand_key,
                                            uint32_t *__restrict__ cand_v, uint32_t cap, uint32_t *__restrict__ status)
{
    if (!(me || mo)) return;
    const uint32_t cnt = (me ? 1u : 0u) + (mo ? 1u : 0u);
    uint32_t p = atomicAdd(&l.n, cnt);
    if (p + cnt <= LCAP) {
        if (me) { l.key[p] = ke; l.v[p] = (uint32_t)(2 * j); ++p; }
        if (mo) { l.key[p] = ko; l.v[p] = (uint32_t)(2 * j + 1); }
    } else {
        // the local list is full (far beyond the expected load): straight to the global list.
        // Reservations only grow, so every one before the first that failed fitted, and they
        // fill [0, first failing offset) without holes.
        atomicMin(&l.fail, p);
        uint32_t q = atomicAdd(&state->ncand, cnt);
        if (me) { if (q < cap) { cand_key[q] = ke; cand_v[q] = (uint32_t)(2 * j); } else atomicOr(status, SGNN_ST_CAND_OVERFLOW); ++q; }
        if (mo) { if (q < cap) { cand_key[q] = ko; cand_v[q] = (uint32_t)(2 * j + 1); } else atomicOr(status, SGNN_ST_CAND_OVERFLOW); }
    }
}

// every thread of the workgroup; NT threads
template <uint32_t LCAP, int NT>
__device__ __forceinline__ void cand_flush(cand_lds<LCAP> &l, sampler_state *__restrict__ state, uint64_t *__restrict__ cand_key,
                                           uint32_t *__restrict__ cand_v, uint32_t cap, uint32_t *__restrict__ status)
{
    __syncthreads();
    const uint32_t n_local = min(l.n, l.fail);
    if (threadIdx.x == 0) l.base = n_local ? atomicAdd(&state->ncand, n_local) : 0u;
    __syncthreads();
    const uint32_t base = l.base;
    for (uint32_t i = threadIdx.x; i < n_local; i += NT) {
        if (base + i < cap) { cand_key[base + i] = l.key[i]; cand_v[base + i] = l.v[i]; }
        else atomicOr(status, SGNN_ST_CAND_OVERFLOW);
    }
}

// The one pass over the keys of a windowed call.  For a sparse sample of a large graph the bin of the threshold is
// known before any key is: the B-th smallest of N uniform keys lies at B/N of the key range, give or take
// sqrt(B (1 - B/N)) / N of it, so the host names a window [b_lo, b_hi] of one or two histogram bins that holds it
// (six standard deviations either side).  This pass then does three things with every key while it has it: counts
// its bin, appends it to the candidate list if the bin is in the window, and sets the vertex's bit in the output
// bitmap if the bin lies below the window (such a vertex is in the sample whatever the threshold turns out to be).
// Nothing per vertex is stored for later passes - no key prefixes - and no later pass touches a key again: the
// threshold comes from the candidates, the candidates at or below it get their bits set (sampler_mark_kernel), and
// the bitmap is complete.  If the threshold's bin is outside the window after all
// (sampler_pick_bin_kernel checks), the recomputing passes run instead and overwrite everything.
constexpr uint32_t WIN_LCAP = 2048;
__global__ __launch_bounds__(SCAN_NT) void sampler_hist_window_kernel(uint64_t N, uint64_t seed, uint64_t step,
                                                                      uint32_t *__restrict__ hist, uint32_t b_lo, uint32_t b_hi,
                                                                      sampler_state *__restrict__ state,
                                                                      uint64_t *__restrict__ cand_key, uint32_t *__restrict__ cand_v,
                                                                      uint32_t cap, uint32_t *__restrict__ status,
                                                                      uint64_t *__restrict__ bitmap, uint64_t W)
{
    __shared__ uint32_t lh[HIST_BINS];
    __shared__ cand_lds<WIN_LCAP> cl;
    __shared__ __attribute__((aligned(8))) uint8_t strip[SCAN_NT / 64][64];
    for (int i = threadIdx.x; i < HIST_BINS; i += SCAN_NT) lh[i] = 0;
    if (threadIdx.x == 0) { cl.n = 0; cl.fail = 0xffffffffu; }
    __syncthreads();
    const unsigned wave = threadIdx.x >> 6, lane = lane_id();
    // A wavefront takes eight bitmap words (512 vertices) per round: lane l computes the keys of vertices 8l .. 8l+7 of
    // the span (four Philox blocks) and reduces them to one byte of the bitmap; the 64 bytes pass through a
    // wavefront-private strip of LDS, from which lanes 0 .. 7 read and write their eight words with one 64-byte store
    // (as the emit pass over stored prefixes does: no bit interleaving of ballots).
    volatile uint8_t *my_bytes = strip[wave];
    volatile uint64_t *my_words = reinterpret_cast<volatile uint64_t *>(strip[wave]);
    const uint64_t W8 = (W + 7) & ~7ull;
    for (uint64_t wb = ((uint64_t)blockIdx.x * (SCAN_NT / 64) + wave) * 8; wb < W8; wb += (uint64_t)gridDim.x * (SCAN_NT / 64) * 8) {
        const uint64_t v0 = wb * 64 + 8 * lane;                  // first of the lane's eight vertices
        uint32_t byte = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint64_t ve = v0 + 2 * q, vo = ve + 1;
            if (ve < N) {
                uint64_t ke, ko;
                vertex_pair_keys(ve >> 1, seed, step, ke, ko);
                const uint32_t be_ = (uint32_t)(ke >> (64 - HIST_BITS)), bo_ = (uint32_t)(ko >> (64 - HIST_BITS));
                atomicAdd(&lh[be_], 1u);
                const bool me = be_ >= b_lo && be_ <= b_hi;
                bool mo = false;
                byte |= (be_ < b_lo ? 1u : 0u) << (2 * q);
                if (vo < N) {
                    atomicAdd(&lh[bo_], 1u);
                    mo = bo_ >= b_lo && bo_ <= b_hi;
                    byte |= (bo_ < b_lo ? 1u : 0u) << (2 * q + 1);
                }
                cand_append(cl, me, mo, ke, ko, ve >> 1, state, cand_key, cand_v, cap, status);
            }
        }
        my_bytes[lane] = (uint8_t)byte;          // volatile: written and read in program order; LDS serves a wavefront in order
        if (lane < 8) {
            const uint64_t word = my_words[lane];
            if (wb + lane < W) bitmap[wb + lane] = word;
        }
    }
    cand_flush<WIN_LCAP, SCAN_NT>(cl, state, cand_key, cand_v, cap, status);
    for (int i = threadIdx.x; i < HIST_BINS; i += SCAN_NT) {
        uint32_t c = lh[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// One workgroup of 1024 threads, two bins a thread.  Leaves the histogram zeroed for the next call.
// windowed: the candidates of bins b_lo .. b_hi are in the list already; they stay if the threshold's bin is one of
// those, otherwise the list is emptied and the call falls back to the recomputing passes.
__global__ __launch_bounds__(1024) void sampler_pick_bin_kernel(uint32_t B, uint32_t *__restrict__ hist,
                                                                sampler_state *__restrict__ state, int windowed, uint32_t b_lo,
                                                                uint32_t b_hi)
{
    __shared__ uint32_t lds[1024 / 64 + 1];
    const uint32_t h0 = hist[2 * threadIdx.x], h1 = hist[2 * threadIdx.x + 1];
    hist[2 * threadIdx.x] = 0;
    hist[2 * threadIdx.x + 1] = 0;
    uint32_t total;
    const uint32_t ex = block_excl_scan<uint32_t, 1024>(h0 + h1, &total, lds);
    // exactly one thread owns the bin of the B-th smallest key (1 <= B <= N)
    uint32_t bin = 0xffffffffu, r = 0;
    if (ex < B && B <= ex + h0) { bin = 2 * threadIdx.x; r = B - ex; }
    else if (ex + h0 < B && B <= ex + h0 + h1) { bin = 2 * threadIdx.x + 1; r = B - ex - h0; }
    if (bin != 0xffffffffu) {
        // with a window, r counts inside the threshold's bin as always: the threshold pass looks only at the candidates of that bin
        const bool miss = windowed && (bin < b_lo || bin > b_hi);
        state->bin = bin;
        state->r = r;
        state->fallback = miss ? 1u : 0u;
        if (!windowed || miss) state->ncand = 0;
    }
}

template <bool PREFIX>
__global__ __launch_bounds__(SCAN_NT) void sampler_collect_kernel(uint64_t N, uint64_t seed, uint64_t step,
                                                                  sampler_state *__restrict__ state,
                                                                  uint64_t *__restrict__ cand_key,
                                                                  uint32_t *__restrict__ cand_v, uint32_t cap,
                                                                  uint32_t *__restrict__ status,
                                                                  const uint32_t *__restrict__ prefix, int only_on_fallback)
{
    // Matches are rare (one vertex in 2048): gathered per workgroup (cand_lds).
    constexpr uint32_t LCAP = 1024;
    __shared__ cand_lds<LCAP> cl;
    if (only_on_fallback && !state->fallback) return;      // a windowed call that found its threshold bin in the window
    const uint32_t bin = state->bin;
    const uint64_t J = (N + 1) >> 1;
    if (threadIdx.x == 0) { cl.n = 0; cl.fail = 0xffffffffu; }
    __syncthreads();
    auto append = [&](bool me, bool mo, uint64_t ke, uint64_t ko, uint64_t j) {
        cand_append(cl, me, mo, ke, ko, j, state, cand_key, cand_v, cap, status);
    };
    const uint64_t J_rounds = PREFIX ? (J + 3) / 4 : J;      // loop items: quads of prefix words, or Philox blocks
    for (uint64_t j = (uint64_t)blockIdx.x * SCAN_NT + threadIdx.x; j < J_rounds; j += (uint64_t)gridDim.x * SCAN_NT) {
        if constexpr (PREFIX) {
            // a thread takes four prefix words (eight vertices) per round; the stored prefixes hold the bin, and the
            // keys themselves are computed for the matches only
            const uint4 pp4 = *reinterpret_cast<const uint4 *>(prefix + 4 * j);      // the array is padded to whole quads
            const uint32_t pw[4] = {pp4.x, pp4.y, pp4.z, pp4.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint64_t jj = 4 * j + q;
                const bool he = 2 * jj < N && ((pw[q] & 0xffffu) >> (16 - HIST_BITS)) == bin;
                const bool ho = 2 * jj + 1 < N && (pw[q] >> (32 - HIST_BITS)) == bin;
                if (he || ho) {
                    uint64_t k0, k1;
                    vertex_pair_keys(jj, seed, step, k0, k1);
                    append(he, ho, k0, k1, jj);
                }
            }
        } else {
            uint64_t ke, ko;
            vertex_pair_keys(j, seed, step, ke, ko);
            append((uint32_t)(ke >> (64 - HIST_BITS)) == bin, (2 * j + 1 < N) && (uint32_t)(ko >> (64 - HIST_BITS)) == bin, ke, ko, j);
        }
    }
    cand_flush<LCAP, SCAN_NT>(cl, state, cand_key, cand_v, cap, status);
}

// Exact r-th smallest (key, v) among the candidates: most-significant-digit radix select over the
// 96-bit composite, 8 bits a pass, starting below the 11 bits that all candidates share.  One
// workgroup; a thread keeps its first THR_R candidates in registers, so that a pass costs no memory
// traffic, and the passes stop as soon as the chosen digit holds a single candidate (after three or
// four of them for keys that differ, instead of eleven).
constexpr int THR_R = 12;

__global__ __launch_bounds__(1024) void sampler_threshold_kernel(sampler_state *__restrict__ state,
                                                                 const uint64_t *__restrict__ cand_key,
                                                                 const uint32_t *__restrict__ cand_v, uint32_t cap)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel_digit, sel_r, sel_cnt;
    __shared__ uint64_t found_key;
    __shared__ uint32_t found_v;
    const uint32_t n = min(state->ncand, cap);
    uint32_t r = state->r;
    uint64_t rk[THR_R];
    uint32_t rv[THR_R];
#pragma unroll
    for (int q = 0; q < THR_R; ++q) {
        const uint32_t i = q * 1024 + threadIdx.x;
        rk[q] = i < n ? cand_key[i] : 0ull;
        rv[q] = i < n ? cand_v[i] : 0u;
    }
    uint64_t pk = (uint64_t)state->bin << (64 - HIST_BITS);   // decided high bits of the key
    uint32_t pv = 0;                                          // decided high bits of the vertex
    int kd = HIST_BITS, vd = 0;                               // how many of each are decided
    if (threadIdx.x == 0) sel_cnt = 0;

    // does (k, v) agree with every decided bit?
    auto agrees = [&](uint64_t k, uint32_t v) {
        if ((k >> (64 - kd)) != (pk >> (64 - kd))) return false;
        return vd == 0 || (v >> (32 - vd)) == (pv >> (32 - vd));
    };
    bool single = false;
    while (kd < 64 || vd < 32) {
        const bool in_key = kd < 64;
        const int width = in_key ? min(8, 64 - kd) : 8;
        const int lo = in_key ? 64 - kd - width : 32 - vd - 8;
        const uint32_t dmask = (1u << width) - 1u;
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        auto count = [&](uint64_t k, uint32_t v) {
            if (agrees(k, v)) atomicAdd(&hist[(in_key ? (uint32_t)(k >> lo) : (v >> lo)) & dmask], 1u);
        };
#pragma unroll
        for (int q = 0; q < THR_R; ++q)
            if (q * 1024 + threadIdx.x < n) count(rk[q], rv[q]);
        for (uint32_t i = THR_R * 1024 + threadIdx.x; i < n; i += 1024) count(cand_key[i], cand_v[i]);
        __syncthreads();
        if (threadIdx.x < 64) {
            // lane l owns digits 4l .. 4l+3
            const uint32_t a0 = hist[4 * threadIdx.x], a1 = hist[4 * threadIdx.x + 1], a2 = hist[4 * threadIdx.x + 2],
                           a3 = hist[4 * threadIdx.x + 3];
            const uint32_t s = a0 + a1 + a2 + a3;
            const uint32_t ex = wave_incl_scan(s) - s;
            if (ex < r && r <= ex + s) {
                uint32_t d = 4 * threadIdx.x, e = ex, c = a0;
                if (r > e + a0) { e += a0; ++d; c = a1; if (r > e + a1) { e += a1; ++d; c = a2; if (r > e + a2) { e += a2; ++d; c = a3; } } }
                sel_digit = d;
                sel_r = r - e;
                sel_cnt = c;
            }
        }
        __syncthreads();
        const uint32_t d = sel_digit;
        r = sel_r;
        single = sel_cnt == 1;
        if (in_key) { pk |= (uint64_t)d << lo; kd += width; }
        else { pv |= d << lo; vd += 8; }
        __syncthreads();
        if (single) break;
    }
    if (single) {
        // exactly one candidate agrees with the decided bits: it is the threshold
        auto take = [&](uint64_t k, uint32_t v) {
            if (agrees(k, v)) { found_key = k; found_v = v; }
        };
#pragma unroll
        for (int q = 0; q < THR_R; ++q)
            if (q * 1024 + threadIdx.x < n) take(rk[q], rv[q]);
        for (uint32_t i = THR_R * 1024 + threadIdx.x; i < n; i += 1024) take(cand_key[i], cand_v[i]);
        __syncthreads();
        pk = found_key;
        pv = found_v;
    }
    if (threadIdx.x == 0) {
        state->thr_key = pk;
        state->thr_v = pv;
        state->nmark = n;
        state->ncand = 0;      // every thread read it long ago (barriers above): the list is empty for the next call
    }
}

// Windowed calls: the candidates at or below the threshold get their bits (the vertices of the bins below the window
// have theirs from the key pass), then the workgroup counts the rank pass wants.
__global__ __launch_bounds__(SAMP_NT) void sampler_mark_kernel(const sampler_state *__restrict__ state,
                                                               const uint64_t *__restrict__ cand_key,
                                                               const uint32_t *__restrict__ cand_v, uint64_t *__restrict__ bitmap)
{
    if (state->fallback) return;
    const uint64_t tk = state->thr_key;
    const uint32_t tv = state->thr_v, n = state->nmark;
    for (uint32_t i = blockIdx.x * SAMP_NT + threadIdx.x; i < n; i += gridDim.x * SAMP_NT) {
        const uint64_t k = cand_key[i];
        const uint32_t v = cand_v[i];
        if (k < tk || (k == tk && v <= tv)) atomicOr((unsigned long long *)&bitmap[v >> 6], 1ull << (v & 63));
    }
}

__global__ __launch_bounds__(SAMP_NT) void sampler_count_kernel(const sampler_state *__restrict__ state,
                                                                const uint64_t *__restrict__ bitmap, uint64_t W, uint64_t wpw,
                                                                uint32_t *__restrict__ wg_count)
{
    __shared__ uint32_t lds[SAMP_NT / 64];
    if (state->fallback) return;       // the recomputing emit pass has written bitmap and counts
    const uint64_t wbeg = (uint64_t)blockIdx.x * wpw;
    const uint64_t wend = min(W, wbeg + wpw);
    uint32_t cnt = 0;
    for (uint64_t w = wbeg + threadIdx.x; w < wend; w += SAMP_NT) cnt += (uint32_t)__popcll(bitmap[w]);
    cnt = block_sum<uint32_t, SAMP_NT>(cnt, lds);
    if (threadIdx.x == 0) wg_count[blockIdx.x] = cnt;
}


// Workgroup g owns bitmap words [g*wpw, (g+1)*wpw), wpw a multiple of 8.  A wavefront takes 64 words
// at a time and builds two of them per iteration: lane l evaluates vertices 2j and 2j+1 of Philox block
// j = 32*w0 + l.  Lane l keeps word l of the 64, so that the wave writes them with one 512-byte store:
// an 8-byte store by a single lane per word reached memory as a partial write of its own, a quarter of a
// million of them at a rate of about one per nanosecond.
__global__ __launch_bounds__(SAMP_NT) void sampler_emit_kernel(uint64_t N, uint64_t seed, uint64_t step,
                                                               const sampler_state *__restrict__ state,
                                                               uint64_t *__restrict__ bitmap, uint64_t W, uint64_t wpw,
                                                               uint32_t *__restrict__ wg_count, int only_on_fallback)
{
    __shared__ uint32_t lds[SAMP_NT / 64];
    if (only_on_fallback && !state->fallback) return;
    const uint64_t tk = state->thr_key;
    const uint32_t tv = state->thr_v;
    const uint64_t wbeg = (uint64_t)blockIdx.x * wpw;
    const uint64_t wend = min(W, wbeg + wpw);
    const unsigned wave = threadIdx.x >> 6, lane = lane_id();
    uint32_t cnt = 0;
    for (uint64_t chunk = wbeg + 64 * wave; chunk < wend; chunk += 64 * (SAMP_NT / 64)) {
        uint64_t mine = 0;
        for (unsigned it = 0; it < 32; ++it) {
            const uint64_t w0 = chunk + 2 * it;
            if (w0 >= wend) break;
            const uint64_t j = w0 * 32 + lane;
            const uint64_t ve = 2 * j, vo = 2 * j + 1;
            bool ie = false, io = false;
            if (ve < N) {
                uint64_t ke, ko;
                vertex_pair_keys(j, seed, step, ke, ko);
                ie = ke < tk || (ke == tk && (uint32_t)ve <= tv);
                io = vo < N && (ko < tk || (ko == tk && (uint32_t)vo <= tv));
            }
            const uint64_t be = __ballot(ie), bo = __ballot(io);
            const uint64_t word0 = spread_even((uint32_t)be) | (spread_even((uint32_t)bo) << 1);
            const uint64_t word1 = spread_even((uint32_t)(be >> 32)) | (spread_even((uint32_t)(bo >> 32)) << 1);
            if (lane == 2 * it) mine = word0;
            if (lane == 2 * it + 1) mine = word1;
            cnt += __popcll(word0) + __popcll(word1);
        }
        if (chunk + lane < wend) bitmap[chunk + lane] = mine;
    }
    if (lane == 0) lds[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int i = 0; i < SAMP_NT / 64; ++i) t += lds[i];
        wg_count[blockIdx.x] = t;
    }
}

// The same from the stored key prefixes.  A wavefront takes eight bitmap words (512 vertices) per round: lane l
// loads the prefixes of vertices 8l .. 8l+7 of the span with one 16-byte load and reduces them to one byte of the
// bitmap (a prefix below the threshold's is in, one above is out, an equal one - 2^-16 of the vertices - has its key
// computed again); the 64 bytes pass through a wavefront-private strip of LDS, from which lanes 0 .. 7 read and
// write their eight words with one 64-byte store.  No scalar bit interleaving, no key arithmetic.
__global__ __launch_bounds__(SAMP_NT) void sampler_emit_prefix_kernel(uint64_t N, uint64_t seed, uint64_t step,
                                                                      const sampler_state *__restrict__ state,
                                                                      uint64_t *__restrict__ bitmap, uint64_t W, uint64_t wpw,
                                                                      uint32_t *__restrict__ wg_count,
                                                                      const uint32_t *__restrict__ prefix)
{
    __shared__ uint32_t lds[SAMP_NT / 64];
    __shared__ __attribute__((aligned(8))) uint8_t strip[SAMP_NT / 64][64];
    const uint64_t tk = state->thr_key;
    const uint32_t tv = state->thr_v;
    const uint32_t tp = (uint32_t)(tk >> 48);
    const uint64_t wbeg = (uint64_t)blockIdx.x * wpw;
    const uint64_t wend = min(W, wbeg + wpw);
    const unsigned wave = threadIdx.x >> 6, lane = lane_id();
    volatile uint8_t *my_bytes = strip[wave];
    volatile uint64_t *my_words = reinterpret_cast<volatile uint64_t *>(strip[wave]);
    uint32_t cnt = 0;
    // wbeg and wpw are multiples of 8: a round's eight words lie inside [wbeg, wend) or behind W (vertices >= N: empty)
    for (uint64_t wb = wbeg + 8 * wave; wb < wend; wb += 8 * (SAMP_NT / 64)) {
        const uint64_t v0 = wb * 64 + 8 * lane;                  // first of the lane's eight vertices
        uint32_t byte = 0;
        if (v0 < N) {
            const uint4 pp4 = *reinterpret_cast<const uint4 *>(prefix + (v0 >> 1));      // the array is padded to whole quads
            const uint32_t pw[4] = {pp4.x, pp4.y, pp4.z, pp4.w};
            bool tie = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t pe = pw[q] & 0xffffu, po = pw[q] >> 16;
                byte |= (pe < tp ? 1u : 0u) << (2 * q) | (po < tp ? 1u : 0u) << (2 * q + 1);
                tie = tie || pe == tp || po == tp;
            }
            if (tie) {
#pragma unroll 1
                for (int q = 0; q < 4; ++q) {
                    const uint32_t pe = pw[q] & 0xffffu, po = pw[q] >> 16;
                    if (pe != tp && po != tp) continue;
                    const uint64_t ve = v0 + 2 * q, vo = ve + 1;
                    uint64_t ke, ko;
                    vertex_pair_keys(ve >> 1, seed, step, ke, ko);
                    const uint32_t ie = (ke < tk || (ke == tk && (uint32_t)ve <= tv)) ? 1u : 0u;
                    const uint32_t io = (ko < tk || (ko == tk && (uint32_t)vo <= tv)) ? 1u : 0u;
                    byte = (byte & ~(3u << (2 * q))) | ie << (2 * q) | io << (2 * q + 1);
                }
            }
            // vertices at and behind N (the odd partner of the last vertex, the padding of the last quad) are out
            if (v0 + 8 > N) byte &= (1u << (N - v0)) - 1u;
        }
        my_bytes[lane] = (uint8_t)byte;          // volatile: written and read in program order; LDS serves a wavefront in order
        if (lane < 8) {
            const uint64_t word = my_words[lane];
            if (wb + lane < wend) bitmap[wb + lane] = word;
            cnt += (uint32_t)__popcll(word);
        }
    }
    cnt = wave_sum(cnt);
    if (lane == 0) lds[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int i = 0; i < SAMP_NT / 64; ++i) t += lds[i];
        wg_count[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(SAMP_NT) void sampler_rank_kernel(const uint64_t *__restrict__ bitmap, uint64_t W,
                                                               uint64_t wpw, const uint32_t *__restrict__ wg_count,
                                                               uint32_t B, uint32_t *__restrict__ rank,
                                                               int32_t *__restrict__ S, uint32_t *__restrict__ status)
{
    __shared__ uint32_t lds[SAMP_NT / 64 + 1];
    // sampled vertices in all earlier workgroups
    uint32_t part = 0;
    for (unsigned i = threadIdx.x; i < blockIdx.x; i += SAMP_NT) part += wg_count[i];
    uint32_t running = block_sum<uint32_t, SAMP_NT>(part, lds);
    const uint64_t wbeg = (uint64_t)blockIdx.x * wpw;
    const uint64_t wend = min(W, wbeg + wpw);
    for (uint64_t base = wbeg; base < wend; base += SAMP_NT) {
        const uint64_t w = base + threadIdx.x;
        uint64_t word = w < wend ? bitmap[w] : 0ull;
        uint32_t total;
        uint32_t ex = block_excl_scan<uint32_t, SAMP_NT>(__popcll(word), &total, lds) + running;
        if (w < wend) rank[w] = ex;
        while (word) {
            const int b = __ffsll((unsigned long long)word) - 1;
            if (ex < B) S[ex] = (int32_t)(w * 64 + b);
            ++ex;
            word &= word - 1;
        }
        running += total;
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0 && running != B) atomicOr(status, SGNN_ST_CAND_OVERFLOW);
}

} // namespace

// scratch layout of the sampler inside the context's persistent area
size_t sgnn_sampler_persist_bytes() { return HIST_BINS * sizeof(uint32_t) + 256; }

static uint32_t cand_capacity(uint64_t N) { return (uint32_t)(2 * (N >> HIST_BITS) + 8192); }

// the key prefixes pay once a pass over the keys costs more than their traffic; below that the keys are recomputed
static size_t prefix_bytes(uint64_t N) { return N >= (1ull << 20) ? (size_t)(((N + 1) >> 1) + 4) * sizeof(uint32_t) : 0; }   // padded to whole quads

size_t sgnn_sampler_ws_bytes(uint64_t N)
{
    const size_t cap = cand_capacity(N);
    return cap * 12 + EMIT_MAX_WG * 4 + 4 * 256 + prefix_bytes(N) + 256;
}

// The six launches.  ctx may be NULL (no profiling, errors through sgnn_fail(NULL, ...)); every buffer
// comes from the caller of this function: hist (HIST_BINS words, zero on entry, left zero), state,
// the candidate list of `cap` entries, EMIT_MAX_WG workgroup counts and the sticky status word.
#define SAMP_LAUNCH(name, kernel, grid, block, ...)                                                        \
    do {                                                                                                  \
        if (ctx && ctx->prof_on) sgnn_prof_begin(ctx, st, name, "");                                       \
        hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                                       \
        if (ctx && ctx->prof_on) sgnn_prof_end(ctx, st);                                                   \
        SGNN_LAUNCH_CHECK(ctx, name);                                                                     \
    } while (0)

// Window of histogram bins that holds the threshold of a sparse sample of a large graph (see
// sampler_hist_window_kernel): the B-th smallest of N uniform keys lies at x = B/N of the key range with a standard
// deviation of sqrt(B (1 - B/N)) / N; six of them either side must span at most two bins, or there is no window.
// shift: moves the window by whole bins (a test's way to the fallback passes; 0 in use).
struct sampler_window { int on; uint32_t b_lo, b_hi; };
static sampler_window sampler_window_for(uint64_t N, uint32_t B, int shift)
{
    sampler_window w = {0, 0, 0};
    if (N < (1ull << 20) || (uint64_t)B * 4 > N) return w;
    const double p = (double)B / (double)N, x = p * HIST_BINS;
    const double h = 6.0 * HIST_BINS * std::sqrt((double)B * (1.0 - p)) / (double)N + 1e-6;
    if (h >= 0.45) return w;
    const long lo = std::lround(std::floor(x - h)) + shift, hi = std::lround(std::floor(x + h)) + shift;
    w.on = 1;
    w.b_lo = (uint32_t)std::min<long>(std::max<long>(lo, 0), HIST_BINS - 1);
    w.b_hi = (uint32_t)std::min<long>(std::max<long>(hi, 0), HIST_BINS - 1);
    return w;
}

static int sampler_launches(sgnn_ctx *ctx, uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S,
                            uint64_t *bitmap, uint32_t *rank, uint32_t *hist, sampler_state *state, uint64_t *cand_key,
                            uint32_t *cand_v, uint32_t cap, uint32_t *wg_count, uint32_t *status, uint32_t *prefix,
                            sampler_window win, hipStream_t st)
{
    const uint64_t J = (N + 1) >> 1;
    const unsigned grid =
        (unsigned)std::min<uint64_t>(cdiv(J, SCAN_NT), std::min<uint64_t>(std::max<uint64_t>(256, N >> 19), 2048));
    const uint64_t W = (N + 63) / 64;
    const unsigned egrid = (unsigned)std::min<uint64_t>(cdiv(W, 8), EMIT_MAX_WG);
    const uint64_t wpw = (uint64_t)cdiv(cdiv(W, egrid), 8) * 8;
    if (win.on) {
        // one pass over the keys; the passes marked "fallback" leave at once unless the threshold's bin missed the window
        SAMP_LAUNCH("sampler_hist_window_kernel", sampler_hist_window_kernel, dim3(grid), dim3(SCAN_NT), N, seed, step, hist, win.b_lo, win.b_hi,
                    state, cand_key, cand_v, cap, status, bitmap, W);
        SAMP_LAUNCH("sampler_pick_bin_kernel", sampler_pick_bin_kernel, dim3(1), dim3(1024), B, hist, state, 1, win.b_lo, win.b_hi);
        SAMP_LAUNCH("sampler_collect_kernel", sampler_collect_kernel<false>, dim3(grid), dim3(SCAN_NT), N, seed, step, state, cand_key,
                    cand_v, cap, status, (const uint32_t *)nullptr, 1);      // fallback
        SAMP_LAUNCH("sampler_threshold_kernel", sampler_threshold_kernel, dim3(1), dim3(1024), state, cand_key, cand_v, cap);
        SAMP_LAUNCH("sampler_mark_kernel", sampler_mark_kernel, dim3(64), dim3(SAMP_NT), (const sampler_state *)state,
                    (const uint64_t *)cand_key, (const uint32_t *)cand_v, bitmap);
        SAMP_LAUNCH("sampler_emit_kernel", sampler_emit_kernel, dim3(egrid), dim3(SAMP_NT), N, seed, step, state, bitmap, W, wpw,
                    wg_count, 1);                                            // fallback
        SAMP_LAUNCH("sampler_count_kernel", sampler_count_kernel, dim3(egrid), dim3(SAMP_NT), (const sampler_state *)state,
                    (const uint64_t *)bitmap, W, wpw, wg_count);
        SAMP_LAUNCH("sampler_rank_kernel", sampler_rank_kernel, dim3(egrid), dim3(SAMP_NT), bitmap, W, wpw, wg_count, B, rank, S,
                    status);
        return SGNN_OK;
    }
    SAMP_LAUNCH("sampler_hist_kernel", sampler_hist_kernel, dim3(grid), dim3(SCAN_NT), N, seed, step, hist, prefix);
    SAMP_LAUNCH("sampler_pick_bin_kernel", sampler_pick_bin_kernel, dim3(1), dim3(1024), B, hist, state, 0, 0u, 0u);
    if (prefix)
        SAMP_LAUNCH("sampler_collect_kernel", sampler_collect_kernel<true>, dim3(grid), dim3(SCAN_NT), N, seed, step, state, cand_key,
                    cand_v, cap, status, (const uint32_t *)prefix, 0);
    else
        SAMP_LAUNCH("sampler_collect_kernel", sampler_collect_kernel<false>, dim3(grid), dim3(SCAN_NT), N, seed, step, state, cand_key,
                    cand_v, cap, status, (const uint32_t *)nullptr, 0);
    SAMP_LAUNCH("sampler_threshold_kernel", sampler_threshold_kernel, dim3(1), dim3(1024), state, cand_key, cand_v, cap);

    if (prefix)
        SAMP_LAUNCH("sampler_emit_kernel", sampler_emit_prefix_kernel, dim3(egrid), dim3(SAMP_NT), N, seed, step, state, bitmap, W,
                    wpw, wg_count, (const uint32_t *)prefix);
    else
        SAMP_LAUNCH("sampler_emit_kernel", sampler_emit_kernel, dim3(egrid), dim3(SAMP_NT), N, seed, step, state, bitmap, W, wpw,
                    wg_count, 0);
    SAMP_LAUNCH("sampler_rank_kernel", sampler_rank_kernel, dim3(egrid), dim3(SAMP_NT), bitmap, W, wpw, wg_count, B, rank, S,
                status);
    return SGNN_OK;
}

int sgnn_launch_sampler(sgnn_ctx *ctx, uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S,
                        uint64_t *bitmap, uint32_t *rank, hipStream_t st)
{
    uint32_t *hist = reinterpret_cast<uint32_t *>(ctx->persist);
    sampler_state *state = reinterpret_cast<sampler_state *>(ctx->persist + HIST_BINS * sizeof(uint32_t));
    ws_alloc ws(ctx);
    const uint32_t cap = cand_capacity(N);
    uint64_t *cand_key = ws.get<uint64_t>(cap);
    uint32_t *cand_v = ws.get<uint32_t>(cap);
    uint32_t *wg_count = ws.get<uint32_t>(EMIT_MAX_WG);
    // SGNN_SAMPLER_WINDOW_SHIFT: whole bins by which the window is moved off its place (tests of the fallback passes)
    const char *shift_env = std::getenv("SGNN_SAMPLER_WINDOW_SHIFT");
    const sampler_window win = sampler_window_for(N, B, shift_env ? std::atoi(shift_env) : 0);
    // a windowed call stores nothing per vertex; otherwise two bytes of key prefix per vertex from 2^20 vertices on
    uint32_t *prefix = (!win.on && prefix_bytes(N)) ? ws.get<uint32_t>(prefix_bytes(N) / sizeof(uint32_t)) : nullptr;
    if (!ws.ok)
        return sgnn_fail(ctx, SGNN_ERR_CAPACITY, "sgnn_sample_uniform: scratch too small (%zu bytes needed): call sgnn_ctx_reserve",
                         ws.off);
    return sampler_launches(ctx, N, B, seed, step, S, bitmap, rank, hist, state, cand_key, cand_v, cap, wg_count, ctx->status, prefix, win,
                            st);
}

// ---- the same sampler without any allocation: scratch in a file-scope device array ---------------------

namespace {

constexpr uint64_t STATIC_MAX_N = SGNN_STATIC_SAMPLER_MAX_N;
constexpr uint32_t STATIC_CAP = (uint32_t)(2 * (STATIC_MAX_N >> HIST_BITS) + 8192);     // cand_capacity(STATIC_MAX_N)
constexpr size_t ST_HIST = 0;                                        // uint32[HIST_BINS]
constexpr size_t ST_STATE = ST_HIST + HIST_BINS * sizeof(uint32_t);  // sampler_state
constexpr size_t ST_STATUS = ST_STATE + 256;                         // uint32 sticky status (when the caller passes none)
constexpr size_t ST_WG = ST_STATUS + 256;                            // uint32[EMIT_MAX_WG]
constexpr size_t ST_CKEY = ST_WG + EMIT_MAX_WG * sizeof(uint32_t);   // uint64[STATIC_CAP]
constexpr size_t ST_CV = ST_CKEY + (size_t)STATIC_CAP * sizeof(uint64_t);   // uint32[STATIC_CAP]
constexpr size_t ST_BYTES = (ST_CV + (size_t)STATIC_CAP * sizeof(uint32_t) + 255) & ~size_t(255);
constexpr int MAX_DEVICES = 64;

// zeroes the histogram and the selection state: the array keeps the last call's contents, and a call that
// was abandoned half way (a failed launch) may have left counts behind
__global__ __launch_bounds__(SAMP_NT) void sampler_static_clear_kernel(uint32_t *__restrict__ words, uint32_t n)
{
    for (uint32_t i = blockIdx.x * SAMP_NT + threadIdx.x; i < n; i += gridDim.x * SAMP_NT) words[i] = 0;
}

} // namespace

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) uint8_t scratch[ST_BYTES];

// device address of `scratch` on each GPU, resolved once per device with that device current
static uint8_t *g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

static int static_scratch(int device, uint8_t **out)
{
    if (device < 0 || device >= MAX_DEVICES)
        return sgnn_fail(nullptr, SGNN_ERR_UNSUPPORTED, "sgnn_sample_uniform_static: device %d outside the supported 0..%d", device,
                         MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        uint8_t *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return sgnn_fail(nullptr, SGNN_ERR_HIP, "sgnn_sample_uniform_static: hipGetSymbolAddress failed on device %d: %s", device,
                             hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SGNN_OK;
}

// Called by sgnn_ctx_create (the library's set-up call) with the context's device current, so that a later
// sgnn_sample_uniform_static on that device finds the address resolved.
int sgnn_static_scratch_init(int device)
{
    uint8_t *p = nullptr;
    return static_scratch(device, &p);
}

extern "C" int sgnn_sample_uniform_static(uint64_t N, uint32_t B, uint64_t seed, uint64_t step, int32_t *S, uint64_t *bitmap,
                                          uint32_t *rank, uint32_t *status_dev, sgnn_stream stream)
{
    if (!S || !bitmap || !rank) return sgnn_fail(nullptr, SGNN_ERR_INVALID_ARG, "sgnn_sample_uniform_static: null output pointer");
    if (B == 0 || B > N)
        return sgnn_fail(nullptr, SGNN_ERR_INVALID_ARG, "sgnn_sample_uniform_static: need 1 <= B <= N (B=%u, N=%llu)", B,
                         (unsigned long long)N);
    if (N > STATIC_MAX_N)
        return sgnn_fail(nullptr, SGNN_ERR_CAPACITY, "sgnn_sample_uniform_static: N = %llu exceeds the %llu vertices the static "
                         "scratch is sized for; use sgnn_sample_uniform with a context", (unsigned long long)N,
                         (unsigned long long)STATIC_MAX_N);
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return sgnn_fail(nullptr, SGNN_ERR_HIP, "sgnn_sample_uniform_static: hipGetDevice failed");
    uint8_t *ptr = nullptr;
    int rc = static_scratch(device, &ptr);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t *hist = reinterpret_cast<uint32_t *>(ptr + ST_HIST);
    sampler_state *state = reinterpret_cast<sampler_state *>(ptr + ST_STATE);
    uint32_t *status = status_dev ? status_dev : reinterpret_cast<uint32_t *>(ptr + ST_STATUS);
    sgnn_ctx *ctx = nullptr;
    // histogram and state are contiguous: one small fill kernel (no memset node: the call may be captured)
    SAMP_LAUNCH("sampler_static_clear_kernel", sampler_static_clear_kernel, dim3(2), dim3(SAMP_NT), hist,
                (uint32_t)((ST_STATUS - ST_HIST) / sizeof(uint32_t)));
    return sampler_launches(nullptr, N, B, seed, step, S, bitmap, rank, hist, state, reinterpret_cast<uint64_t *>(ptr + ST_CKEY),
                            reinterpret_cast<uint32_t *>(ptr + ST_CV), cand_capacity(N), reinterpret_cast<uint32_t *>(ptr + ST_WG),
                            status, nullptr, sampler_window{0, 0, 0}, st);      // no room for key prefixes in the static array: every pass recomputes the keys
}
