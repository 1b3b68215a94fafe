// Wavefront (64 lanes) and workgroup primitives used by the integer kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ unsigned lane_id() { return threadIdx.x & 63u; }

// Inclusive prefix sum across the 64 lanes of a wavefront.
template <class T> __device__ __forceinline__ T wave_incl_scan(T x)
{
    const unsigned lane = lane_id();
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        T y = __shfl_up(x, o, 64);
        if (lane >= (unsigned)o) x += y;
    }
    return x;
}

template <class T> __device__ __forceinline__ T wave_sum(T x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// Exclusive prefix sum over the NT threads of a workgroup (NT a multiple of 64, <= 1024).
// Returns the exclusive prefix of x in thread order and stores the workgroup total in *total.
// lds must hold NT/64 + 1 elements; the call contains two barriers and may be repeated
// immediately (it ends with a barrier).
template <class T, int NT> __device__ __forceinline__ T block_excl_scan(T x, T *total, T *lds)
{
    constexpr int NW = NT / 64;
    const unsigned lane = lane_id(), w = threadIdx.x >> 6;
    T inc = wave_incl_scan(x);
    if (lane == 63) lds[w] = inc;
    __syncthreads();
    if (w == 0) {
        T v = lane < NW ? lds[lane] : T(0);
        T s = wave_incl_scan(v);
        if (lane < NW) lds[lane] = s - v;
        if (lane == NW - 1) lds[NW] = s;
    }
    __syncthreads();
    T res = lds[w] + inc - x;
    *total = lds[NW];
    __syncthreads();
    return res;
}

template <class T, int NT> __device__ __forceinline__ T block_sum(T x, T *lds)
{
    constexpr int NW = NT / 64;
    const unsigned lane = lane_id(), w = threadIdx.x >> 6;
    T s = wave_sum(x);
    if (lane == 0) lds[w] = s;
    __syncthreads();
    T t = T(0);
#pragma unroll
    for (int i = 0; i < NW; ++i) t += lds[i];
    __syncthreads();
    return t;
}

// exp(x) for x <= 0 to about 2 ulp with one hardware exponential: 2^(x log2 e), the rounding error of that product
// (and the low part of log2 e) carried as a first-order correction.  The library expf costs some forty instructions:
// a softmax over 172 classes of a million rows is then bound by them, not by memory.
__device__ __forceinline__ float exp_neg(float x)
{
    const float l2e_hi = 1.44269502162933349609375f, l2e_lo = 1.925963033500011e-8f;
    const float t = x * l2e_hi;
    float r = fmaf(x, l2e_hi, -t);
    r = fmaf(x, l2e_lo, r);
    const float e = __builtin_amdgcn_exp2f(t);        // 0 below 2^-126: such a probability is 0 in fp32 anyway
    return fmaf(e, r * 0.693147182464599609375f, e);
}

// log(s) for s >= 1 with the hardware logarithm (1 ulp of log2 s)
__device__ __forceinline__ float log_ge1(float s) { return __builtin_amdgcn_logf(s) * 0.693147182464599609375f; }

