// Pieces of the "fitting" requantization that several kernels share: an exact accumulator tensor is stored in
// WL bits with the smallest right shift that makes its largest magnitude fit (the gradient tensors of the
// chained step; Sec. 3.3 "Dealing with Fixed-Points Limited Range" makes their common scale irrelevant).
#pragma once
#include "common.hpp"

namespace adapt {

struct FitArgs {
    const void *acc;
    void *q;
    const uint64_t *part;
    int nparts;
    uint64_t n;
    int wl, mode;
    uint64_t seed, stream;
    int32_t *shift_out;
    unsigned long long *sumsq;
    // exponent of the codes: *e_out = (e_in ? *e_in : 0) + e_add - shift (device memory; e_out may be null)
    const long long *e_in;
    long long e_add;
    long long *e_out;
};

__device__ __forceinline__ uint64_t magnitude(long long v) { return v < 0 ? 0ull - (uint64_t)v : (uint64_t)v; }

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t o = __shfl_xor((unsigned long long)v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// The requantize rule for a shift that was fitted to the tensor: |acc| >> shift is below 2^(wl-1)
// <= 2^15, so after one 64-bit shift everything is 32-bit arithmetic.  floor((acc + r') / 2^s) is
// taken as (acc >> s) + carry of the dropped bits plus r', which cannot overflow.
__device__ __forceinline__ int fit_one(long long acc, int shift, uint32_t r16, int qlo, int qhi)
{
    int q;
    if (shift == 0) {
        q = (int)acc;
    } else if (shift <= 16) {
        const uint32_t low = (uint32_t)acc & ((1u << shift) - 1u);
        q = (int)(acc >> shift) + (int)((low + (r16 >> (16 - shift))) >> shift);
    } else {
        const int t = (int)(acc >> (shift - 16));            // |t| < 2^(wl-1+16) <= 2^31
        q = (t >> 16) + (int)((((uint32_t)t & 0xffffu) + r16) >> 16);
    }
    return min(max(q, qlo), qhi);
}

// shift = max(0, bit_length(m) - (wl - 1)) for the largest magnitude m
__device__ __forceinline__ int fit_shift_of(uint64_t m, int wl)
{
    const int bits = m ? 64 - __clzll((long long)m) : 0;
    return max(0, bits - (wl - 1));
}

// block-wide maximum of per-thread values (all threads get it); sm: one word per wavefront
__device__ __forceinline__ uint64_t block_max_u64(uint64_t m, uint64_t *sm, int nwaves)
{
    m = wave_max_u64(m);
    if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
    __syncthreads();
    m = sm[0];
    for (int i = 1; i < nwaves; ++i) m = sm[i] > m ? sm[i] : m;
    __syncthreads();
    return m;
}

}  // namespace adapt
