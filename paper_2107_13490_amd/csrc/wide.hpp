// 128-bit integer pieces shared by the code paths for word lengths 17..32 (Sec. 3.3 bounds the precision that
// PushUp may ask for at 32 bits): codes are int32, products of two codes take 62 bits and their sums more.
#pragma once
#include "common.hpp"

namespace adapt {

typedef __int128 i128;
typedef unsigned __int128 u128;

// the contraction epilogue's rule on a 128-bit accumulator, output of up to 32 bits
__device__ __forceinline__ int requantize_wide_one(i128 acc, int shift, int wl, int relu, uint32_t r16)
{
    i128 q;
    if (shift <= 0) {
        const i128 lim = (i128)1 << 33;                      // beyond any 32-bit range: saturates below
        const i128 c = acc > lim ? lim : acc < -lim ? -lim : acc;
        const int l = -shift > 62 ? 62 : -shift;
        q = (i128)((u128)c << l);
    } else if (shift <= 16) {
        q = (acc + (i128)(r16 >> (16 - shift))) >> shift;
    } else {
        q = ((acc >> (shift - 16)) + (i128)r16) >> 16;
    }
    if (relu && q < 0) q = 0;
    const i128 qmax = ((i128)1 << (wl - 1)) - 1, qmin = -((i128)1 << (wl - 1));
    return (int)(q > qmax ? qmax : q < qmin ? qmin : q);
}

// number of bits of |v| (0 for 0)
__device__ __forceinline__ int bit_length_128(i128 v)
{
    const u128 m = v < 0 ? (u128)0 - (u128)v : (u128)v;
    const uint64_t hi = (uint64_t)(m >> 64), lo = (uint64_t)m;
    return hi ? 128 - __clzll((long long)hi) : (lo ? 64 - __clzll((long long)lo) : 0);
}

// nearest double (ties to even) of an unsigned 128-bit integer given as two words
__device__ __forceinline__ double u128_to_double(uint64_t lo, uint64_t hi)
{
    if (hi == 0) return (double)lo;                            // the conversion instruction rounds to nearest even
    const int sh = 64 - __clzll((long long)hi);                // 1..64: bits of the value above the low word
    // keep the top 64 bits and fold everything below into the lowest kept bit: 64 bits are at least 11 more than a
    // double holds, so the sticky bit decides ties exactly as the dropped bits would
    const uint64_t top = sh == 64 ? hi : ((hi << (64 - sh)) | (lo >> sh));
    const uint64_t rest = sh == 64 ? lo : (lo << (64 - sh));
    return ldexp((double)(top | (rest != 0)), sh);
}

// *acc (two words, low first) += v, exactly, whatever other threads add meanwhile: a wrap of the low word is seen by
// exactly the addition that causes it
__device__ __forceinline__ void atomic_add_u128(unsigned long long *acc, u128 v)
{
    const unsigned long long lo = (unsigned long long)v, hi = (unsigned long long)(v >> 64);
    unsigned long long carry = 0;
    if (lo) {
        const unsigned long long old = atomicAdd(acc, lo);
        carry = (old + lo) < old;
    }
    if (hi + carry) atomicAdd(acc + 1, hi + carry);
}

__device__ __forceinline__ u128 wave_sum_u128(u128 v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long lo = __shfl_xor((unsigned long long)v, off, 64);
        const unsigned long long hi = __shfl_xor((unsigned long long)(v >> 64), off, 64);
        v += ((u128)hi << 64) | lo;
    }
    return v;
}

}  // namespace adapt
