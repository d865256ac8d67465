// Shared device / host helpers of the gfx950 fixed-point library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adapt_fxp.h"

namespace adapt {

constexpr int kWave = 64;

struct adapt_ctx_impl;

// ---------------------------------------------------------------------------------------------
// Philox-4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1).  One call yields the
// 16 rounding bits of 8 consecutive elements.  The key schedule depends only on the seed, so
// the compiler keeps it in scalar registers.
// ---------------------------------------------------------------------------------------------
struct u32x4 { uint32_t x, y, z, w; };

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)M0 * c0;
        const uint64_t p1 = (uint64_t)M1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += W0;
        k1 += W1;
    }
    return {c0, c1, c2, c3};
}

// Rounding bits of the 8 elements 8*j .. 8*j+7 of a tensor: lane l is (w[l/2] >> 16*(l%2)) & 0xffff.
__device__ __forceinline__ u32x4 rounding_block(uint64_t seed, uint64_t stream, uint64_t j)
{
    return philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), (uint32_t)stream, (uint32_t)(stream >> 32),
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

__device__ __forceinline__ uint32_t lane16(const u32x4 &b, int lane)
{
    const uint32_t w = (lane >> 1) == 0 ? b.x : (lane >> 1) == 1 ? b.y : (lane >> 1) == 2 ? b.z : b.w;
    return (lane & 1) ? (w >> 16) : (w & 0xffffu);
}

// 16 rounding bits of one element (used where elements are not handled 8 at a time)
__device__ __forceinline__ uint32_t rounding_bits_of(uint64_t seed, uint64_t stream, uint64_t i, int mode)
{
    if (mode != ADAPT_SR) return 0x8000u;
    return lane16(rounding_block(seed, stream, i >> 3), (int)(i & 7));
}

// ---------------------------------------------------------------------------------------------
// fp32 -> fixed-point code (Sec. 3.2 SR rule with 16 guard bits, two's-complement saturation)
// ---------------------------------------------------------------------------------------------
struct QuantParams {
    float scale;     // 2^fl
    float qminf, qmaxf;
    int qmax;
};

__host__ __device__ inline QuantParams make_quant_params(int wl, int fl)
{
    QuantParams p;
    p.scale = (float)(1ull << fl);
    p.qmaxf = (float)((1 << (wl - 1)) - 1);
    p.qminf = -(float)(1 << (wl - 1));
    p.qmax = (1 << (wl - 1)) - 1;
    return p;
}

// returns the code; sat is set to 1 when x*2^fl lies outside the representable range
__device__ __forceinline__ int quantize_one(float x, uint32_t r16, const QuantParams &p, int &sat)
{
    const float y = x * p.scale;                       // exact (power of two), may become +-inf
    sat = (y < p.qminf) | (y > p.qmaxf);               // false for NaN
    const float yc = fminf(fmaxf(y, p.qminf), p.qmaxf);
    const int t = (int)floorf(yc * 65536.0f);          // exact, |t| <= 2^31 - 2^16 ... -2^31
    int q = (t + (int)r16) >> 16;
    q = min(q, p.qmax);
    return (x != x) ? 0 : q;
}

// ---------------------------------------------------------------------------------------------
// exact accumulator -> code of the output format: right shift with the SR rule on the dropped bits
// (shift <= 0: left shift), optional ReLU, saturation to wl bits
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int requantize_one(long long acc, int shift, int wl, int relu, uint32_t r16)
{
    long long q;
    if (shift <= 0) {
        const long long lim = 1ll << 20;               // beyond any 16-bit range: saturates below
        const long long c = acc > lim ? lim : acc < -lim ? -lim : acc;
        q = (-shift >= 40) ? (c > 0 ? (1ll << 60) : c < 0 ? -(1ll << 60) : 0) : (long long)((unsigned long long)c << -shift);
    } else if (shift <= 16) {
        q = (acc + (long long)(r16 >> (16 - shift))) >> shift;
    } else {
        q = ((acc >> (shift - 16)) + (long long)r16) >> 16;
    }
    if (relu && q < 0) q = 0;
    const long long qmax = (1ll << (wl - 1)) - 1, qmin = -(1ll << (wl - 1));
    return (int)(q > qmax ? qmax : q < qmin ? qmin : q);
}

// ---------------------------------------------------------------------------------------------
// eight consecutive codes (group index grp) of an int8 / int16 tensor, 16-byte aligned base
// ---------------------------------------------------------------------------------------------
template <typename GT>
__device__ __forceinline__ void load_codes8(const GT *g, uint64_t grp, int (&c)[8]);
template <>
__device__ __forceinline__ void load_codes8<int8_t>(const int8_t *g, uint64_t grp, int (&c)[8])
{
    const uint2 v = reinterpret_cast<const uint2 *>(g)[grp];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = (int)(int8_t)((j < 4 ? v.x : v.y) >> (8 * (j & 3)));
}
template <>
__device__ __forceinline__ void load_codes8<int16_t>(const int16_t *g, uint64_t grp, int (&c)[8])
{
    const uint4 v = reinterpret_cast<const uint4 *>(g)[grp];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = (int)(int16_t)(w[j >> 1] >> (16 * (j & 1)));
}

template <>
__device__ __forceinline__ void load_codes8<int32_t>(const int32_t *g, uint64_t grp, int (&c)[8])
{
    const int4 a = reinterpret_cast<const int4 *>(g)[2 * grp], b = reinterpret_cast<const int4 *>(g)[2 * grp + 1];
    c[0] = a.x; c[1] = a.y; c[2] = a.z; c[3] = a.w; c[4] = b.x; c[5] = b.y; c[6] = b.z; c[7] = b.w;
}

template <typename OutT>
__device__ __forceinline__ void store_codes8(OutT *q, uint64_t grp, const int (&v)[8]);
template <>
__device__ __forceinline__ void store_codes8<int8_t>(int8_t *q, uint64_t grp, const int (&v)[8])
{
    uint2 o;
    o.x = (uint32_t)(v[0] & 0xff) | ((uint32_t)(v[1] & 0xff) << 8) | ((uint32_t)(v[2] & 0xff) << 16) | ((uint32_t)(v[3] & 0xff) << 24);
    o.y = (uint32_t)(v[4] & 0xff) | ((uint32_t)(v[5] & 0xff) << 8) | ((uint32_t)(v[6] & 0xff) << 16) | ((uint32_t)(v[7] & 0xff) << 24);
    reinterpret_cast<uint2 *>(q)[grp] = o;
}
template <>
__device__ __forceinline__ void store_codes8<int16_t>(int16_t *q, uint64_t grp, const int (&v)[8])
{
    uint4 o;
    o.x = (uint32_t)(v[0] & 0xffff) | ((uint32_t)v[1] << 16);
    o.y = (uint32_t)(v[2] & 0xffff) | ((uint32_t)v[3] << 16);
    o.z = (uint32_t)(v[4] & 0xffff) | ((uint32_t)v[5] << 16);
    o.w = (uint32_t)(v[6] & 0xffff) | ((uint32_t)v[7] << 16);
    reinterpret_cast<uint4 *>(q)[grp] = o;
}

template <>
__device__ __forceinline__ void store_codes8<int32_t>(int32_t *q, uint64_t grp, const int (&v)[8])
{
    reinterpret_cast<int4 *>(q)[2 * grp] = make_int4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<int4 *>(q)[2 * grp + 1] = make_int4(v[4], v[5], v[6], v[7]);
}

// Word lengths 17..32 (Sec. 3.3 bounds precision at 32 bits): int32 codes.  The scaled value with its 16 guard bits
// needs up to 48 bits, so the rule of quantize_one is evaluated in fp64 and 64-bit integers (all steps exact).
__device__ __forceinline__ int quantize_one_wide(float x, uint32_t r16, int wl, int fl, int &sat)
{
    const double y = ldexp((double)x, fl);
    const double qmin = -ldexp(1.0, wl - 1), qmax = ldexp(1.0, wl - 1) - 1.0;
    sat = (y < qmin) | (y > qmax);                         // false for NaN
    const double yc = fmin(fmax(y, qmin), qmax);
    const long long t = (long long)floor(yc * 65536.0);
    long long q = (t + (long long)r16) >> 16;
    q = q > (long long)qmax ? (long long)qmax : q;
    return (x != x) ? 0 : (int)q;
}

// ---------------------------------------------------------------------------------------------
// wavefront reductions (64 lanes)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_min_f32(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_max_f32(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

}  // namespace adapt
