// PushUp (Sec. 3.3 "The PushUp Operation", "Dealing with Fixed-Points Limited Range",
// "Strategy, Resolution and Lookback") for gfx950.
//
// Device part: the gradient-diversity equation over a lookback window of gradient tensors held
// as fixed-point codes.  One pass over the window: every thread owns 16 consecutive elements,
// reads them from each tensor in turn (eight tensors' loads in flight), keeps the running
// element-wise sum of the aligned codes in registers and the per-tensor sums of squares in
// per-wavefront counters.  All sums are integers (exact, order-independent); a one-block
// follow-up kernel adds the block partials and forms the norms and the ratio in fp64.
//
// Host part: the scalar rules that turn the diversity into a new <WL,FL>, lookback,
// resolution and strategy.  They are plain functions and need no device.
#include <algorithm>
#include <cmath>

#include "common.hpp"
#include "context.hpp"
#include "grad_window.hpp"
#include "wide.hpp"

namespace adapt {

constexpr int kGdThreads = 256;
constexpr int kGdPerThread = 16;          // elements per thread
constexpr int kGdFinalThreads = 1024;

typedef unsigned gd_v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor((unsigned long long)v, off, 64);
    return v;
}

// 16 codes of tensor k starting at element e0.  The buffer descriptor covers the tensor rounded up
// to whole 16-byte units (the tensor is 16-byte aligned, so the last unit lies in a mapped page):
// units past it read as 0; the codes past n inside the last unit are cleared by the caller.
__device__ __forceinline__ void load16(const GradWindow &w, int k, uint32_t n, uint32_t e0, gd_v4u (&raw)[2])
{
    const uint32_t es = w.es[k];
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(w.g[k]), 0, (int)((n * es + 15u) & ~15u), 0x00020000);
    raw[0] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, e0 * es, 0, 0);
    raw[1] = es == 2 ? __builtin_amdgcn_raw_buffer_load_b128(rsrc, e0 * es + 16, 0, 0) : gd_v4u{0, 0, 0, 0};
}

__device__ __forceinline__ void unpack16(const gd_v4u (&raw)[2], int es, int (&c)[16])
{
    if (es == 1) {
#pragma unroll
        for (int j = 0; j < 16; ++j) c[j] = (int)(int8_t)(raw[0][j >> 2] >> (8 * (j & 3)));
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) c[j] = (int)(int16_t)(raw[j >> 3][(j >> 1) & 3] >> (16 * (j & 1)));
    }
}

// partial[col][block]: col k < count: sum of squares of tensor k; col count / count+1: sums of the
// low / high 32-bit halves of (aligned element sum)^2
// BYPTR: the window description lies in device memory (written by chain_prep_kernel) instead of the
// kernel arguments
// blk of nblk: this block's place among the blocks of the tensor (a chained step runs all layers in one launch)
__device__ __forceinline__ void gd_partial_body(const GradWindow &w, uint32_t n, uint64_t *partial, const uint32_t blk, const uint32_t nblk)
{
    __shared__ uint64_t wave_part[kGdThreads / kWave][kGdMaxTensors + 2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const uint32_t e0 = (blk * kGdThreads + threadIdx.x) * kGdPerThread;
    int S[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) S[j] = 0;
    constexpr int U = 8;                  // tensors whose loads are in flight together
    for (int k0 = 0; k0 < w.count; k0 += U) {
        gd_v4u raw[U][2];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (k0 + u < w.count) load16(w, k0 + u, n, e0, raw[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (k0 + u >= w.count) break;
            const int es = w.es[k0 + u], sh = w.shift[k0 + u];
            if (e0 + 16 > n) {                 // last unit of the tensor: clear the codes past n
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (e0 + j >= n) {
                        if (es == 1) raw[u][0][j >> 2] &= ~(0xffu << (8 * (j & 3)));
                        else raw[u][j >> 3][(j >> 1) & 3] &= ~(0xffffu << (16 * (j & 1)));
                    }
            }
            int c[16];
            unpack16(raw[u], es, c);
#pragma unroll
            for (int j = 0; j < 16; ++j) S[j] += (int)((unsigned)c[j] << sh);
            // sums of squares with the packed dot-product instructions: 4 (int8) or 2 (int16) codes each
            uint64_t sq;
            if (es == 1) {
                int d = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) d = __builtin_amdgcn_sdot4((int)raw[u][0][i], (int)raw[u][0][i], d, false);
                sq = wave_sum_u32((uint32_t)d);                    // <= 64 * 16 * 2^14
            } else {
                uint64_t t = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    typedef short gd_v2s __attribute__((ext_vector_type(2)));
                    const uint32_t x = raw[u][i >> 2][i & 3];
                    const gd_v2s v = {(short)(x & 0xffff), (short)(x >> 16)};
                    t += (uint32_t)__builtin_amdgcn_sdot2(v, v, 0, false);      // <= 2^31
                }
                sq = wave_sum_u64(t);
            }
            if (lane == 0) wave_part[wave][k0 + u] = sq;
        }
    }
    uint64_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const uint64_t q = (uint64_t)((long long)S[j] * (long long)S[j]);
        lo += q & 0xffffffffull;
        hi += q >> 32;
    }
    lo = wave_sum_u64(lo);
    hi = wave_sum_u64(hi);
    if (lane == 0) { wave_part[wave][w.count] = lo; wave_part[wave][w.count + 1] = hi; }
    __syncthreads();
    for (int col = threadIdx.x; col < w.count + 2; col += kGdThreads) {
        uint64_t v = 0;
#pragma unroll
        for (int i = 0; i < kGdThreads / kWave; ++i) v += wave_part[i][col];
        partial[(size_t)col * nblk + blk] = v;
    }
}

template <bool BYPTR>
__global__ void __launch_bounds__(kGdThreads)
gd_partial_kernel(const GradWindow wv, const GradWindow *__restrict__ wp, uint32_t n, uint64_t *partial)
{
    gd_partial_body(BYPTR ? *wp : wv, n, partial, blockIdx.x, gridDim.x);
}

// One block: column sums (one wavefront per column at a time), then the norms and the ratio.
__device__ __forceinline__ void gd_final_body(const GradWindow &w, const uint64_t *__restrict__ partial, int nblocks, uint64_t *sums_out,
                                              double *out)
{
    __shared__ uint64_t col_sum[kGdMaxTensors + 2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int col = wave; col < w.count + 2; col += kGdFinalThreads / kWave) {
        const uint64_t *p = partial + (size_t)col * nblocks;
        uint64_t v = 0;
        int b = lane;
        for (; b + 7 * kWave < nblocks; b += 8 * kWave) {
            uint64_t t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = p[b + u * kWave];
#pragma unroll
            for (int u = 0; u < 8; ++u) v += t[u];
        }
        for (; b < nblocks; b += kWave) v += p[b];
        v = wave_sum_u64(v);
        if (lane == 0) {
            col_sum[col] = v;
            if (sums_out) sums_out[col] = v;
        }
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    double num = 0.0;
    for (int k = 0; k < w.count; ++k) num += ldexp(sqrt((double)col_sum[k]), -(int)w.fl[k]);
    const double sq = (double)col_sum[w.count + 1] * 4294967296.0 + (double)col_sum[w.count];
    const double den = ldexp(sqrt(sq), -w.fl_max);
    const double ds = den > 0.0 ? num / den : (num > 0.0 ? (double)INFINITY : (double)NAN);
    out[0] = ds;
    out[1] = (ds > 0.0 && ds < (double)INFINITY) ? log(ds) : 1.0;
}

template <bool BYPTR>
__global__ void __launch_bounds__(kGdFinalThreads)
gd_final_kernel(const GradWindow wv, const GradWindow *__restrict__ wp, const uint64_t *__restrict__ partial, int nblocks,
                uint64_t *sums_out, double *out)
{
    gd_final_body(BYPTR ? *wp : wv, partial, nblocks, sums_out, out);
}

// ---- windows that hold int32 codes (word lengths 17..32) --------------------------------------------------------
// The aligned element sum is kept in 64 bits (its bound is below 2^48), every sum of squares in 128 bits.
// partial[col][block] as two words, low first: col k < count: sum of squares of tensor k; col count: sum of the
// squared aligned element sums.
__device__ __forceinline__ void load16_any(const void *g, int es, uint32_t n, uint32_t e0, int (&c)[16])
{
    if (e0 + 16 <= n) {
        if (es == 4) {
            const int4 *p = reinterpret_cast<const int4 *>(static_cast<const int32_t *>(g) + e0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int4 v = p[i];
                c[4 * i] = v.x; c[4 * i + 1] = v.y; c[4 * i + 2] = v.z; c[4 * i + 3] = v.w;
            }
        } else {
            gd_v4u raw[2];
            const gd_v4u *p = reinterpret_cast<const gd_v4u *>(static_cast<const char *>(g) + (size_t)e0 * es);
            raw[0] = p[0];
            raw[1] = es == 2 ? p[1] : gd_v4u{0, 0, 0, 0};
            unpack16(raw, es, c);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            int v = 0;
            if (e0 + j < n) v = es == 4 ? static_cast<const int32_t *>(g)[e0 + j] : es == 2 ? (int)static_cast<const int16_t *>(g)[e0 + j]
                                                                                          : (int)static_cast<const int8_t *>(g)[e0 + j];
            c[j] = v;
        }
    }
}

__device__ __forceinline__ void gd_partial_wide_body(const GradWindow &w, uint32_t n, uint64_t *partial, const uint32_t blk,
                                                     const uint32_t nblk)
{
    __shared__ unsigned long long wave_part[kGdThreads / kWave][kGdMaxTensors + 1][2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const uint32_t e0 = (blk * kGdThreads + threadIdx.x) * kGdPerThread;
    long long S[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) S[j] = 0;
    for (int k = 0; k < w.count; ++k) {
        int c[16];
        if (e0 < n) {
            load16_any(w.g[k], w.es[k], n, e0, c);
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) c[j] = 0;
        }
        const int sh = w.shift[k];
        u128 sq = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            S[j] += (long long)((unsigned long long)(long long)c[j] << sh);
            sq += (u128)(unsigned long long)((long long)c[j] * (long long)c[j]);
        }
        sq = wave_sum_u128(sq);
        if (lane == 0) { wave_part[wave][k][0] = (unsigned long long)sq; wave_part[wave][k][1] = (unsigned long long)(sq >> 64); }
    }
    u128 t = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) t += (u128)((i128)S[j] * (i128)S[j]);
    t = wave_sum_u128(t);
    if (lane == 0) { wave_part[wave][w.count][0] = (unsigned long long)t; wave_part[wave][w.count][1] = (unsigned long long)(t >> 64); }
    __syncthreads();
    for (int col = threadIdx.x; col < w.count + 1; col += kGdThreads) {
        u128 v = 0;
#pragma unroll
        for (int i = 0; i < kGdThreads / kWave; ++i) v += ((u128)wave_part[i][col][1] << 64) | wave_part[i][col][0];
        uint64_t *dst = partial + 2 * ((size_t)col * nblk + blk);
        dst[0] = (uint64_t)v;
        dst[1] = (uint64_t)(v >> 64);
    }
}

template <bool BYPTR>
__global__ void __launch_bounds__(kGdThreads)
gd_partial_wide_kernel(const GradWindow wv, const GradWindow *__restrict__ wp, uint32_t n, uint64_t *partial)
{
    gd_partial_wide_body(BYPTR ? *wp : wv, n, partial, blockIdx.x, gridDim.x);
}

__device__ __forceinline__ void gd_final_wide_body(const GradWindow &w, const uint64_t *__restrict__ partial, int nblocks,
                                                   uint64_t *sums_out, double *out)
{
    __shared__ unsigned long long col_sum[kGdMaxTensors + 1][2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int col = wave; col < w.count + 1; col += kGdFinalThreads / kWave) {
        const uint64_t *p = partial + 2 * (size_t)col * nblocks;
        u128 v = 0;
        for (int b = lane; b < nblocks; b += kWave) v += ((u128)p[2 * b + 1] << 64) | p[2 * b];
        v = wave_sum_u128(v);
        if (lane == 0) {
            col_sum[col][0] = (unsigned long long)v;
            col_sum[col][1] = (unsigned long long)(v >> 64);
            if (sums_out) { sums_out[2 * col] = (uint64_t)v; sums_out[2 * col + 1] = (uint64_t)(v >> 64); }
        }
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    double num = 0.0;
    for (int k = 0; k < w.count; ++k) num += ldexp(sqrt(u128_to_double(col_sum[k][0], col_sum[k][1])), -(int)w.fl[k]);
    const double den = ldexp(sqrt(u128_to_double(col_sum[w.count][0], col_sum[w.count][1])), -w.fl_max);
    const double ds = den > 0.0 ? num / den : (num > 0.0 ? (double)INFINITY : (double)NAN);
    out[0] = ds;
    out[1] = (ds > 0.0 && ds < (double)INFINITY) ? log(ds) : 1.0;
}

template <bool BYPTR>
__global__ void __launch_bounds__(kGdFinalThreads)
gd_final_wide_kernel(const GradWindow wv, const GradWindow *__restrict__ wp, const uint64_t *__restrict__ partial, int nblocks,
                     uint64_t *sums_out, double *out)
{
    gd_final_wide_body(BYPTR ? *wp : wv, partial, nblocks, sums_out, out);
}

size_t ws_need_gradient_diversity(uint64_t n, int count);

// All layers of a chained step in one launch per phase: the blocks of layer l are [first[l], first[l + 1]), its
// partial sums start part_off[l] words into the scratch.
struct ChainGeo {
    uint32_t first[kGdMaxLayers + 1];
    uint32_t n[kGdMaxLayers];
    uint64_t part_off[kGdMaxLayers];
    uint8_t wide[kGdMaxLayers];
    int nlayers;
};

__global__ void __launch_bounds__(kGdThreads)
gd_partial_chain_kernel(const ChainGeo geo, const GradWindow *__restrict__ win, uint64_t *partial)
{
    // the layer this block belongs to: every lane compares one table entry, the wavefront votes
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t first = lane < geo.nlayers ? geo.first[lane] : 0xffffffffu;
    const int l = __popcll(__ballot(blockIdx.x >= first)) - 1;
    const uint32_t blk = blockIdx.x - geo.first[l], nblk = geo.first[l + 1] - geo.first[l];
    if (geo.wide[l]) gd_partial_wide_body(win[l], geo.n[l], partial + geo.part_off[l], blk, nblk);
    else gd_partial_body(win[l], geo.n[l], partial + geo.part_off[l], blk, nblk);
}

__global__ void __launch_bounds__(kGdFinalThreads)
gd_final_chain_kernel(const ChainGeo geo, const GradWindow *__restrict__ win, const uint64_t *__restrict__ partial, ChainLayerOut *out)
{
    const int l = blockIdx.x;
    const int nblk = (int)(geo.first[l + 1] - geo.first[l]);
    if (geo.wide[l]) gd_final_wide_body(win[l], partial + geo.part_off[l], nblk, nullptr, &out[l].ds);
    else gd_final_body(win[l], partial + geo.part_off[l], nblk, nullptr, &out[l].ds);
}

// One thread per layer of a chained step: the exponent of this batch's gradient lies in device memory (the fitting
// pass of the backward pass wrote it), so the window can be laid out without the host reading it first.  The aligned
// element sum of the diversity kernel is a 32-bit integer (a 64-bit one with the bound 2^48 when the window holds codes
// above 16 bits): when the scales of the window lie too far apart for that, the oldest entries are left out until the
// rest fits (at least the newest entry stays).
__global__ void chain_prep_kernel(const ChainLayerIn *__restrict__ in, int nlayers, const long long *__restrict__ e_g, size_t e_stride,
                                  GradWindow *__restrict__ win, ChainLayerOut *__restrict__ out)
{
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= nlayers) return;
    const ChainLayerIn &c = in[l];
    const int count = c.count;
    const long long e_new = e_g[(size_t)l * e_stride];
    auto exp_of = [&](int k) { return k == count - 1 ? e_new : c.exp[k]; };
    bool wide = false;                              // codes above 16 bits: 64-bit element sums, bound 2^48
    for (int k = 0; k < count; ++k) wide = wide || c.wl[k] > 16;
    const int cap = wide ? 48 : 31;
    int first = 0;
    long long e_min = 0, e_max = 0;
    for (;; ++first) {
        e_min = e_max = exp_of(first);
        for (int k = first + 1; k < count; ++k) {
            const long long e = exp_of(k);
            e_min = e < e_min ? e : e_min;
            e_max = e > e_max ? e : e_max;
        }
        unsigned long long bound = 0;               // sum of 2^(wl - 1 + e_max - e_k), capped
        for (int k = first; k < count; ++k) {
            const long long b = (long long)c.wl[k] - 1 + e_max - exp_of(k);
            bound += b >= cap ? (1ull << cap) : (1ull << b);
        }
        if (bound < (1ull << cap) || first == count - 1) break;
    }
    GradWindow &w = win[l];
    const int used = count - first;
    for (int i = 0; i < used; ++i) {
        const int k = first + i;
        w.g[i] = c.g[k];
        w.es[i] = (uint8_t)(c.wl[k] <= 8 ? 1 : c.wl[k] <= 16 ? 2 : 4);
        w.shift[i] = (uint8_t)(e_max - exp_of(k));
        w.fl[i] = (int8_t)(exp_of(k) - e_min);
    }
    w.count = used;
    w.fl_max = (int)(e_max - e_min);
    out[l].exp_new = e_new;
    out[l].used = used;
}

int gradient_diversity_chain(adapt_ctx *ctx, const ChainLayerIn *in, int nlayers, const size_t *n, const long long *e_g, size_t e_stride,
                             GradWindow *win, ChainLayerOut *out)
{
    if (nlayers < 1) return ADAPT_EINVAL;
    if (nlayers > kGdMaxLayers) return ADAPT_EUNSUPPORTED;
    const size_t per_block = (size_t)kGdThreads * kGdPerThread;
    ChainGeo geo = {};
    geo.nlayers = nlayers;
    size_t words = 0;
    uint64_t blocks = 0;
    for (int l = 0; l < nlayers; ++l) {
        if (in[l].count < 1 || in[l].count > kGdMaxTensors || n[l] > ((size_t)1 << 30)) return ADAPT_EUNSUPPORTED;
        bool wide = false;
        for (int k = 0; k < in[l].count; ++k) wide = wide || in[l].wl[k] > 16;
        const uint64_t grid = std::max<size_t>(1, (n[l] + per_block - 1) / per_block);
        geo.first[l] = (uint32_t)blocks;
        geo.n[l] = (uint32_t)n[l];
        geo.part_off[l] = words;
        geo.wide[l] = wide;
        blocks += grid;
        words += ws_need_gradient_diversity(n[l], in[l].count) / sizeof(uint64_t);
    }
    geo.first[nlayers] = (uint32_t)blocks;
    if (blocks >= ((uint64_t)1 << 31)) return ADAPT_EUNSUPPORTED;
    if (words * sizeof(uint64_t) > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    uint64_t *partial = reinterpret_cast<uint64_t *>(scratch(ctx));
    hipLaunchKernelGGL(chain_prep_kernel, dim3(1), dim3(64), 0, ctx->stream, in, nlayers, e_g, e_stride, win, out);
    hipLaunchKernelGGL(gd_partial_chain_kernel, dim3((unsigned)blocks), dim3(kGdThreads), 0, ctx->stream, geo, win, partial);
    hipLaunchKernelGGL(gd_final_chain_kernel, dim3(nlayers), dim3(kGdFinalThreads), 0, ctx->stream, geo, win, partial, out);
    return hip_status(ctx, hipGetLastError());
}

size_t ws_need_gradient_diversity(uint64_t n, int count)
{
    const size_t per_block = (size_t)kGdThreads * kGdPerThread;
    // (count + 2) words per block, or (count + 1) pairs of words for windows with int32 codes
    return std::max<size_t>(1, (n + per_block - 1) / per_block) * (size_t)(count + 1) * 2 * sizeof(uint64_t);
}

}  // namespace adapt

using namespace adapt;

extern "C" int adapt_gradient_diversity(adapt_ctx *ctx, const adapt_grad_item *items, int count, size_t n,
                                        uint64_t *sums, double *out)
{
    if (!ctx || !items || !out || count < 1) return ADAPT_EINVAL;
    if (count > kGdMaxTensors) return ADAPT_EUNSUPPORTED;
    if (((uintptr_t)out & 7) || (sums && ((uintptr_t)sums & 7))) return ADAPT_EINVAL;
    if (n > ((size_t)1 << 30)) return ADAPT_EUNSUPPORTED;      // 32-bit byte offsets, with room for the last block's overhang
    GradWindow w;
    w.count = count;
    w.fl_max = 0;
    int wl_max = 0;
    for (int k = 0; k < count; ++k) {
        const adapt_fmt f = adapt_fmt{items[k].wl, items[k].fl};
        if (!fmt_ok_wide(f)) return ADAPT_EINVAL;
        if (n > 0 && (!items[k].g || !aligned16(items[k].g))) return ADAPT_EINVAL;
        w.fl_max = std::max(w.fl_max, f.fl);
        wl_max = std::max(wl_max, f.wl);
    }
    // the aligned element sum is kept in int32: count * 2^(wl-1) * 2^(fl_max - fl) must stay below 2^31
    double bound = 0.0;
    for (int k = 0; k < count; ++k) {
        w.g[k] = items[k].g;
        w.es[k] = (uint8_t)(items[k].wl <= 8 ? 1 : items[k].wl <= 16 ? 2 : 4);
        w.shift[k] = (uint8_t)(w.fl_max - items[k].fl);
        w.fl[k] = (int8_t)items[k].fl;
        bound += std::ldexp(1.0, items[k].wl - 1 + w.fl_max - items[k].fl);
    }
    const size_t per_block = (size_t)kGdThreads * kGdPerThread;
    const int grid = (int)std::max<size_t>(1, (n + per_block - 1) / per_block);
    if (wl_max > 16) {           // int32 codes in the window: 64-bit element sums (bound 2^48), 128-bit sums of squares
        if (bound >= 281474976710656.0) return ADAPT_EUNSUPPORTED;
        if ((size_t)grid * (count + 1) * 2 * sizeof(uint64_t) > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
        uint64_t *part = reinterpret_cast<uint64_t *>(scratch(ctx));
        hipLaunchKernelGGL(gd_partial_wide_kernel<false>, dim3(grid), dim3(kGdThreads), 0, ctx->stream, w, nullptr, (uint32_t)n, part);
        hipLaunchKernelGGL(gd_final_wide_kernel<false>, dim3(1), dim3(kGdFinalThreads), 0, ctx->stream, w, nullptr, part, grid, sums, out);
        return hip_status(ctx, hipGetLastError());
    }
    if (bound >= 2147483648.0) return ADAPT_EUNSUPPORTED;
    if ((size_t)grid * (count + 2) * sizeof(uint64_t) > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    uint64_t *partial = reinterpret_cast<uint64_t *>(scratch(ctx));
    hipLaunchKernelGGL(gd_partial_kernel<false>, dim3(grid), dim3(kGdThreads), 0, ctx->stream, w, nullptr, (uint32_t)n, partial);
    hipLaunchKernelGGL(gd_final_kernel<false>, dim3(1), dim3(kGdFinalThreads), 0, ctx->stream, w, nullptr, partial, grid, sums, out);
    return hip_status(ctx, hipGetLastError());
}

// ---- host-side scalar rules ------------------------------------------------------------------

static bool usable(double ds) { return ds > 0.0 && ds < (double)INFINITY; }

extern "C" int adapt_pushup_suggest(double ds, int wl_min, int fl_min, int strategy, int buff, int wl_cap,
                                    adapt_pushup_result *res)
{
    if (!res || wl_cap < 2 || wl_cap > 32 || buff < 0 || buff > wl_cap || wl_min < 1 || fl_min < 0) return ADAPT_EINVAL;
    if (strategy != ADAPT_ST_MIN && strategy != ADAPT_ST_MEAN && strategy != ADAPT_ST_MAX) return ADAPT_EINVAL;
    const double L = usable(ds) ? std::log(ds) : 1.0;
    int s1 = 1, s2 = 1, s = 1;
    if (L > 0.0) {
        s1 = L == 1.0 ? wl_cap : (int)std::min<double>(std::max(std::ceil(1.0 / (L - 1.0)), 1.0), (double)wl_cap);
        const double s2f = std::max(std::min(32.0 * L * L - 1.0, 32.0) - (double)fl_min, 1.0);
        s2 = (int)std::min<double>(std::ceil(s2f), (double)wl_cap);
        if (strategy == ADAPT_ST_MIN) s = std::min(s1, s2);
        else if (strategy == ADAPT_ST_MEAN) s = (int)std::ceil(0.5 * (s1 + s2));
        else s = std::max(s1, s2);
    }
    int fl = std::min(fl_min + s, wl_cap);
    int wl = std::min(std::max(wl_min, fl_min) + 1, wl_cap);
    fl = std::min(fl, wl_cap - buff);
    wl = std::max(std::min(fl + buff, wl_cap), wl);
    res->wl = wl; res->fl = fl; res->s1 = s1; res->s2 = s2; res->s = s;
    return ADAPT_OK;
}

extern "C" int adapt_strategy_next(int strategy, double loss_avg, double loss_now)
{
    if (std::fabs(loss_avg) > std::fabs(loss_now)) return ADAPT_ST_MIN;
    return strategy == ADAPT_ST_MIN ? ADAPT_ST_MEAN : ADAPT_ST_MAX;
}

extern "C" int adapt_lookback_next(int lb, double ds, int lb_lwr, int lb_upr, double gamma)
{
    double lb_new = (double)lb_upr;
    if (usable(ds)) lb_new = std::min(std::max(std::ceil((double)lb_upr / ds), (double)lb_lwr), (double)lb_upr);
    return (int)std::ceil(lb_new * gamma + (1.0 - gamma) * (double)lb);
}

extern "C" int adapt_resolution_next(int r, int lb, int lb_lwr, int lb_upr, int r_lwr, int r_upr)
{
    if (lb == lb_upr) return std::min(std::max(r + 1, r_lwr), r_upr);
    if (lb == lb_lwr) return std::min(std::max(r - 1, r_lwr), r_upr);
    return r;
}
