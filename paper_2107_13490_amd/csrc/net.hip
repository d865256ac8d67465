// One chained fixed-point training step of a feed-forward network (Alg. 1 for one batch:
// ForwardPass on the quantized layers, the backward pass, the update of the master weights and the
// per-layer Quantize), and the element-wise integer operations it needs between the contractions:
// 2x2 max-pooling of codes, the routing of a gradient back through pooling and ReLU, the conversion
// of exact gradient accumulators to WL-bit codes with the smallest shift that fits, and the
// residual addition of two fixed-point tensors.
//
// The paper gives the training loop; how a fixed-point backward pass keeps gradients in range is
// left open.  Back-propagation is linear in the incoming gradient and the update divides each
// layer's gradient by its 2-norm (Sec. 3.3 "Dealing with Fixed-Points Limited Range"), so a gradient
// tensor may carry any power-of-two factor: each exact accumulator tensor is shifted right just far
// enough for its largest magnitude to fit WL-1 bits, with the SR rule of Sec. 3.2 on the dropped
// bits.
//
// All four element-wise kernels are bound by HBM traffic (one read of every input, one write of
// every output, 16-byte accesses); the chain itself is host code that enqueues this library's own
// entry points on the context's stream.
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "common.hpp"
#include "context.hpp"
#include "fit.hpp"
#include "grad_window.hpp"
#include "update_batch.hpp"
#include "wide.hpp"

namespace adapt {

constexpr int kEwThreads = 256;

template <typename T, int V>
struct alignas(sizeof(T) * V) CodeVec {
    T v[V];
};

// pooled geometry: rows = n * (h/2), wo = w/2, cv = vectors per pixel; items = rows * wo * cv
struct PoolGeo {
    uint32_t wo, cv, items;
};

// a[n,i,j,c] = max over the 2x2 window of y[n,2i..2i+1,2j..2j+1,c]; codes compare like values
template <typename T, int V>
__global__ void __launch_bounds__(kEwThreads) maxpool2_kernel(const T *__restrict__ y, T *__restrict__ a, const PoolGeo g)
{
    typedef CodeVec<T, V> Vec;
    const Vec *yv = reinterpret_cast<const Vec *>(y);
    Vec *av = reinterpret_cast<Vec *>(a);
    const uint32_t stride = gridDim.x * kEwThreads;
    for (uint32_t i = blockIdx.x * kEwThreads + threadIdx.x; i < g.items; i += stride) {
        const uint32_t pix = i / g.cv, cv = i - pix * g.cv;
        const uint32_t row = pix / g.wo, wo = pix - row * g.wo;      // row = n*(h/2) + i: input row 2*row
        const uint64_t down = 2ull * g.wo * g.cv;
        const uint64_t p00 = (2ull * row * (2ull * g.wo) + 2ull * wo) * g.cv + cv;
        const Vec v0 = yv[p00], v1 = yv[p00 + g.cv], v2 = yv[p00 + down], v3 = yv[p00 + down + g.cv];
        Vec o;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const T m0 = v0.v[e] > v1.v[e] ? v0.v[e] : v1.v[e], m1 = v2.v[e] > v3.v[e] ? v2.v[e] : v3.v[e];
            o.v[e] = m0 > m1 ? m0 : m1;
        }
        av[i] = o;
    }
}

// POOL: dy = da at the first maximum (scan order) of each window of the stored output y, zero
// elsewhere; with relu also zero where that maximum is not positive.  !POOL: dy = da where y > 0.
template <typename T, int V, bool POOL>
__global__ void __launch_bounds__(kEwThreads)
relu_pool_bwd_kernel(const T *__restrict__ da, const T *__restrict__ y, T *__restrict__ dy, const PoolGeo g, const int relu)
{
    typedef CodeVec<T, V> Vec;
    const Vec *yv = reinterpret_cast<const Vec *>(y);
    const Vec *dv = reinterpret_cast<const Vec *>(da);
    Vec *ov = reinterpret_cast<Vec *>(dy);
    const uint32_t stride = gridDim.x * kEwThreads;
    for (uint32_t i = blockIdx.x * kEwThreads + threadIdx.x; i < g.items; i += stride) {
        if (POOL) {
            const uint32_t pix = i / g.cv, cv = i - pix * g.cv;
            const uint32_t row = pix / g.wo, wo = pix - row * g.wo;
            const uint64_t down = 2ull * g.wo * g.cv;
            const uint64_t p00 = (2ull * row * (2ull * g.wo) + 2ull * wo) * g.cv + cv;
            const Vec v0 = yv[p00], v1 = yv[p00 + g.cv], v2 = yv[p00 + down], v3 = yv[p00 + down + g.cv], d = dv[i];
            Vec o0, o1, o2, o3;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const T m0 = v0.v[e] > v1.v[e] ? v0.v[e] : v1.v[e], m1 = v2.v[e] > v3.v[e] ? v2.v[e] : v3.v[e];
                const T m = m0 > m1 ? m0 : m1;
                const int first = v0.v[e] == m ? 0 : v1.v[e] == m ? 1 : v2.v[e] == m ? 2 : 3;
                const T val = (!relu || m > 0) ? d.v[e] : (T)0;
                o0.v[e] = first == 0 ? val : (T)0;
                o1.v[e] = first == 1 ? val : (T)0;
                o2.v[e] = first == 2 ? val : (T)0;
                o3.v[e] = first == 3 ? val : (T)0;
            }
            ov[p00] = o0; ov[p00 + g.cv] = o1; ov[p00 + down] = o2; ov[p00 + down + g.cv] = o3;
        } else {
            const Vec v = yv[i], d = dv[i];
            Vec o;
#pragma unroll
            for (int e = 0; e < V; ++e) o.v[e] = (!relu || v.v[e] > 0) ? d.v[e] : (T)0;
            ov[i] = o;
        }
    }
}

template <typename AccT>
__device__ __forceinline__ void load_acc8(const AccT *acc, uint64_t grp, long long (&v)[8]);
template <>
__device__ __forceinline__ void load_acc8<int32_t>(const int32_t *acc, uint64_t grp, long long (&v)[8])
{
    const int4 a = reinterpret_cast<const int4 *>(acc)[2 * grp], b = reinterpret_cast<const int4 *>(acc)[2 * grp + 1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
template <>
__device__ __forceinline__ void load_acc8<int64_t>(const int64_t *acc, uint64_t grp, long long (&v)[8])
{
    const longlong2 *p = reinterpret_cast<const longlong2 *>(acc) + 4 * grp;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const longlong2 t = p[i];
        v[2 * i] = t.x; v[2 * i + 1] = t.y;
    }
}

// largest magnitude of acc[0..n): one partial per block; block 0 also clears the sum of squares that
// the pass after this one accumulates
template <typename AccT>
__global__ void __launch_bounds__(kEwThreads)
absmax_kernel(const AccT *__restrict__ acc, const uint64_t n, uint64_t *__restrict__ part, unsigned long long *sumsq)
{
    uint64_t m = 0;
    const uint64_t groups = n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kEwThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kEwThreads;
    for (uint64_t grp = first; grp < groups; grp += stride) {
        long long v[8];
        load_acc8<AccT>(acc, grp, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint64_t a = magnitude(v[e]);
            m = a > m ? a : m;
        }
    }
    if ((n & 7) && first == 0)
        for (uint64_t i = groups << 3; i < n; ++i) {
            const uint64_t a = magnitude((long long)acc[i]);
            m = a > m ? a : m;
        }
    __shared__ uint64_t sm[kEwThreads / kWave];
    m = wave_max_u64(m);
    if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 1; i < kEwThreads / kWave; ++i) m = sm[i] > m ? sm[i] : m;
        part[blockIdx.x] = m;
        if (blockIdx.x == 0 && sumsq) *sumsq = 0;
    }
}

// codes = requantize(acc, shift) with shift = max(0, bit_length(max |acc|) - (wl-1)); every block
// derives the shift from the partial maxima itself
template <typename AccT, typename OutT>
__global__ void __launch_bounds__(kEwThreads) requant_fit_kernel(const FitArgs a)
{
    __shared__ uint64_t sm[kEwThreads / kWave];
    uint64_t m = 0;
    for (int i = threadIdx.x; i < a.nparts; i += kEwThreads) m = a.part[i] > m ? a.part[i] : m;
    m = wave_max_u64(m);
    if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = m;
    __syncthreads();
    m = sm[0];
#pragma unroll
    for (int i = 1; i < kEwThreads / kWave; ++i) m = sm[i] > m ? sm[i] : m;
    const int bits = m ? 64 - __clzll((long long)m) : 0;
    const int shift = max(0, bits - (a.wl - 1));
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (a.shift_out) *a.shift_out = shift;
        if (a.e_out) *a.e_out = (a.e_in ? *a.e_in : 0) + a.e_add - shift;
    }
    __syncthreads();                                    // sm is reused below
    const int qhi = (1 << (a.wl - 1)) - 1, qlo = -(1 << (a.wl - 1));

    const AccT *acc = static_cast<const AccT *>(a.acc);
    OutT *q = static_cast<OutT *>(a.q);
    uint64_t ss = 0;
    const uint64_t groups = a.n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kEwThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kEwThreads;
    for (uint64_t grp = first; grp < groups; grp += stride) {
        long long v[8];
        load_acc8<AccT>(acc, grp, v);
        uint32_t r[8];
        if (a.mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(a.seed, a.stream, grp);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
        int code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            code[e] = fit_one(v[e], shift, r[e], qlo, qhi);
            ss += (uint32_t)(code[e] * code[e]);
        }
        store_codes8<OutT>(q, grp, code);
    }
    if ((a.n & 7) && first == 0)
        for (uint64_t i = groups << 3; i < a.n; ++i) {
            const int c = fit_one((long long)acc[i], shift, rounding_bits_of(a.seed, a.stream, i, a.mode), qlo, qhi);
            q[i] = (OutT)c;
            ss += (uint32_t)(c * c);
        }
    if (a.sumsq) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor((unsigned long long)ss, off, 64);
        if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = ss;
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int i = 1; i < kEwThreads / kWave; ++i) ss += sm[i];
            if (ss) atomicAdd(a.sumsq, (unsigned long long)ss);
        }
    }
}

struct AddArgs {
    const void *a, *b;
    void *out;
    uint64_t n;
    int sa, sb, shift, wl, relu, mode;
    uint64_t seed, stream;
};

// out = requantize(a * 2^sa + b * 2^sb, shift): the exact sum on the finer of the two grids
template <typename TA, typename TB, typename TO>
__global__ void __launch_bounds__(kEwThreads) residual_add_kernel(const AddArgs p)
{
    const TA *a = static_cast<const TA *>(p.a);
    const TB *b = static_cast<const TB *>(p.b);
    TO *out = static_cast<TO *>(p.out);
    const uint64_t groups = p.n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kEwThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kEwThreads;
    for (uint64_t grp = first; grp < groups; grp += stride) {
        int ca[8], cb[8], code[8];
        load_codes8<TA>(a, grp, ca);
        load_codes8<TB>(b, grp, cb);
        uint32_t r[8];
        if (p.mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(p.seed, p.stream, grp);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const long long s = (long long)ca[e] * (1ll << p.sa) + (long long)cb[e] * (1ll << p.sb);
            code[e] = requantize_one(s, p.shift, p.wl, p.relu, r[e]);
        }
        store_codes8<TO>(out, grp, code);
    }
    if ((p.n & 7) && first == 0)
        for (uint64_t i = groups << 3; i < p.n; ++i) {
            const long long s = (long long)a[i] * (1ll << p.sa) + (long long)b[i] * (1ll << p.sb);
            out[i] = (TO)requantize_one(s, p.shift, p.wl, p.relu, rounding_bits_of(p.seed, p.stream, i, p.mode));
        }
}

// the same sum for tensors above 16 bits (int32 codes): 128-bit arithmetic, storage widths chosen at run time
__global__ void __launch_bounds__(kEwThreads) residual_add_wide_kernel(const AddArgs p, int es_a, int es_b, int es_o)
{
    auto code_at = [](const void *q, int es, uint64_t i) -> long long {
        return es == 1 ? (long long)static_cast<const int8_t *>(q)[i] : es == 2 ? (long long)static_cast<const int16_t *>(q)[i]
                                                                              : (long long)static_cast<const int32_t *>(q)[i];
    };
    for (uint64_t i = (uint64_t)blockIdx.x * kEwThreads + threadIdx.x; i < p.n; i += (uint64_t)gridDim.x * kEwThreads) {
        const i128 s = (i128)((u128)(i128)code_at(p.a, es_a, i) << p.sa) + (i128)((u128)(i128)code_at(p.b, es_b, i) << p.sb);
        const int c = requantize_wide_one(s, p.shift, p.wl, p.relu, rounding_bits_of(p.seed, p.stream, i, p.mode));
        if (es_o == 1) static_cast<int8_t *>(p.out)[i] = (int8_t)c;
        else if (es_o == 2) static_cast<int16_t *>(p.out)[i] = (int16_t)c;
        else static_cast<int32_t *>(p.out)[i] = c;
    }
}

static int ew_grid(const adapt_ctx *ctx, uint64_t items)
{
    const uint64_t blocks = (items + kEwThreads - 1) / kEwThreads;
    return (int)std::min<uint64_t>(std::max<uint64_t>(blocks, 1), (uint64_t)ctx->num_cu * 8);
}

static bool rng_ok(adapt_rng r) { return r.mode == ADAPT_SR || r.mode == ADAPT_RN_HALF_UP; }

// geometry of a pooled / unpooled element-wise pass over an n x h x w x c tensor of es-byte codes
static int pool_geo(int es, int n, int h, int w, int c, bool pool, PoolGeo &g, int &vec)
{
    if (n < 0 || h < 1 || w < 1 || c < 1) return ADAPT_EINVAL;
    if (pool && ((h | w) & 1)) return ADAPT_EINVAL;
    const int full = 16 / es;
    vec = (c % full == 0) ? full : 1;
    // without pooling the tensor is a flat array: vectors may straddle pixels
    if (!pool && ((uint64_t)n * h * w * c) % full == 0) vec = full;
    const uint64_t elems = (uint64_t)n * (pool ? h / 2 : h) * (pool ? w / 2 : w) * c;
    const uint64_t items = elems / vec;
    if ((uint64_t)n * h * w * c * es >= ((uint64_t)1 << 32) || items >= ((uint64_t)1 << 31)) return ADAPT_EUNSUPPORTED;
    g.wo = (uint32_t)(pool ? w / 2 : w);
    g.cv = (uint32_t)(pool ? c / vec : 1);
    g.items = (uint32_t)items;
    return ADAPT_OK;
}

size_t ws_need_requantize_fit(int num_cu, uint64_t n)
{
    const uint64_t groups = (n + 7) >> 3;
    return (size_t)std::min<uint64_t>(std::max<uint64_t>((groups + kEwThreads - 1) / kEwThreads, 1), (uint64_t)num_cu * 4) * 8;
}

}  // namespace adapt

using namespace adapt;

extern "C" int adapt_maxpool2_fwd(adapt_ctx *ctx, const void *y, adapt_fmt f, int n, int h, int w, int c, void *a)
{
    if (!ctx || !fmt_ok_wide(f)) return ADAPT_EINVAL;
    const int es = storage_bytes(f);
    PoolGeo g;
    int vec;
    if (int s = pool_geo(es, n, h, w, c, true, g, vec)) return s;
    if (g.items == 0) return ADAPT_OK;
    if (!y || !a || !aligned16(y) || !aligned16(a)) return ADAPT_EINVAL;
    const dim3 grid(ew_grid(ctx, g.items)), block(kEwThreads);
    if (es == 4 && vec == 4) hipLaunchKernelGGL((maxpool2_kernel<int32_t, 4>), grid, block, 0, ctx->stream, (const int32_t *)y, (int32_t *)a, g);
    else if (es == 4) hipLaunchKernelGGL((maxpool2_kernel<int32_t, 1>), grid, block, 0, ctx->stream, (const int32_t *)y, (int32_t *)a, g);
    else if (es == 1 && vec == 16) hipLaunchKernelGGL((maxpool2_kernel<int8_t, 16>), grid, block, 0, ctx->stream, (const int8_t *)y, (int8_t *)a, g);
    else if (es == 1) hipLaunchKernelGGL((maxpool2_kernel<int8_t, 1>), grid, block, 0, ctx->stream, (const int8_t *)y, (int8_t *)a, g);
    else if (vec == 8) hipLaunchKernelGGL((maxpool2_kernel<int16_t, 8>), grid, block, 0, ctx->stream, (const int16_t *)y, (int16_t *)a, g);
    else hipLaunchKernelGGL((maxpool2_kernel<int16_t, 1>), grid, block, 0, ctx->stream, (const int16_t *)y, (int16_t *)a, g);
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_relu_pool_bwd(adapt_ctx *ctx, const void *da, const void *y, adapt_fmt f, int n, int h, int w, int c,
                                   int relu, int pool, void *dy)
{
    if (!ctx || !fmt_ok_wide(f)) return ADAPT_EINVAL;
    const int es = storage_bytes(f);
    PoolGeo g;
    int vec;
    if (int s = pool_geo(es, n, h, w, c, pool != 0, g, vec)) return s;
    if (g.items == 0) return ADAPT_OK;
    if (!da || !y || !dy || !aligned16(da) || !aligned16(y) || !aligned16(dy)) return ADAPT_EINVAL;
    const dim3 grid(ew_grid(ctx, g.items)), block(kEwThreads);
#define ADAPT_BWD(T, V, P) hipLaunchKernelGGL((relu_pool_bwd_kernel<T, V, P>), grid, block, 0, ctx->stream, (const T *)da, (const T *)y, (T *)dy, g, relu)
    if (pool) {
        if (es == 4 && vec == 4) ADAPT_BWD(int32_t, 4, true);
        else if (es == 4) ADAPT_BWD(int32_t, 1, true);
        else if (es == 1 && vec == 16) ADAPT_BWD(int8_t, 16, true);
        else if (es == 1) ADAPT_BWD(int8_t, 1, true);
        else if (vec == 8) ADAPT_BWD(int16_t, 8, true);
        else ADAPT_BWD(int16_t, 1, true);
    } else {
        if (es == 4 && vec == 4) ADAPT_BWD(int32_t, 4, false);
        else if (es == 4) ADAPT_BWD(int32_t, 1, false);
        else if (es == 1 && vec == 16) ADAPT_BWD(int8_t, 16, false);
        else if (es == 1) ADAPT_BWD(int8_t, 1, false);
        else if (vec == 8) ADAPT_BWD(int16_t, 8, false);
        else ADAPT_BWD(int16_t, 1, false);
    }
#undef ADAPT_BWD
    return hip_status(ctx, hipGetLastError());
}

// ext_part / ext_n: per-block maxima that the kernel which produced `acc` has already stored (and, with sumsq, a cleared
// *sumsq): the pass over the accumulators that finds them is skipped
static int requantize_fit_exp(adapt_ctx *ctx, const void *acc, int acc_bits, size_t n, int wl, adapt_rng rng, void *q, int32_t *shift,
                              uint64_t *sumsq, const long long *e_in, long long e_add, long long *e_out,
                              const unsigned long long *ext_part = nullptr, int ext_n = 0)
{
    if (ctx && (acc_bits == 128 || (wl > 16 && wl <= 32)))
        return requantize_fit_wide(ctx, acc, acc_bits, n, wl, rng, q, shift, sumsq, e_in, e_add, e_out);
    if (!ctx || (acc_bits != 32 && acc_bits != 64) || wl < 2 || wl > 16 || !rng_ok(rng)) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if ((shift && ((uintptr_t)shift & 3)) || (sumsq && ((uintptr_t)sumsq & 7))) return ADAPT_EINVAL;
    if (n > 0 && (!acc || !q || !aligned16(acc) || !aligned16(q))) return ADAPT_EINVAL;
    const uint64_t groups = ((uint64_t)n + 7) >> 3;
    const int grid1 = (int)std::min<uint64_t>(std::max<uint64_t>((groups + kEwThreads - 1) / kEwThreads, 1), (uint64_t)ctx->num_cu * 4);
    // Atomic additions to one address retire at about one per 10 ns on this chip, whoever issues them:
    // with the sum of squares asked for, fewer and longer-running blocks keep that tail short.
    const int grid2 = sumsq ? std::min(ew_grid(ctx, groups), ctx->num_cu * 2) : ew_grid(ctx, groups);
    if ((size_t)grid1 * 8 > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    uint64_t *part = reinterpret_cast<uint64_t *>(scratch(ctx));
    unsigned long long *ss = reinterpret_cast<unsigned long long *>(sumsq);
    FitArgs a;
    a.acc = acc; a.q = q; a.part = part; a.nparts = grid1; a.n = n; a.wl = wl; a.mode = rng.mode; a.seed = rng.seed;
    a.stream = rng.stream; a.shift_out = shift; a.sumsq = ss; a.e_in = e_in; a.e_add = e_add; a.e_out = e_out;
    const dim3 block(kEwThreads);
    if (ext_part != nullptr && ext_n > 0) {
        a.part = reinterpret_cast<const uint64_t *>(ext_part);
        a.nparts = ext_n;
    } else if (acc_bits == 32) {
        hipLaunchKernelGGL(absmax_kernel<int32_t>, dim3(grid1), block, 0, ctx->stream, (const int32_t *)acc, (uint64_t)n, part, ss);
    } else {
        hipLaunchKernelGGL(absmax_kernel<int64_t>, dim3(grid1), block, 0, ctx->stream, (const int64_t *)acc, (uint64_t)n, part, ss);
    }
    const bool o8 = wl <= 8;
    if (acc_bits == 32 && o8) hipLaunchKernelGGL((requant_fit_kernel<int32_t, int8_t>), dim3(grid2), block, 0, ctx->stream, a);
    else if (acc_bits == 32) hipLaunchKernelGGL((requant_fit_kernel<int32_t, int16_t>), dim3(grid2), block, 0, ctx->stream, a);
    else if (o8) hipLaunchKernelGGL((requant_fit_kernel<int64_t, int8_t>), dim3(grid2), block, 0, ctx->stream, a);
    else hipLaunchKernelGGL((requant_fit_kernel<int64_t, int16_t>), dim3(grid2), block, 0, ctx->stream, a);
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_requantize_fit(adapt_ctx *ctx, const void *acc, int acc_bits, size_t n, int wl, adapt_rng rng, void *q,
                                    int32_t *shift, uint64_t *sumsq)
{
    return requantize_fit_exp(ctx, acc, acc_bits, n, wl, rng, q, shift, sumsq, nullptr, 0, nullptr);
}

// *dst = (src ? *src : 0) + add: the exponent bookkeeping of the chained step stays on the device
__global__ void exp_set_kernel(long long *dst, const long long *src, long long add) { *dst = (src ? *src : 0) + add; }

extern "C" int adapt_residual_add(adapt_ctx *ctx, const void *a, adapt_fmt fa, const void *b, adapt_fmt fb, size_t n,
                                  adapt_fmt fo, adapt_rng rng, int relu, void *out)
{
    if (!ctx || !fmt_ok_wide(fa) || !fmt_ok_wide(fb) || !fmt_ok_wide(fo) || !rng_ok(rng)) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if (n == 0) return ADAPT_OK;
    if (!a || !b || !out || !aligned16(a) || !aligned16(b) || !aligned16(out)) return ADAPT_EINVAL;
    const int f = std::max(fa.fl, fb.fl);
    AddArgs p;
    p.a = a; p.b = b; p.out = out; p.n = n; p.sa = f - fa.fl; p.sb = f - fb.fl; p.shift = f - fo.fl; p.wl = fo.wl;
    p.relu = relu != 0; p.mode = rng.mode; p.seed = rng.seed; p.stream = rng.stream;
    if (fa.wl > 16 || fb.wl > 16 || fo.wl > 16) {
        hipLaunchKernelGGL(residual_add_wide_kernel, dim3(ew_grid(ctx, (uint64_t)n)), dim3(kEwThreads), 0, ctx->stream, p, storage_bytes(fa),
                           storage_bytes(fb), storage_bytes(fo));
        return hip_status(ctx, hipGetLastError());
    }
    const dim3 grid(ew_grid(ctx, ((uint64_t)n + 7) >> 3)), block(kEwThreads);
    const int sel = (storage_bytes(fa) == 2) * 4 + (storage_bytes(fb) == 2) * 2 + (storage_bytes(fo) == 2);
#define ADAPT_ADD(TA, TB, TO) hipLaunchKernelGGL((residual_add_kernel<TA, TB, TO>), grid, block, 0, ctx->stream, p)
    switch (sel) {
    case 0: ADAPT_ADD(int8_t, int8_t, int8_t); break;
    case 1: ADAPT_ADD(int8_t, int8_t, int16_t); break;
    case 2: ADAPT_ADD(int8_t, int16_t, int8_t); break;
    case 3: ADAPT_ADD(int8_t, int16_t, int16_t); break;
    case 4: ADAPT_ADD(int16_t, int8_t, int8_t); break;
    case 5: ADAPT_ADD(int16_t, int8_t, int16_t); break;
    case 6: ADAPT_ADD(int16_t, int16_t, int8_t); break;
    default: ADAPT_ADD(int16_t, int16_t, int16_t); break;
    }
#undef ADAPT_ADD
    return hip_status(ctx, hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// the chained step
// ---------------------------------------------------------------------------------------------

namespace {

constexpr int kMaxLayers = 64;
constexpr int kRingMax = 65;           // ring slots per layer: the longest window and the gradient being made
constexpr size_t kStatBytes = 64;      // per layer: the adapt_net_stats record
constexpr int kAmaxCap = 8192;         // per-block maxima a gradient contraction may leave for the fitting pass (more: a pass of its own)
constexpr size_t kExpBytes = 32;       // per layer: exponents of da, of the gradient at the convolution output, of dW

// random streams of the steps that only residual / batch-norm networks have
constexpr uint64_t kStreamX = (uint64_t)1 << 20;
enum { X_BN = 0, X_BNB = 1, X_GAP = 2, X_MERGE = 3 };

struct NetLayer {
    adapt_layer_desc d;
    int bn, src, res, gap;    // src: the layer that feeds the convolution (-1: the network input); res: shortcut layer or -1
    adapt_fmt fmt;
    float *w;                 // master weights (caller's)
    float *gamma, *beta;      // batch-norm parameters (caller's) or null
    int p, q;                 // contraction output size
    size_t n_y, n_a, n_in, n_w;
    size_t off_y, off_a, off_dy, off_da, off_qw, off_g, off_stat, off_ring, off_ds, off_kld, off_sel;
    size_t off_yc, off_dyc, off_bn, off_dgam, off_dbet, off_dgap, off_exp;
    // state of the last backward pass
    int g_wl;                 // word length of the gradient codes
    int g_slot;               // with precision switching: the ring slot that holds them (never one of the window's)
    int fl_in, fl_w;          // FL of the layer's input activations and of its weight codes
    bool range_valid;         // the statistics record holds the range of the master weights as they are now
    // precision switch (Alg. 2)
    int lb, res_bins;
    std::vector<int> win;     // ring slots of the window, oldest first
    int slot_wl[kRingMax];
    long long slot_exp[kRingMax];
    size_t slot_bytes;

    // where the gradient codes of the last backward pass lie in the workspace
    size_t g_off() const { return g_slot >= 0 ? off_ring + (size_t)g_slot * slot_bytes : off_g; }
};

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr size_t kKldStride = 256;      // bytes per layer for the KL values of up to 31 candidates

struct NetPlan {
    size_t off_in, off_accx, off_accw, off_amax, off_stats, off_sel_group, off_kld_group, off_win, off_tmp, bytes;
};

// Lays the workspace out; returns false for an invalid network.
// wl_max: the largest word length any layer may take (16: int16 storage everywhere; 32: int32 storage and 128-bit
// accumulators)
bool plan_net(const adapt_node_desc *descs, int count, int lb_upr, int wl_max, std::vector<NetLayer> &L, NetPlan &P)
{
    if (!descs || count < 1 || count > kMaxLayers || lb_upr < 0 || lb_upr > 64 || (wl_max != 16 && wl_max != 32)) return false;
    const size_t cb = wl_max > 16 ? 4 : 2;              // bytes per code
    const size_t ab = wl_max > 16 ? 16 : 8;             // bytes per exact accumulator
    L.assign(count, NetLayer());
    size_t off = 0, max_in = 0, max_w = 0, max_merge = 0;
    auto take = [&off](size_t bytes) { const size_t o = off; off += align_up(std::max<size_t>(bytes, 16)); return o; };
    const int n = descs[0].conv.n;
    if (n < 1) return false;
    // records that the host reads back in one copy each: stats, diversities, selections, KL values
    P.off_stats = take((size_t)count * kStatBytes);
    const size_t off_ds = take((size_t)count * 16), off_sel = take((size_t)count * 8), off_kld = take((size_t)count * kKldStride);
    P.off_sel_group = off_sel;     // the batched searches of a precision switch write their results densely, in group order
    P.off_kld_group = off_kld;
    P.off_win = take((size_t)count * sizeof(GradWindow));
    const size_t off_exp = take((size_t)count * kExpBytes);
    std::vector<int> consumers(count, 0);
    for (int l = 0; l < count; ++l) {
        const adapt_conv_desc &c = descs[l].conv;
        if (c.n != n || c.h < 1 || c.w < 1 || c.c < 1 || c.k < 1 || c.r < 1 || c.s < 1 || c.stride < 1 || c.pad < 0) return false;
        if (c.h + 2 * c.pad < c.r || c.w + 2 * c.pad < c.s) return false;
        NetLayer &y = L[l];
        y.d.conv = c;
        y.d.relu = descs[l].relu;
        y.d.pool = descs[l].pool;
        y.bn = descs[l].bn != 0;
        y.gap = descs[l].gap != 0;
        y.src = descs[l].src >= 0 ? descs[l].src : l - 1;
        y.res = descs[l].res;
        if (y.src >= l || descs[l].src < -1 || y.res >= l || y.res < -1) return false;
        if (y.res >= 0 && !y.bn) return false;                     // the shortcut is added inside the batch-norm output
        if (y.gap && y.d.pool) return false;
        y.fmt = adapt_fmt{8, 4};
        y.w = nullptr;
        y.gamma = y.beta = nullptr;
        y.p = (c.h + 2 * c.pad - c.r) / c.stride + 1;
        y.q = (c.w + 2 * c.pad - c.s) / c.stride + 1;
        if (y.d.pool && ((y.p | y.q) & 1)) return false;
        if (y.gap && (((y.p * y.q) & (y.p * y.q - 1)) || (c.k & 7))) return false;
        if (y.bn && ((c.k & 7) || c.k > 4096 || (size_t)n * y.p * y.q > ((size_t)1 << 23))) return false;
        y.n_in = (size_t)n * c.h * c.w * c.c;
        y.n_y = (size_t)n * y.p * y.q * c.k;
        y.n_a = y.d.pool ? y.n_y / 4 : y.gap ? (size_t)n * c.k : y.n_y;
        y.n_w = (size_t)c.k * c.r * c.s * c.c;
        if (y.src >= 0 && L[y.src].n_a != y.n_in) return false;   // the output of the source layer is what this one reads
        if (y.res >= 0 && L[y.res].n_a != y.n_y) return false;
        if (y.src >= 0) ++consumers[y.src];
        if (y.res >= 0) ++consumers[y.res];
        // every code buffer holds the widest storage, so a layer may change its word length later
        const bool post = y.d.pool || y.gap;                        // something follows the activation
        y.off_y = take(cb * y.n_y);
        y.off_a = post ? take(cb * y.n_a) : y.off_y;
        y.off_da = take(cb * y.n_a);
        y.off_dgap = y.gap ? take(cb * y.n_y) : 0;
        y.off_dy = (y.d.pool || y.d.relu) ? take(cb * y.n_y) : (y.gap ? y.off_dgap : y.off_da);
        y.off_yc = y.bn ? take(cb * y.n_y) : 0;
        y.off_dyc = y.bn ? take(cb * y.n_y) : y.off_dy;
        y.off_bn = y.bn ? take(adapt_bn_state_bytes(c.k)) : 0;
        y.off_dgam = y.bn ? take((size_t)c.k * 8) : 0;
        y.off_dbet = y.bn ? take((size_t)c.k * 8) : 0;
        y.off_qw = take(cb * y.n_w);
        // The weight gradient is written straight into a slot of the lookback ring (one slot more than the longest
        // window, so a free one always exists); without precision switching it has a buffer of its own.
        y.off_g = lb_upr ? 0 : take(cb * y.n_w);
        y.g_slot = -1;
        y.slot_bytes = align_up(cb * y.n_w);
        y.off_stat = P.off_stats + (size_t)l * kStatBytes;
        y.off_exp = off_exp + (size_t)l * kExpBytes;
        y.off_ds = off_ds + (size_t)l * 16;
        y.off_sel = off_sel + (size_t)l * 8;
        y.off_kld = off_kld + (size_t)l * kKldStride;
        y.off_ring = lb_upr ? take((size_t)(lb_upr + 1) * y.slot_bytes) : 0;
        y.g_wl = 0;
        y.range_valid = false;
        if (y.src >= 0) max_in = std::max(max_in, y.n_in);
        max_w = std::max(max_w, y.n_w);
    }
    for (int l = 0; l < count; ++l) {
        if (l < count - 1 && consumers[l] == 0) return false;     // an output nobody reads has no gradient
        if (consumers[l] > 4) return false;
        if (consumers[l] > 1) max_merge = std::max(max_merge, L[l].n_a);
    }
    P.off_in = take(cb * L[0].n_in);
    P.off_accx = take(ab * max_in);
    P.off_accw = take(ab * max_w);
    P.off_tmp = max_merge ? take(cb * max_merge) : 0;
    P.off_amax = take((size_t)2 * kAmaxCap * 8);                 // per-block maxima of the two gradient contractions of a layer
    P.bytes = off;
    return true;
}

struct ExpRec { long long e_da, e_dyc, e_g, spare; };

}  // namespace

struct adapt_net {
    adapt_ctx *ctx;
    std::vector<NetLayer> L;
    char *ws;
    NetPlan P;
    double bn_eps;
    int wl_max;               // 16, or 32 for a chain laid out for int32 codes
    bool forward_done, backward_done;
    int dlogits_fl;
    // precision switch
    bool has_switch;
    bool switch_due;          // a backward pass whose gradients have not joined the windows yet
    adapt_switch_params sp;
    int strategy;
    std::vector<double> losses;
    void *pinned;             // host-pinned, device-visible: count ChainLayerIn records, then count ChainLayerOut
    ChainLayerIn *chain_in;
    ChainLayerOut *chain_out;

    ExpRec *exps(int l) const { return reinterpret_cast<ExpRec *>(ws + L[l].off_exp); }
};

namespace {

adapt_rng slot_rng(adapt_rng r, int layer, int slot)
{
    r.stream += (uint64_t)(8 * layer + slot);
    return r;
}
adapt_rng slot_rng_x(adapt_rng r, int layer, int slot)
{
    r.stream += kStreamX + (uint64_t)(8 * layer + slot);
    return r;
}

adapt_epilogue exact_ep()
{
    adapt_epilogue e = {};
    e.raw = 1;
    e.fmt = adapt_fmt{8, 0};
    e.rng.mode = ADAPT_RN_HALF_UP;
    return e;
}

}  // namespace

static bool switch_params_ok(const adapt_switch_params &p, int wl_max)
{
    if (p.lb_lwr < 1 || p.lb_upr < p.lb_lwr || p.lb_upr > 64 || p.lb_init < p.lb_lwr || p.lb_init > p.lb_upr) return false;
    if (p.r_lwr < 2 || p.r_upr < p.r_lwr || p.r_upr > 65536 || p.r_init < p.r_lwr || p.r_init > p.r_upr) return false;
    if (!(p.gamma >= 0.0 && p.gamma <= 1.0) || !(p.eps >= 0.0)) return false;
    if (p.buff < 1 || p.buff > wl_max - 1 || p.wl_lo < 2 || p.wl_hi < p.wl_lo || p.wl_hi > wl_max) return false;
    return p.strategy_init >= ADAPT_ST_MIN && p.strategy_init <= ADAPT_ST_MAX;
}

static std::vector<adapt_node_desc> plain_nodes(const adapt_layer_desc *layers, int count)
{
    std::vector<adapt_node_desc> nodes;
    if (!layers || count < 1 || count > kMaxLayers) return nodes;
    nodes.resize(count);
    for (int l = 0; l < count; ++l) {
        nodes[l] = adapt_node_desc{};
        nodes[l].conv = layers[l].conv;
        nodes[l].relu = layers[l].relu;
        nodes[l].pool = layers[l].pool;
        nodes[l].src = nodes[l].res = -1;
    }
    return nodes;
}

extern "C" size_t adapt_graph_workspace_bytes(const adapt_node_desc *nodes, int count, int lb_upr)
{
    std::vector<NetLayer> L;
    NetPlan P;
    return plan_net(nodes, count, lb_upr, 16, L, P) ? P.bytes : 0;
}

extern "C" size_t adapt_net_workspace_bytes(const adapt_layer_desc *layers, int count, int lb_upr)
{
    const std::vector<adapt_node_desc> nodes = plain_nodes(layers, count);
    return nodes.empty() ? 0 : adapt_graph_workspace_bytes(nodes.data(), count, lb_upr);
}

extern "C" size_t adapt_graph_workspace_bytes_wide(const adapt_node_desc *nodes, int count, int lb_upr, int wl_max)
{
    std::vector<NetLayer> L;
    NetPlan P;
    return plan_net(nodes, count, lb_upr, wl_max, L, P) ? P.bytes : 0;
}

extern "C" size_t adapt_net_workspace_bytes_wide(const adapt_layer_desc *layers, int count, int lb_upr, int wl_max)
{
    const std::vector<adapt_node_desc> nodes = plain_nodes(layers, count);
    std::vector<NetLayer> L;
    NetPlan P;
    return (!nodes.empty() && plan_net(nodes.data(), count, lb_upr, wl_max, L, P)) ? P.bytes : 0;
}

static int graph_create(adapt_ctx *ctx, const adapt_node_desc *nodes, int count, float *const *weights, float *const *gammas,
                        float *const *betas, double bn_eps, const adapt_switch_params *sp, int wl_max, void *workspace,
                        size_t workspace_bytes, adapt_net **out)
{
    if (!ctx || !out || !weights || !workspace || ((uintptr_t)workspace & 255) || !(bn_eps >= 0.0)) return ADAPT_EINVAL;
    if (wl_max != 16 && wl_max != 32) return ADAPT_EINVAL;
    if (sp && !switch_params_ok(*sp, wl_max)) return ADAPT_EINVAL;
    adapt_net *net = new (std::nothrow) adapt_net();
    if (!net) return ADAPT_EINVAL;
    net->ctx = ctx;
    net->ws = static_cast<char *>(workspace);
    net->forward_done = net->backward_done = false;
    net->dlogits_fl = 0;
    net->bn_eps = bn_eps;
    net->wl_max = wl_max;
    net->has_switch = sp != nullptr;
    net->switch_due = false;
    if (sp) net->sp = *sp;
    net->strategy = sp ? sp->strategy_init : ADAPT_ST_MIN;
    net->pinned = nullptr;
    net->chain_in = nullptr;
    net->chain_out = nullptr;
    const bool planned = plan_net(nodes, count, sp ? sp->lb_upr : 0, wl_max, net->L, net->P);
    bool ok = planned && net->P.bytes <= workspace_bytes;
    for (int l = 0; ok && l < count; ++l) {
        NetLayer &y = net->L[l];
        y.w = weights[l];
        y.lb = sp ? sp->lb_init : 0;
        y.res_bins = sp ? sp->r_init : 0;
        ok = weights[l] != nullptr && aligned16(weights[l]);
        if (ok && y.bn) {
            ok = gammas && betas && gammas[l] && betas[l];
            if (ok) { y.gamma = gammas[l]; y.beta = betas[l]; }
        }
    }
    if (ok && sp) {
        const size_t in_bytes = align_up((size_t)count * sizeof(ChainLayerIn));
        const hipError_t e = hipHostMalloc(&net->pinned, in_bytes + (size_t)count * sizeof(ChainLayerOut), hipHostMallocDefault);
        if (e != hipSuccess) {
            delete net;
            return hip_status(ctx, e);
        }
        net->chain_in = static_cast<ChainLayerIn *>(net->pinned);
        net->chain_out = reinterpret_cast<ChainLayerOut *>(static_cast<char *>(net->pinned) + in_bytes);
    }
    if (!ok) {
        const int s = (planned && net->P.bytes > workspace_bytes) ? ADAPT_EWORKSPACE : ADAPT_EINVAL;
        delete net;
        return s;
    }
    *out = net;
    return ADAPT_OK;
}

extern "C" int adapt_graph_create(adapt_ctx *ctx, const adapt_node_desc *nodes, int count, float *const *weights, float *const *gammas,
                                  float *const *betas, double bn_eps, const adapt_switch_params *sp, void *workspace,
                                  size_t workspace_bytes, adapt_net **out)
{
    return graph_create(ctx, nodes, count, weights, gammas, betas, bn_eps, sp, 16, workspace, workspace_bytes, out);
}

extern "C" int adapt_graph_create_wide(adapt_ctx *ctx, const adapt_node_desc *nodes, int count, float *const *weights,
                                       float *const *gammas, float *const *betas, double bn_eps, const adapt_switch_params *sp, int wl_max,
                                       void *workspace, size_t workspace_bytes, adapt_net **out)
{
    return graph_create(ctx, nodes, count, weights, gammas, betas, bn_eps, sp, wl_max, workspace, workspace_bytes, out);
}

extern "C" int adapt_net_create(adapt_ctx *ctx, const adapt_layer_desc *layers, int count, float *const *weights,
                                const adapt_switch_params *sp, void *workspace, size_t workspace_bytes, adapt_net **out)
{
    const std::vector<adapt_node_desc> nodes = plain_nodes(layers, count);
    if (nodes.empty()) return ADAPT_EINVAL;
    return graph_create(ctx, nodes.data(), count, weights, nullptr, nullptr, 0.0, sp, 16, workspace, workspace_bytes, out);
}

extern "C" int adapt_net_create_wide(adapt_ctx *ctx, const adapt_layer_desc *layers, int count, float *const *weights,
                                     const adapt_switch_params *sp, int wl_max, void *workspace, size_t workspace_bytes,
                                     adapt_net **out)
{
    const std::vector<adapt_node_desc> nodes = plain_nodes(layers, count);
    if (nodes.empty()) return ADAPT_EINVAL;
    return graph_create(ctx, nodes.data(), count, weights, nullptr, nullptr, 0.0, sp, wl_max, workspace, workspace_bytes, out);
}

extern "C" int adapt_net_destroy(adapt_net *net)
{
    if (net && net->pinned) {
        // the device may still be reading or writing the pinned records of the last precision switch
        (void)hipStreamSynchronize(net->ctx->stream);
        (void)hipHostFree(net->pinned);
    }
    delete net;
    return ADAPT_OK;
}

extern "C" int adapt_net_set_format(adapt_net *net, int layer, adapt_fmt f)
{
    if (!net || layer < 0 || layer >= (int)net->L.size() || !fmt_ok_wide(f) || f.wl > net->wl_max) return ADAPT_EINVAL;
    net->L[layer].fmt = f;
    net->forward_done = net->backward_done = false;
    return ADAPT_OK;
}

extern "C" int adapt_net_tensor(const adapt_net *net, int layer, int which, size_t *offset, size_t *count, int *elem_bytes)
{
    if (!net || !offset || !count || !elem_bytes) return ADAPT_EINVAL;
    if (which == ADAPT_NT_INPUT) layer = 0;                 // the network input belongs to no layer
    if (layer < 0 || layer >= (int)net->L.size()) return ADAPT_EINVAL;
    const NetLayer &y = net->L[layer];
    const int es = storage_bytes(y.fmt);
    switch (which) {
    case ADAPT_NT_INPUT: *offset = net->P.off_in; *count = net->L[0].n_in; *elem_bytes = storage_bytes(net->L[0].fmt); break;
    case ADAPT_NT_Y: *offset = y.off_y; *count = y.n_y; *elem_bytes = es; break;
    case ADAPT_NT_A: *offset = y.off_a; *count = y.n_a; *elem_bytes = es; break;
    case ADAPT_NT_DY: *offset = y.off_dy; *count = y.n_y; *elem_bytes = es; break;
    case ADAPT_NT_DA: *offset = y.off_da; *count = y.n_a; *elem_bytes = es; break;
    case ADAPT_NT_QW: *offset = y.off_qw; *count = y.n_w; *elem_bytes = es; break;
    case ADAPT_NT_G: *offset = y.g_off(); *count = y.n_w; *elem_bytes = y.g_wl ? storage_bytes(adapt_fmt{y.g_wl, 0}) : es; break;
    case ADAPT_NT_STATS: *offset = y.off_stat; *count = 1; *elem_bytes = (int)sizeof(adapt_net_stats); break;
    case ADAPT_NT_YC: if (!y.bn) return ADAPT_EINVAL; *offset = y.off_yc; *count = y.n_y; *elem_bytes = es; break;
    case ADAPT_NT_DYC: *offset = y.off_dyc; *count = y.n_y; *elem_bytes = es; break;
    case ADAPT_NT_BN: if (!y.bn) return ADAPT_EINVAL; *offset = y.off_bn; *count = adapt_bn_state_bytes(y.d.conv.k); *elem_bytes = 1; break;
    case ADAPT_NT_EXP: *offset = y.off_exp; *count = 4; *elem_bytes = 8; break;
    case ADAPT_NT_DGAMMA: if (!y.bn) return ADAPT_EINVAL; *offset = y.off_dgam; *count = (size_t)y.d.conv.k; *elem_bytes = 8; break;
    case ADAPT_NT_DBETA: if (!y.bn) return ADAPT_EINVAL; *offset = y.off_dbet; *count = (size_t)y.d.conv.k; *elem_bytes = 8; break;
    default: return ADAPT_EINVAL;
    }
    return ADAPT_OK;
}

extern "C" int adapt_net_quantize_weights(adapt_net *net, adapt_rng rng)
{
    if (!net || !rng_ok(rng)) return ADAPT_EINVAL;
    const int count = (int)net->L.size();
    for (NetLayer &y : net->L) y.range_valid = false;          // the caller may have written the master weights
    adapt_quantize_item items[kMaxLayers];
    for (int l = 0; l < count; ++l) {
        const NetLayer &y = net->L[l];
        items[l].x = y.w;
        items[l].q = net->ws + y.off_qw;
        items[l].n = y.n_w;
        items[l].wl = y.fmt.wl;
        items[l].fl = y.fmt.fl;
        items[l].stream = rng.stream + (uint64_t)(8 * l + 5);
    }
    return adapt_quantize_batched(net->ctx, items, count, rng.mode, rng.seed, nullptr);
}

extern "C" int adapt_net_forward(adapt_net *net, const float *x, adapt_rng rng)
{
    if (!net || !x || !aligned16(x) || !rng_ok(rng)) return ADAPT_EINVAL;
    adapt_ctx *ctx = net->ctx;
    const int count = (int)net->L.size();
    net->forward_done = net->backward_done = false;
    if (int s = adapt_quantize(ctx, x, net->L[0].n_in, net->L[0].fmt, slot_rng(rng, 0, 4), net->ws + net->P.off_in, nullptr, nullptr))
        return s;
    for (int l = 0; l < count; ++l) {
        const NetLayer &y = net->L[l];
        const adapt_conv_desc &c = y.d.conv;
        const void *cur = y.src >= 0 ? net->ws + net->L[y.src].off_a : net->ws + net->P.off_in;
        const adapt_fmt fcur = y.src >= 0 ? net->L[y.src].fmt : net->L[0].fmt;
        adapt_epilogue ep = {};
        ep.raw = 0;
        ep.fmt = y.fmt;
        ep.rng = slot_rng(rng, l, 0);
        ep.relu = !y.bn && y.d.relu != 0;                           // with batch norm the ReLU follows the normalisation
        char *conv_out = net->ws + (y.bn ? y.off_yc : y.off_y);
        if (int s = adapt_conv_fwd(ctx, c, cur, fcur, net->ws + y.off_qw, y.fmt, conv_out, ep)) return s;
        if (y.bn) {
            const void *res = y.res >= 0 ? net->ws + net->L[y.res].off_a : nullptr;
            const adapt_fmt fres = y.res >= 0 ? net->L[y.res].fmt : adapt_fmt{8, 0};
            if (int s = adapt_bn_forward(ctx, conv_out, y.fmt, (size_t)c.n * y.p * y.q, c.k, y.gamma, y.beta, net->bn_eps, res, fres, y.fmt,
                                         slot_rng_x(rng, l, X_BN), y.d.relu, net->ws + y.off_y, net->ws + y.off_bn))
                return s;
        }
        if (y.d.pool)
            if (int s = adapt_maxpool2_fwd(ctx, net->ws + y.off_y, y.fmt, c.n, y.p, y.q, c.k, net->ws + y.off_a)) return s;
        if (y.gap)
            if (int s = adapt_gap_fwd(ctx, net->ws + y.off_y, y.fmt, c.n, y.p * y.q, c.k, slot_rng_x(rng, l, X_GAP), net->ws + y.off_a)) return s;
    }
    net->forward_done = true;
    return ADAPT_OK;
}

extern "C" int adapt_net_backward(adapt_net *net, const void *dlogits, int dlogits_fl, adapt_rng rng)
{
    if (!net || !dlogits || !aligned16(dlogits) || !rng_ok(rng)) return ADAPT_EINVAL;
    if (!net->forward_done) return ADAPT_EINVAL;
    adapt_ctx *ctx = net->ctx;
    const int count = (int)net->L.size();
    const adapt_epilogue ex = exact_ep();
    net->backward_done = false;
    net->dlogits_fl = dlogits_fl;
    int ncontrib[kMaxLayers] = {};
    // The gradient of layer j's output is the sum of what its consumers hand back.  The first contribution is stored
    // (refitted to layer j's word length when it comes from a layer of another word length), every later one is added
    // to it exactly and the sum refitted.  Exponents stay in device memory.
    auto contribute = [&](int j, const void *codes, int wl, const long long *e, bool fitted) -> int {
        NetLayer &t = net->L[j];
        const int k = ncontrib[j]++;
        char *dst = net->ws + t.off_da;
        long long *e_dst = &net->exps(j)->e_da;
        if (k == 0 && fitted) return ADAPT_OK;                       // written in place by the fitting pass
        if (k == 0) return adapt_grad_add(ctx, codes, wl, (const int64_t *)e, nullptr, 8, nullptr, t.n_a, t.fmt.wl,
                                          slot_rng_x(rng, j, X_MERGE), dst, nullptr, (int64_t *)e_dst);
        return adapt_grad_add(ctx, dst, t.fmt.wl, (const int64_t *)e_dst, codes, wl, (const int64_t *)e, t.n_a, t.fmt.wl,
                              slot_rng_x(rng, j, X_MERGE + k), dst, nullptr, (int64_t *)e_dst);
    };
    hipLaunchKernelGGL(exp_set_kernel, dim3(1), dim3(1), 0, ctx->stream, &net->exps(count - 1)->e_da, (const long long *)nullptr,
                       (long long)dlogits_fl);
    for (int l = count - 1; l >= 0; --l) {
        NetLayer &y = net->L[l];
        const adapt_conv_desc &c = y.d.conv;
        ExpRec *ex_l = net->exps(l);
        const void *da = (l == count - 1) ? dlogits : net->ws + y.off_da;
        const long long *e_cur = &ex_l->e_da;
        if (y.gap) {
            int up = 0;
            while ((1 << up) < y.p * y.q) ++up;
            if (int s = adapt_gap_bwd(ctx, da, y.fmt.wl, c.n, y.p * y.q, c.k, net->ws + y.off_dgap)) return s;
            hipLaunchKernelGGL(exp_set_kernel, dim3(1), dim3(1), 0, ctx->stream, &ex_l->spare, e_cur, (long long)up);
            da = net->ws + y.off_dgap;
            e_cur = &ex_l->spare;
        }
        const void *dz = da;
        if (y.d.relu || y.d.pool) {
            if (int s = adapt_relu_pool_bwd(ctx, da, net->ws + y.off_y, y.fmt, c.n, y.p, y.q, c.k, y.d.relu, y.d.pool, net->ws + y.off_dy))
                return s;
            dz = net->ws + y.off_dy;
        }
        if (y.res >= 0)
            if (int s = contribute(y.res, dz, y.fmt.wl, e_cur, false)) return s;
        adapt_net_stats *st = reinterpret_cast<adapt_net_stats *>(net->ws + y.off_stat);
        const void *dyc = dz;
        if (y.bn) {
            if (int s = adapt_bn_backward(ctx, dz, y.fmt.wl, net->ws + y.off_yc, y.fmt, (size_t)c.n * y.p * y.q, c.k, net->ws + y.off_bn,
                                          y.fmt.wl, slot_rng_x(rng, l, X_BNB), net->ws + y.off_dyc,
                                          reinterpret_cast<double *>(net->ws + y.off_dgam), reinterpret_cast<double *>(net->ws + y.off_dbet),
                                          &st->reserved[0], (const int64_t *)e_cur, (int64_t *)&ex_l->e_dyc))
                return s;
            dyc = net->ws + y.off_dyc;
            e_cur = &ex_l->e_dyc;
        }
        const adapt_fmt fdy = {y.fmt.wl, 0};                       // gradient codes of the layer's word length
        const adapt_fmt fin = y.src >= 0 ? net->L[y.src].fmt : net->L[0].fmt;
        const void *a_prev = y.src >= 0 ? net->ws + net->L[y.src].off_a : net->ws + net->P.off_in;
        y.g_wl = y.fmt.wl;
        y.fl_in = fin.fl;
        y.fl_w = y.fmt.fl;
        if (net->has_switch) {                                    // a ring slot outside the window
            bool used[kRingMax] = {};
            for (int s2 : y.win) used[s2] = true;
            y.g_slot = 0;
            while (used[y.g_slot]) ++y.g_slot;
        }
        char *accw = net->ws + net->P.off_accw, *accx = net->ws + net->P.off_accx;
        // The launches that write the exact gradients also leave their blocks' largest magnitudes (and clear the sum of
        // squares the fitting pass adds to), so that the fitting passes need no pass of their own to find them.  The
        // composed contractions above 16 bits do not (the sinks stay unarmed for them): their counts stay 0.
        unsigned long long *amax_x = reinterpret_cast<unsigned long long *>(net->ws + net->P.off_amax), *amax_w = amax_x + kAmaxCap;
        if (fdy.wl <= 16 && y.fmt.wl <= 16 && fin.wl <= 16) {
            ctx->amax[0] = adapt_amax_sink{amax_x, nullptr, kAmaxCap, 0};
            ctx->amax[1] = adapt_amax_sink{amax_w, reinterpret_cast<unsigned long long *>(&st->g_sumsq), kAmaxCap, 0};
        }
        int s_bwd;
        if (y.src >= 0) s_bwd = adapt_conv_backward(ctx, c, dyc, fdy, net->ws + y.off_qw, y.fmt, a_prev, fin, accx, ex, accw, ex);
        else s_bwd = adapt_conv_wgrad(ctx, c, dyc, fdy, a_prev, fin, accw, ex);
        const int n_amax_x = ctx->amax[0].count, n_amax_w = ctx->amax[1].count;
        ctx->amax[0] = ctx->amax[1] = adapt_amax_sink{};
        if (s_bwd) return s_bwd;
        const int bits_w = adapt_acc_bits((int64_t)c.n * y.p * y.q, fdy, fin);
        if (int s = requantize_fit_exp(ctx, accw, bits_w, y.n_w, y.fmt.wl, slot_rng(rng, l, 2), net->ws + y.g_off(), &st->shift_w,
                                       &st->g_sumsq, e_cur, fin.fl, &ex_l->e_g, amax_w, n_amax_w))
            return s;
        if (y.src >= 0) {
            NetLayer &t = net->L[y.src];
            const bool first = ncontrib[y.src] == 0;
            const int bits_x = adapt_acc_bits((int64_t)c.r * c.s * c.k, fdy, y.fmt);
            char *dst = first ? net->ws + t.off_da : net->ws + net->P.off_tmp;
            long long *e_dst = first ? &net->exps(y.src)->e_da : &ex_l->spare;
            if (int s = requantize_fit_exp(ctx, accx, bits_x, y.n_in, t.fmt.wl, slot_rng(rng, l, 1), dst, &st->shift_a, nullptr, e_cur,
                                           y.fmt.fl, e_dst, amax_x, n_amax_x))
                return s;
            if (int s = contribute(y.src, dst, t.fmt.wl, e_dst, true)) return s;
        }
    }
    net->backward_done = true;
    net->switch_due = net->has_switch;
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_net_precision_switch(adapt_net *net, double loss, adapt_rng rng, adapt_switch_report *report, int *strategy)
{
    if (!net || !net->has_switch || !net->backward_done || !net->switch_due || !rng_ok(rng) || !(loss == loss)) return ADAPT_EINVAL;
    adapt_ctx *ctx = net->ctx;
    const adapt_switch_params &sp = net->sp;
    const int count = (int)net->L.size();
    // Nothing of the network's state changes before the last step that can fail has passed: a call that returns an
    // error leaves strategy, loss history, windows, lookbacks, resolutions and formats as they were, and may be repeated.
    for (const NetLayer &y : net->L)
        if (y.fmt.wl - y.fmt.fl < 1 || y.g_slot < 0) return ADAPT_EINVAL;

    // strategy from the loss history (the current batch excluded)
    int strategy_new = net->strategy;
    if (!net->losses.empty()) {
        long long lb_sum = 0;
        for (const NetLayer &y : net->L) lb_sum += y.lb;
        const size_t k = std::min<size_t>(net->losses.size(), (size_t)std::ceil((double)lb_sum / (double)count));
        double acc = 0.0;
        for (size_t i = net->losses.size() - k; i < net->losses.size(); ++i) acc += net->losses[i];
        strategy_new = adapt_strategy_next(net->strategy, acc / (double)k, loss);
    }

    // Windows as they will be once this batch's gradients have joined them, and their diversities.  The exponent of
    // every gradient tensor of this backward pass lies in device memory (the fitting passes wrote it), so the device
    // lays the windows out itself.
    std::vector<std::vector<int>> win_new(count);
    size_t n_w[kMaxLayers];
    for (int l = count - 1; l >= 0; --l) {
        const NetLayer &y = net->L[l];
        std::vector<int> &w = win_new[l];
        w.assign(y.win.begin() + ((int)y.win.size() == sp.lb_upr ? 1 : 0), y.win.end());      // full: the oldest entry makes room
        w.push_back(y.g_slot);
        const int use = std::min<int>((int)w.size(), y.lb);
        ChainLayerIn &c = net->chain_in[l];
        c.count = use;
        for (int i = 0; i < use; ++i) {
            const int s2 = w[w.size() - use + i];
            c.g[i] = net->ws + y.off_ring + (size_t)s2 * y.slot_bytes;
            c.wl[i] = (uint8_t)(i == use - 1 ? y.g_wl : y.slot_wl[s2]);
            c.exp[i] = i == use - 1 ? 0 : y.slot_exp[s2];
        }
        n_w[l] = y.n_w;
    }
    if (int s = gradient_diversity_chain(ctx, net->chain_in, count, n_w, &net->exps(0)->e_g, kExpBytes / 8,
                                         reinterpret_cast<GradWindow *>(net->ws + net->P.off_win), net->chain_out))
        return s;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_status(ctx, e);
    const ChainLayerOut *out = net->chain_out;

    // lookback, resolution; PushDown for the layers whose window is long enough: one batched search per group of
    // layers that share the lowest candidate word length (the batched call takes one candidate range)
    std::vector<int> lb_new(count), res_new(count), lo_of(count, 0), group_slot(count, 0);
    std::vector<char> switches(count, 0);
    for (int l = 0; l < count; ++l) {
        const NetLayer &y = net->L[l];
        lb_new[l] = adapt_lookback_next(y.lb, out[l].ds, sp.lb_lwr, sp.lb_upr, sp.gamma);
        res_new[l] = adapt_resolution_next(y.res_bins, lb_new[l], sp.lb_lwr, sp.lb_upr, sp.r_lwr, sp.r_upr);
        switches[l] = (int)win_new[l].size() >= lb_new[l];
        if (switches[l]) lo_of[l] = std::max(sp.wl_lo, y.fmt.wl - y.fmt.fl);
    }
    int group_base = 0;
    for (int lo = 2; lo <= sp.wl_hi; ++lo) {
        adapt_kld_item items[kMaxLayers];
        const float *ranges[kMaxLayers];       // the last update left the range of the weights it wrote
        int members[kMaxLayers], m = 0;
        for (int l = 0; l < count; ++l) {
            const NetLayer &y = net->L[l];
            if (!switches[l] || lo_of[l] != lo) continue;
            items[m].w = y.w;
            items[m].n = y.n_w;
            items[m].il = y.fmt.wl - y.fmt.fl;
            items[m].bins = res_new[l];
            items[m].stream = rng.stream + (uint64_t)(8 * l + 6);
            ranges[m] = y.range_valid ? &reinterpret_cast<const adapt_net_stats *>(net->ws + y.off_stat)->range_lo : nullptr;
            members[m++] = l;
        }
        if (m == 0) continue;
        // the t-th member of a group writes kld[32 * (group_base + t)...] and sel[2 * (group_base + t)]
        double *gk = reinterpret_cast<double *>(net->ws + net->P.off_kld_group);
        int32_t *gs = reinterpret_cast<int32_t *>(net->ws + net->P.off_sel_group);
        if (int s = adapt_kld_precision_search_batched_ranged(ctx, items, ranges, m, lo, sp.wl_hi, sp.eps, -1.0, rng.mode, rng.seed,
                                                              gk + (size_t)group_base * 32, gs + 2 * (size_t)group_base))
            return s;
        for (int t = 0; t < m; ++t) group_slot[members[t]] = group_base + t;
        group_base += m;
    }
    std::vector<int32_t> sel(2 * (size_t)count, 0);
    if (group_base > 0) {
        e = hipMemcpyAsync(sel.data(), net->ws + net->P.off_sel_group, (size_t)group_base * 8, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) return hip_status(ctx, e);
    }
    std::vector<adapt_fmt> fmt_new(count);
    std::vector<int> wl_min_of(count, 0), fl_min_of(count, 0);
    for (int l = 0; l < count; ++l) {
        const NetLayer &y = net->L[l];
        fmt_new[l] = y.fmt;
        if (!switches[l]) continue;
        const int il = y.fmt.wl - y.fmt.fl;
        int wl_min = y.fmt.wl;
        if (lo_of[l] <= sp.wl_hi) wl_min = std::min<int>(sel[2 * (size_t)group_slot[l]], y.fmt.wl);
        const int fl_min = wl_min - il;
        adapt_pushup_result r;
        if (int s = adapt_pushup_suggest(out[l].ds, wl_min, fl_min, strategy_new, sp.buff, net->wl_max, &r)) return s;
        fmt_new[l] = adapt_fmt{r.wl, r.fl};
        wl_min_of[l] = wl_min;
        fl_min_of[l] = fl_min;
    }

    // commit
    net->strategy = strategy_new;
    net->losses.push_back(loss);
    net->switch_due = false;
    if (strategy) *strategy = strategy_new;
    for (int l = 0; l < count; ++l) {
        NetLayer &y = net->L[l];
        y.slot_wl[y.g_slot] = y.g_wl;
        y.slot_exp[y.g_slot] = out[l].exp_new;
        y.win.swap(win_new[l]);
        y.lb = lb_new[l];
        y.res_bins = res_new[l];
        if (switches[l]) {
            y.fmt = fmt_new[l];
            y.win.clear();
            net->forward_done = false;                   // activations of the old format no longer match
        }
        if (report) {
            report[l] = adapt_switch_report{};
            report[l].ds = out[l].ds;
            report[l].lb = y.lb;
            report[l].res = y.res_bins;
            report[l].used = out[l].used;
            report[l].switched = switches[l];
            report[l].wl_min = wl_min_of[l];
            report[l].fl_min = fl_min_of[l];
            report[l].wl = y.fmt.wl;
            report[l].fl = y.fmt.fl;
        }
    }
    return ADAPT_OK;
}

extern "C" int adapt_net_update(adapt_net *net, adapt_sgd_params opt, adapt_rng rng)
{
    if (!net || !rng_ok(rng)) return ADAPT_EINVAL;
    const int count = (int)net->L.size();
    for (int l = 0; l < count; ++l) {
        net->L[l].range_valid = false;
        if (net->L[l].g_wl == 0) return ADAPT_EINVAL;                // no backward pass yet
    }
    // gamma and beta of every normalisation layer in one launch
    std::vector<BnUpdateItem> bn_items;
    for (int l = 0; l < count; ++l) {
        NetLayer &y = net->L[l];
        if (y.bn)
            bn_items.push_back(BnUpdateItem{y.gamma, y.beta, reinterpret_cast<const double *>(net->ws + y.off_dgam),
                                            reinterpret_cast<const double *>(net->ws + y.off_dbet), y.d.conv.k});
    }
    // the weights: every layer whose gradient and weight codes have at most 16 bits in one batched launch pair, the
    // others one call each
    std::vector<SgdBatchItem> items;
    std::vector<int> single;
    for (int l = 0; l < count; ++l) {
        NetLayer &y = net->L[l];
        adapt_net_stats *st = reinterpret_cast<adapt_net_stats *>(net->ws + y.off_stat);
        if (y.g_wl > 16 || y.fmt.wl > 16) {
            if (ws_need_sgd_update(net->ctx->num_cu, y.n_w) > scratch_bytes(net->ctx)) return ADAPT_EWORKSPACE;
            single.push_back(l);
            continue;
        }
        const adapt_rng r = slot_rng(rng, l, 3);
        SgdBatchItem it = {};
        it.w = y.w; it.g = net->ws + y.g_off(); it.q = net->ws + y.off_qw; it.g_sumsq = &st->g_sumsq; it.n = y.n_w;
        it.seed = r.seed; it.stream = r.stream; it.counters = &st->nnz; it.range = &st->range_lo;
        it.es_g = (int8_t)(y.g_wl <= 8 ? 1 : 2); it.es_q = (int8_t)(y.fmt.wl <= 8 ? 1 : 2); it.fl_g = 0;
        it.wl = (int8_t)y.fmt.wl; it.fl = (int8_t)y.fmt.fl;
        items.push_back(it);
    }
    // The batched launch checks its arguments and its scratch before it enqueues anything, and it comes first: a call
    // that fails has changed nothing.  (The scratch it needs is what adapt_net_quantize_weights needs for the same layers:
    // a context that could quantize the weights can update them.)
    if (!items.empty())
        if (int s = sgd_update_batch(net->ctx, items.data(), (int)items.size(), opt, rng.mode)) return s;
    if (int s = bn_update_batch(net->ctx, bn_items.data(), (int)bn_items.size(), opt.lr)) return s;
    for (int l : single) {
        NetLayer &y = net->L[l];
        adapt_net_stats *st = reinterpret_cast<adapt_net_stats *>(net->ws + y.off_stat);
        const adapt_fmt fg = {y.g_wl, 0};                            // the gradient keeps the word length it was made with
        if (int s = adapt_sgd_update_quantize(net->ctx, y.w, y.n_w, net->ws + y.g_off(), fg, &st->g_sumsq, opt, y.fmt,
                                              slot_rng(rng, l, 3), net->ws + y.off_qw, &st->nnz, &st->range_lo))
            return s;
    }
    for (int l = 0; l < count; ++l) net->L[l].range_valid = true;
    net->forward_done = net->backward_done = false;
    return ADAPT_OK;
}
