// Quantize(L, <WL,FL>) of Alg. 1 / Alg. 3 (rounding rule SR of Sec. 3.2) for gfx950.
//
// HBM-bound streaming kernel: every thread converts groups of 8 consecutive elements
// (two 16-byte loads, one 8- or 16-byte store) with one Philox block per group.
// nnz / saturated are reduced per wavefront, then per block; a one-block follow-up kernel sums
// the block partials (integer, order-independent).
#include <cstdlib>

#include <algorithm>

#include "common.hpp"
#include "context.hpp"

namespace adapt {

constexpr int kQThreads = 256;

template <typename OutT>
__device__ __forceinline__ void store8(OutT *q, const int (&v)[8]);

template <>
__device__ __forceinline__ void store8<int8_t>(int8_t *q, const int (&v)[8])
{
    uint2 o;
    o.x = (uint32_t)(v[0] & 0xff) | ((uint32_t)(v[1] & 0xff) << 8) | ((uint32_t)(v[2] & 0xff) << 16) |
          ((uint32_t)(v[3] & 0xff) << 24);
    o.y = (uint32_t)(v[4] & 0xff) | ((uint32_t)(v[5] & 0xff) << 8) | ((uint32_t)(v[6] & 0xff) << 16) |
          ((uint32_t)(v[7] & 0xff) << 24);
    *reinterpret_cast<uint2 *>(q) = o;
}
template <>
__device__ __forceinline__ void store8<int16_t>(int16_t *q, const int (&v)[8])
{
    uint4 o;
    o.x = (uint32_t)(v[0] & 0xffff) | ((uint32_t)v[1] << 16);
    o.y = (uint32_t)(v[2] & 0xffff) | ((uint32_t)v[3] << 16);
    o.z = (uint32_t)(v[4] & 0xffff) | ((uint32_t)v[5] << 16);
    o.w = (uint32_t)(v[6] & 0xffff) | ((uint32_t)v[7] << 16);
    *reinterpret_cast<uint4 *>(q) = o;
}

// Converts the elements [0, n) of one tensor; this block handles the groups
// first_group, first_group + group_stride, ...  Returns the thread's (nnz, sat) counts.
// With RANGE, lo / hi also track the smallest and largest finite input value.
template <typename OutT, bool RANGE = false>
__device__ __forceinline__ void quantize_span(const float *__restrict__ x, OutT *__restrict__ q, uint64_t n,
                                              const QuantParams p, int mode, uint64_t seed, uint64_t stream,
                                              uint64_t first_group, uint64_t group_stride, uint32_t &nnz,
                                              uint32_t &nsat, float &lo, float &hi)
{
    const uint64_t full_groups = n >> 3;
    auto convert = [&](uint64_t g, const float4 &a, const float4 &b) {
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t r[8];
        if (mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(seed, stream, g);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
        int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int s;
            c[e] = quantize_one(v[e], r[e], p, s);
            nnz += (c[e] != 0);
            nsat += s;
            if (RANGE && fabsf(v[e]) < INFINITY) { lo = fminf(lo, v[e]); hi = fmaxf(hi, v[e]); }
        }
        store8<OutT>(q + 8 * g, c);
    };
    // two groups per iteration: four 16-byte loads in flight per thread
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    uint64_t g = first_group;
    for (; g + group_stride < full_groups; g += 2 * group_stride) {
        const uint64_t h = g + group_stride;
        const float4 a0 = x4[2 * g], b0 = x4[2 * g + 1], a1 = x4[2 * h], b1 = x4[2 * h + 1];
        convert(g, a0, b0);
        convert(h, a1, b1);
    }
    if (g < full_groups) convert(g, x4[2 * g], x4[2 * g + 1]);
    // ragged tail (< 8 elements): the thread that would own group `full_groups`
    if ((n & 7) && first_group <= full_groups && (full_groups - first_group) % group_stride == 0) {
        for (uint64_t i = full_groups << 3; i < n; ++i) {
            int s;
            const int c = quantize_one(x[i], rounding_bits_of(seed, stream, i, mode), p, s);
            q[i] = (OutT)c;
            nnz += (c != 0);
            nsat += s;
            if (RANGE && fabsf(x[i]) < INFINITY) { lo = fminf(lo, x[i]); hi = fmaxf(hi, x[i]); }
        }
    }
}

__device__ __forceinline__ void block_sum2(uint32_t a, uint32_t b, uint64_t &sa, uint64_t &sb)
{
    __shared__ uint32_t part[2][kQThreads / kWave];
    a = wave_sum_u32(a);
    b = wave_sum_u32(b);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { part[0][wave] = a; part[1][wave] = b; }
    __syncthreads();
    sa = 0; sb = 0;
#pragma unroll
    for (int w = 0; w < kQThreads / kWave; ++w) { sa += part[0][w]; sb += part[1][w]; }
    __syncthreads();
}

template <typename OutT>
__global__ void __launch_bounds__(kQThreads)
quantize_kernel(const float *__restrict__ x, OutT *__restrict__ q, uint64_t n, int wl, int fl, int mode,
                uint64_t seed, uint64_t stream, uint32_t *partial /* [2][gridDim.x] or null */)
{
    const QuantParams p = make_quant_params(wl, fl);
    uint32_t nnz = 0, nsat = 0;
    // n <= 2^40 (checked by the host): per-thread and per-block counts stay below 2^32
    float lo = 0.0f, hi = 0.0f;
    quantize_span<OutT>(x, q, n, p, mode, seed, stream, (uint64_t)blockIdx.x * kQThreads + threadIdx.x,
                        (uint64_t)gridDim.x * kQThreads, nnz, nsat, lo, hi);
    if (partial == nullptr) return;
    uint64_t bn, bs;
    block_sum2(nnz, nsat, bn, bs);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = (uint32_t)bn;
        partial[gridDim.x + blockIdx.x] = (uint32_t)bs;
    }
}

__global__ void __launch_bounds__(kQThreads)
quantize_wide_kernel(const float *__restrict__ x, int32_t *__restrict__ q, uint64_t n, int wl, int fl, int mode, uint64_t seed,
                     uint64_t stream, uint32_t *partial /* [2][gridDim.x] or null */, float *range_partial = nullptr /* [2][gridDim.x] */)
{
    uint32_t nnz = 0, nsat = 0;
    float lo = INFINITY, hi = -INFINITY;                   // finite range of the input (only stored when asked for)
    const uint64_t full_groups = n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kQThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kQThreads;
    for (uint64_t g = first; g < full_groups; g += stride) {
        const float4 a = reinterpret_cast<const float4 *>(x)[2 * g], b = reinterpret_cast<const float4 *>(x)[2 * g + 1];
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        uint32_t r[8];
        if (mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(seed, stream, g);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
        int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int s;
            c[e] = quantize_one_wide(v[e], r[e], wl, fl, s);
            nnz += (c[e] != 0);
            nsat += s;
            if (fabsf(v[e]) < INFINITY) { lo = fminf(lo, v[e]); hi = fmaxf(hi, v[e]); }
        }
        reinterpret_cast<int4 *>(q)[2 * g] = make_int4(c[0], c[1], c[2], c[3]);
        reinterpret_cast<int4 *>(q)[2 * g + 1] = make_int4(c[4], c[5], c[6], c[7]);
    }
    if ((n & 7) && first == 0)
        for (uint64_t i = full_groups << 3; i < n; ++i) {
            int s;
            const int c = quantize_one_wide(x[i], rounding_bits_of(seed, stream, i, mode), wl, fl, s);
            q[i] = c;
            nnz += (c != 0);
            nsat += s;
            if (fabsf(x[i]) < INFINITY) { lo = fminf(lo, x[i]); hi = fmaxf(hi, x[i]); }
        }
    if (range_partial != nullptr) {
        __shared__ float wr[2][kQThreads / kWave];
        lo = wave_min_f32(lo);
        hi = wave_max_f32(hi);
        if ((threadIdx.x & (kWave - 1)) == 0) { wr[0][threadIdx.x / kWave] = lo; wr[1][threadIdx.x / kWave] = hi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < kQThreads / kWave; ++w) { lo = fminf(lo, wr[0][w]); hi = fmaxf(hi, wr[1][w]); }
            range_partial[blockIdx.x] = lo;
            range_partial[gridDim.x + blockIdx.x] = hi;
        }
    }
    if (partial == nullptr) return;
    uint64_t bn, bs;
    block_sum2(nnz, nsat, bn, bs);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = (uint32_t)bn;
        partial[gridDim.x + blockIdx.x] = (uint32_t)bs;
    }
}

// Sums the per-block partial counts (partial[col][block]) into out[col]: one wavefront per column,
// all loads of a lane in flight at once.  A separate launch: the kernel boundary makes the
// partials visible without fences that would force the L2 to write back the freshly quantized
// tensor.
constexpr int kSumThreads = 1024;
__global__ void __launch_bounds__(kSumThreads)
sum_partials_kernel(const uint32_t *__restrict__ partial, int nblocks, int cols, uint64_t *out0, uint64_t *out1,
                    const float *__restrict__ range_partial = nullptr /* [rcols][nblocks]: even columns min, odd max */,
                    int rcols = 0, float *range_out = nullptr)
{
    // a column per wavefront; several blocks share the columns of a batched call
    const int lane = threadIdx.x & (kWave - 1), wave = blockIdx.x * (kSumThreads / kWave) + threadIdx.x / kWave;
    const int nwaves = gridDim.x * (kSumThreads / kWave);
    // range columns are taken by the last wavefronts so that they run beside the counter columns
    for (int j = nwaves - 1 - wave; j < rcols; j += nwaves) {
        const float *col = range_partial + (size_t)j * nblocks;
        const bool is_min = (j & 1) == 0;
        float v = is_min ? INFINITY : -INFINITY;
        int b = lane;
        for (; b + 15 * kWave < nblocks; b += 16 * kWave) {        // all loads of a round in flight
            float t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) t[u] = col[b + u * kWave];
#pragma unroll
            for (int u = 0; u < 16; ++u) v = is_min ? fminf(v, t[u]) : fmaxf(v, t[u]);
        }
        for (; b < nblocks; b += kWave) v = is_min ? fminf(v, col[b]) : fmaxf(v, col[b]);
        v = is_min ? wave_min_f32(v) : wave_max_f32(v);
        if (lane == 0) range_out[j] = v;
    }
    if (out0 == nullptr) return;
    for (int j = wave; j < cols; j += nwaves) {
        const uint32_t *col = partial + (size_t)j * nblocks;
        uint64_t sum = 0;
        int b = lane;
        for (; b + 15 * kWave < nblocks; b += 16 * kWave) {
            uint32_t t[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) t[u] = col[b + u * kWave];
#pragma unroll
            for (int u = 0; u < 16; ++u) sum += t[u];
        }
        for (; b < nblocks; b += kWave) sum += col[b];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane == 0) {
            // out0 / out1: separate destinations of columns 0 and 1 (single tensor), or out0 = array
            uint64_t *dst = out1 == nullptr ? out0 + j : (j == 0 ? out0 : out1);
            if (dst) *dst = sum;
        }
    }
}

// ---- batched form: up to kMaxItems tensors per launch, descriptors in the kernel arguments ----
constexpr int kMaxItems = 64;
struct QuantBatch {
    adapt_quantize_item item[kMaxItems];
    int count;
};

// nnz / saturated of every tensor: per-block partial counts in `partial[2*count][block]`, summed
// by sum_partials_kernel (no same-address atomics, no zero-fill launch).
__global__ void __launch_bounds__(kQThreads)
quantize_batched_kernel(const QuantBatch batch, int mode, uint64_t seed, uint32_t *partial /* or null */,
                        float *range_partial /* [2*count][gridDim.x] or null */, uint64_t range_mask /* bit t: tensor t */)
{
    __shared__ uint32_t wave_part[2][kQThreads / kWave];
    __shared__ float wave_range[2][kQThreads / kWave];
    const int wave = threadIdx.x / kWave;
    // Blocks are dealt to tensors round-robin: tensor t starts at block `rot` so that small
    // tensors do not all land on block 0.
    uint32_t rot = 0;
    for (int t = 0; t < batch.count; ++t) {
        const adapt_quantize_item it = batch.item[t];
        const uint64_t groups = (it.n + 7) >> 3;
        const uint32_t blocks_needed = (uint32_t)min((uint64_t)gridDim.x, (groups + kQThreads - 1) / kQThreads);
        const uint32_t slot = (blockIdx.x + gridDim.x - rot % gridDim.x) % gridDim.x;
        rot += blocks_needed;
        uint32_t nnz = 0, nsat = 0;
        float lo = INFINITY, hi = -INFINITY;
        if (slot < blocks_needed) {
            const QuantParams p = make_quant_params(it.wl, it.fl);
            const uint64_t first = (uint64_t)slot * kQThreads + threadIdx.x;
            const uint64_t stride = (uint64_t)blocks_needed * kQThreads;
            if (range_partial != nullptr && ((range_mask >> t) & 1)) {
                if (it.wl <= 8)
                    quantize_span<int8_t, true>(it.x, (int8_t *)it.q, it.n, p, mode, seed, it.stream, first, stride, nnz, nsat, lo, hi);
                else
                    quantize_span<int16_t, true>(it.x, (int16_t *)it.q, it.n, p, mode, seed, it.stream, first, stride, nnz, nsat, lo, hi);
            } else {
                if (it.wl <= 8)
                    quantize_span<int8_t>(it.x, (int8_t *)it.q, it.n, p, mode, seed, it.stream, first, stride, nnz, nsat, lo, hi);
                else
                    quantize_span<int16_t>(it.x, (int16_t *)it.q, it.n, p, mode, seed, it.stream, first, stride, nnz, nsat, lo, hi);
            }
        }
        // one barrier pair per tensor: counters and (for the tensors that asked for it) the range
        const bool want_range = range_partial != nullptr && ((range_mask >> t) & 1);
        if (partial != nullptr || want_range) {
            const bool lead = (threadIdx.x & (kWave - 1)) == 0;
            if (partial != nullptr) {
                nnz = wave_sum_u32(nnz);
                nsat = wave_sum_u32(nsat);
                if (lead) { wave_part[0][wave] = nnz; wave_part[1][wave] = nsat; }
            }
            if (want_range) {
                lo = wave_min_f32(lo);
                hi = wave_max_f32(hi);
                if (lead) { wave_range[0][wave] = lo; wave_range[1][wave] = hi; }
            }
            __syncthreads();
            if (threadIdx.x < 2 && partial != nullptr) {
                uint32_t v = 0;
                for (int w = 0; w < kQThreads / kWave; ++w) v += wave_part[threadIdx.x][w];
                partial[(size_t)(2 * t + threadIdx.x) * gridDim.x + blockIdx.x] = v;
            }
            if (threadIdx.x >= kWave && threadIdx.x < kWave + 2 && want_range) {      // a second wavefront: runs beside the first
                const int m = threadIdx.x - kWave;
                float v = wave_range[m][0];
                for (int w = 1; w < kQThreads / kWave; ++w) v = m == 0 ? fminf(v, wave_range[0][w]) : fmaxf(v, wave_range[1][w]);
                range_partial[(size_t)(2 * t + m) * gridDim.x + blockIdx.x] = v;
            }
            __syncthreads();
        }
        if (range_partial != nullptr && !want_range && threadIdx.x < 2)      // not asked for: the neutral pair
            range_partial[(size_t)(2 * t + threadIdx.x) * gridDim.x + blockIdx.x] = threadIdx.x == 0 ? INFINITY : -INFINITY;
    }
}

static int grid_for(const adapt_ctx *ctx, uint64_t n)
{
    const uint64_t groups = (n + 7) >> 3;
    uint64_t blocks = (groups + kQThreads - 1) / kQThreads;
    const uint64_t cap = (uint64_t)ctx->num_cu * 8;
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    return (int)blocks;
}

size_t ws_need_quantize(int num_cu, uint64_t n)
{
    adapt_ctx c = {};
    c.num_cu = num_cu;
    return (((size_t)grid_for(&c, n) * 8 + 255) & ~(size_t)255) + 16;      // per-block counters, and the dummy slot
}

// the batched call takes at most 4 blocks per CU; counter and range partials per block and tensor
size_t ws_need_quantize_batched(int num_cu, int count)
{
    const size_t per = std::min(std::max(count, 1), kMaxItems);
    return 2 * (((size_t)num_cu * 4 * 2 * per * sizeof(uint32_t) + 255) & ~(size_t)255);
}

}  // namespace adapt

using namespace adapt;

// adapt_quantize with the per-block counter partials at `base` (room for `room` bytes): the context's workspace, or
// the static array of the entry point that allocates nothing
static int quantize_on(adapt_ctx *ctx, const float *x, size_t n, adapt_fmt fmt, adapt_rng rng, void *q, uint64_t *nnz,
                       uint64_t *saturated, char *base, size_t room)
{
    if (!ctx || !fmt_ok_wide(fmt) || (rng.mode != ADAPT_SR && rng.mode != ADAPT_RN_HALF_UP)) return ADAPT_EINVAL;
    if (n > 0 && (!x || !q || !aligned16(x) || !aligned16(q))) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if ((nnz && ((uintptr_t)nnz & 7)) || (saturated && ((uintptr_t)saturated & 7))) return ADAPT_EINVAL;
    const int grid = grid_for(ctx, n);
    const bool count = nnz || saturated;
    const size_t part_bytes = ((size_t)grid * 8 + 255) & ~(size_t)255;
    if (part_bytes + 16 > room) return ADAPT_EWORKSPACE;
    uint32_t *partial = count ? reinterpret_cast<uint32_t *>(base) : nullptr;
    if (fmt.wl > 16)
        hipLaunchKernelGGL(quantize_wide_kernel, dim3(grid), dim3(kQThreads), 0, ctx->stream, x, (int32_t *)q, (uint64_t)n, fmt.wl,
                           fmt.fl, rng.mode, rng.seed, rng.stream, partial);
    else if (fmt.wl <= 8)
        hipLaunchKernelGGL(quantize_kernel<int8_t>, dim3(grid), dim3(kQThreads), 0, ctx->stream, x, (int8_t *)q,
                           (uint64_t)n, fmt.wl, fmt.fl, rng.mode, rng.seed, rng.stream, partial);
    else
        hipLaunchKernelGGL(quantize_kernel<int16_t>, dim3(grid), dim3(kQThreads), 0, ctx->stream, x, (int16_t *)q,
                           (uint64_t)n, fmt.wl, fmt.fl, rng.mode, rng.seed, rng.stream, partial);
    if (count) {
        // out1 != null selects the two-destination form; a null destination is redirected to a dummy slot
        uint64_t *dummy = reinterpret_cast<uint64_t *>(base + part_bytes);
        hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(kSumThreads), 0, ctx->stream, partial, grid, 2,
                           nnz ? nnz : dummy, saturated ? saturated : dummy + 1);
    }
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_quantize(adapt_ctx *ctx, const float *x, size_t n, adapt_fmt fmt, adapt_rng rng, void *q,
                              uint64_t *nnz, uint64_t *saturated)
{
    if (!ctx) return ADAPT_EINVAL;
    return quantize_on(ctx, x, n, fmt, rng, q, nnz, saturated, scratch(ctx), scratch_bytes(ctx));
}

// ---- the entry point that allocates nothing ------------------------------------------------------------------
// Its scratch (the per-block counter partials and the dummy slot) is a file-scope device array: every GPU the
// library runs on holds its own copy at its own address for the life of the process.  The array's name is a
// host-side stand-in, not a device address; host code uses the address hipGetSymbolAddress returns for the
// device that is current, taken once per context at creation and kept in the context.
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

namespace adapt {
hipError_t static_scratch_address(void **ptr)
{
    *ptr = nullptr;
    return hipGetSymbolAddress(ptr, HIP_SYMBOL(g_static_scratch));
}
}  // namespace adapt

extern "C" int adapt_quantize_noalloc(adapt_ctx *ctx, const float *x, size_t n, adapt_fmt fmt, adapt_rng rng, void *q,
                                      uint64_t *nnz, uint64_t *saturated)
{
    if (!ctx) return ADAPT_EINVAL;
    if (!ctx->static_scratch) return ADAPT_EHIP;      // the address could not be taken when the context was created
    // at most 8 blocks per compute unit, 8 bytes each: more than kStaticScratchBytes only on a device with more
    // than 4,000 compute units, which quantize_on reports as ADAPT_EWORKSPACE
    return quantize_on(ctx, x, n, fmt, rng, q, nnz, saturated, static_cast<char *>(ctx->static_scratch), kStaticScratchBytes);
}

extern "C" int adapt_quantize_batched(adapt_ctx *ctx, const adapt_quantize_item *items, int count, int mode,
                                      uint64_t seed, uint64_t *counters)
{
    return adapt_quantize_batched_ranges(ctx, items, count, mode, seed, counters, nullptr, 0);
}

extern "C" int adapt_quantize_batched_ranges(adapt_ctx *ctx, const adapt_quantize_item *items, int count, int mode,
                                             uint64_t seed, uint64_t *counters, float *ranges, uint64_t range_mask)
{
    if (ranges && count > 64) return ADAPT_EUNSUPPORTED;      // one mask bit per tensor
    if (!ctx || count < 0 || (count > 0 && !items)) return ADAPT_EINVAL;
    if (mode != ADAPT_SR && mode != ADAPT_RN_HALF_UP) return ADAPT_EINVAL;
    if ((counters && ((uintptr_t)counters & 7)) || (ranges && ((uintptr_t)ranges & 3))) return ADAPT_EINVAL;
    for (int t = 0; t < count; ++t) {
        const adapt_quantize_item &it = items[t];
        if (!fmt_ok_wide(adapt_fmt{it.wl, it.fl}) || it.n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
        if (it.n > 0 && (!it.x || !it.q || !aligned16(it.x) || !aligned16(it.q))) return ADAPT_EINVAL;
    }
    if (count == 0) return ADAPT_OK;
    for (int base = 0; base < count; base += kMaxItems) {
        QuantBatch batch;
        batch.count = count - base < kMaxItems ? count - base : kMaxItems;
        uint64_t total_blocks = 0;
        for (int t = 0; t < batch.count; ++t) {
            batch.item[t] = items[base + t];
            if (items[base + t].wl > 16) {             // int32 codes: a launch of its own below; an empty placeholder here
                batch.item[t].n = 0;
                batch.item[t].wl = 8;
            }
            total_blocks += (((batch.item[t].n + 7) >> 3) + kQThreads - 1) / kQThreads;
        }
        uint64_t grid = total_blocks;
        uint64_t cap = (uint64_t)ctx->num_cu * 4;
        if (grid > cap) grid = cap;
        if (grid == 0) grid = 1;     // still writes the (zero) counters
        const size_t part_bytes = (grid * 2 * batch.count * sizeof(uint32_t) + 255) & ~(size_t)255;
        if (2 * part_bytes > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
        uint32_t *partial = counters ? reinterpret_cast<uint32_t *>(scratch(ctx)) : nullptr;
        float *range_partial = ranges ? reinterpret_cast<float *>(scratch(ctx) + part_bytes) : nullptr;
        hipLaunchKernelGGL(quantize_batched_kernel, dim3((unsigned)grid), dim3(kQThreads), 0, ctx->stream, batch, mode,
                           seed, partial, range_partial, range_mask >> base);
        // one wavefront per column: enough blocks for all the columns of the batch to run side by side
        const int sum_cols = (counters ? 2 * batch.count : 0) + (ranges ? 2 * batch.count : 0);
        const int sum_blocks = std::min(std::max((sum_cols + kSumThreads / kWave - 1) / (kSumThreads / kWave), 1), 16);
        if (counters || ranges)
            hipLaunchKernelGGL(sum_partials_kernel, dim3(sum_blocks), dim3(kSumThreads), 0, ctx->stream, partial, (int)grid,
                               2 * batch.count, counters ? counters + 2 * base : (uint64_t *)nullptr, (uint64_t *)nullptr,
                               range_partial, ranges ? 2 * batch.count : 0, ranges ? ranges + 2 * base : (float *)nullptr);
    }
    // tensors above 16 bits, one after the other; their counters and ranges replace the placeholders' zeros
    for (int t = 0; t < count; ++t) {
        const adapt_quantize_item &it = items[t];
        if (it.wl <= 16) continue;
        const int grid = grid_for(ctx, it.n);
        const size_t part_bytes = ((size_t)grid * 2 * sizeof(uint32_t) + 255) & ~(size_t)255;
        if (2 * part_bytes > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
        const bool want_range = ranges && ((range_mask >> t) & 1);
        uint32_t *partial = counters ? reinterpret_cast<uint32_t *>(scratch(ctx)) : nullptr;
        float *range_partial = want_range ? reinterpret_cast<float *>(scratch(ctx) + part_bytes) : nullptr;
        hipLaunchKernelGGL(quantize_wide_kernel, dim3(grid), dim3(kQThreads), 0, ctx->stream, it.x, static_cast<int32_t *>(it.q), it.n,
                           (int)it.wl, (int)it.fl, mode, seed, it.stream, partial, range_partial);
        if (counters || want_range)
            hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(kSumThreads), 0, ctx->stream, partial, grid, counters ? 2 : 0,
                               counters ? counters + 2 * t : (uint64_t *)nullptr, (uint64_t *)nullptr, range_partial,
                               want_range ? 2 : 0, want_range ? ranges + 2 * t : (float *)nullptr);
    }
    return hip_status(ctx, hipGetLastError());
}
