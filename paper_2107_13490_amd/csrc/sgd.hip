// Master-weight update of AdaPT-SGD fused with the re-quantization that follows it (Alg. 1:
// the backward-pass line and the per-layer Quantize loop; gradient normalisation of Sec. 3.3
// "Dealing with Fixed-Points Limited Range"; L1 / L2 terms of Sec. 3.4 "Inducing Sparsity").
//
// One pass over the layer: read the fp32 master weight and the gradient code, apply
//     d  = fma(l2, w, l1 * sign(w));   w1 = fma(-step, c, w);   w' = fma(-lr, d, w1)
// (three explicit fp32 fused multiply-adds: the order is part of the contract), write w' back,
// quantize it to <WL,FL> with the Sec. 3.2 rule, count non-zero and saturated codes and track the
// finite range of w' for the next precision search.  10-12 bytes of HBM traffic per element
// instead of the 18 of separate update, range and quantize passes.
#include <algorithm>
#include <type_traits>

#include "common.hpp"
#include "context.hpp"
#include "update_batch.hpp"
#include "wide.hpp"

namespace adapt {

constexpr int kSgdThreads = 256;
constexpr int kSgdFinalThreads = 1024;

struct SgdArgs {
    float *w;
    const void *g;
    void *q;
    const uint64_t *g_sumsq;     // device: sum of squared gradient codes (two words, low first, for int32 codes), or null
    uint64_t n;
    double lr;
    float l1, l2;
    int fl_g;
    int wl, fl, mode;
    uint64_t seed, stream;
};

__device__ __forceinline__ float sgd_one(float w, int c, float step, float lr, float l1, float l2)
{
    const float s = w > 0.0f ? l1 : (w < 0.0f ? -l1 : 0.0f);
    const float d = __builtin_fmaf(l2, w, s);
    const float w1 = __builtin_fmaf(-step, (float)c, w);
    return __builtin_fmaf(-lr, d, w1);
}

// One tensor's share of a block: groups first, first + stride, ...; the thread with first == 0 also takes the ragged
// tail.  Adds to the caller's counters and range.
template <typename GT, typename OutT>
__device__ __forceinline__ void sgd_span(const SgdArgs &a, uint64_t first, uint64_t stride, uint32_t &nnz, uint32_t &nsat, float &lo,
                                         float &hi)
{
    float step;
    if (a.g_sumsq != nullptr) {
        // int32 codes: the sum of squares has 128 bits; its nearest double enters the quotient
        const double s = std::is_same<GT, int32_t>::value ? u128_to_double(a.g_sumsq[0], a.g_sumsq[1]) : (double)a.g_sumsq[0];
        step = s != 0.0 ? (float)(a.lr / sqrt(s)) : 0.0f;
    } else {
        step = (float)ldexp(a.lr, -a.fl_g);
    }
    const float lr = (float)a.lr;
    const QuantParams p = make_quant_params(std::is_same<OutT, int32_t>::value ? 8 : a.wl, a.fl);      // unused for int32 codes
    const GT *g = static_cast<const GT *>(a.g);
    OutT *q = static_cast<OutT *>(a.q);
    float4 *w4 = reinterpret_cast<float4 *>(a.w);

    auto one = [&](float w, int c, uint32_t r, int &code) {
        const float wn = sgd_one(w, c, step, lr, a.l1, a.l2);
        int s;
        if (std::is_same<OutT, int32_t>::value) code = quantize_one_wide(wn, r, a.wl, a.fl, s);
        else code = quantize_one(wn, r, p, s);
        nnz += (code != 0);
        nsat += s;
        if (fabsf(wn) < INFINITY) { lo = fminf(lo, wn); hi = fmaxf(hi, wn); }
        return wn;
    };

    const uint64_t full_groups = a.n >> 3;
    for (uint64_t grp = first; grp < full_groups; grp += stride) {
        const float4 x0 = w4[2 * grp], x1 = w4[2 * grp + 1];
        int c[8];
        load_codes8<GT>(g, grp, c);
        uint32_t r[8];
        if (a.mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(a.seed, a.stream, grp);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
        const float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        float o[8];
        int code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = one(v[e], c[e], r[e], code[e]);
        w4[2 * grp] = make_float4(o[0], o[1], o[2], o[3]);
        w4[2 * grp + 1] = make_float4(o[4], o[5], o[6], o[7]);
        store_codes8<OutT>(q, grp, code);
    }
    if ((a.n & 7) && first == 0) {                 // ragged tail (< 8 elements)
        for (uint64_t i = full_groups << 3; i < a.n; ++i) {
            int code;
            a.w[i] = one(a.w[i], (int)g[i], rounding_bits_of(a.seed, a.stream, i, a.mode), code);
            q[i] = (OutT)code;
        }
    }
}

// The block's totals of the four per-thread values: counts[block] = nnz, counts[nblocks + block] = saturated,
// range[2 block] = min, range[2 block + 1] = max (one barrier; the shared arrays may be reused after the next one)
__device__ __forceinline__ void sgd_block_partials(uint32_t nnz, uint32_t nsat, float lo, float hi, uint32_t *counts, float *range,
                                                   uint32_t block, uint32_t nblocks, uint32_t (*sc)[kSgdThreads / kWave],
                                                   float (*sr)[kSgdThreads / kWave])
{
    nnz = wave_sum_u32(nnz);
    nsat = wave_sum_u32(nsat);
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { sc[0][wave] = nnz; sc[1][wave] = nsat; sr[0][wave] = lo; sr[1][wave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 1; i < kSgdThreads / kWave; ++i) {
            nnz += sc[0][i]; nsat += sc[1][i];
            lo = fminf(lo, sr[0][i]); hi = fmaxf(hi, sr[1][i]);
        }
        counts[block] = nnz;
        counts[nblocks + block] = nsat;
        range[2 * block] = lo;
        range[2 * block + 1] = hi;
    }
}

// counts[2][grid] (nnz, saturated) and range[grid][2] (min, max of the finite new weights)
template <typename GT, typename OutT>
__global__ void __launch_bounds__(kSgdThreads)
sgd_update_quantize_kernel(const SgdArgs a, uint32_t *counts, float *range)
{
    __shared__ uint32_t sc[2][kSgdThreads / kWave];
    __shared__ float sr[2][kSgdThreads / kWave];
    uint32_t nnz = 0, nsat = 0;
    float lo = INFINITY, hi = -INFINITY;
    sgd_span<GT, OutT>(a, (uint64_t)blockIdx.x * kSgdThreads + threadIdx.x, (uint64_t)gridDim.x * kSgdThreads, nnz, nsat, lo, hi);
    sgd_block_partials(nnz, nsat, lo, hi, counts, range, blockIdx.x, gridDim.x, sc, sr);
}

// Several layers per launch.  Blocks are dealt to the tensors round-robin, tensor t starting where tensor t-1 ended,
// so that small tensors do not all land on block 0; every block writes its partials of every tensor (neutral values
// where it had no share), tensor t's at counts + 2 t grid and range + 2 t grid, laid out as above.
struct SgdBatch {
    SgdBatchItem item[kUpdateMaxItems];
    int count;
};

__global__ void __launch_bounds__(kSgdThreads)
sgd_update_batch_kernel(const SgdBatch batch, double lr, float l1, float l2, int mode, uint32_t *counts, float *range)
{
    __shared__ uint32_t sc[2][kSgdThreads / kWave];
    __shared__ float sr[2][kSgdThreads / kWave];
    uint32_t rot = 0;
    for (int t = 0; t < batch.count; ++t) {
        const SgdBatchItem &it = batch.item[t];
        const uint64_t groups = (it.n + 7) >> 3;
        const uint32_t blocks_needed = (uint32_t)min((uint64_t)gridDim.x, max((groups + kSgdThreads - 1) / kSgdThreads, (uint64_t)1));
        const uint32_t slot = (blockIdx.x + gridDim.x - rot % gridDim.x) % gridDim.x;
        rot += blocks_needed;
        uint32_t nnz = 0, nsat = 0;
        float lo = INFINITY, hi = -INFINITY;
        if (slot < blocks_needed) {
            SgdArgs a;
            a.w = it.w; a.g = it.g; a.q = it.q; a.g_sumsq = it.g_sumsq; a.n = it.n; a.lr = lr; a.l1 = l1; a.l2 = l2;
            a.fl_g = it.fl_g; a.wl = it.wl; a.fl = it.fl; a.mode = mode; a.seed = it.seed; a.stream = it.stream;
            const uint64_t first = (uint64_t)slot * kSgdThreads + threadIdx.x, stride = (uint64_t)blocks_needed * kSgdThreads;
            if (it.es_g == 1) {
                if (it.es_q == 1) sgd_span<int8_t, int8_t>(a, first, stride, nnz, nsat, lo, hi);
                else sgd_span<int8_t, int16_t>(a, first, stride, nnz, nsat, lo, hi);
            } else {
                if (it.es_q == 1) sgd_span<int16_t, int8_t>(a, first, stride, nnz, nsat, lo, hi);
                else sgd_span<int16_t, int16_t>(a, first, stride, nnz, nsat, lo, hi);
            }
        }
        sgd_block_partials(nnz, nsat, lo, hi, counts + (size_t)2 * t * gridDim.x, range + (size_t)2 * t * gridDim.x, blockIdx.x,
                           gridDim.x, sc, sr);
        __syncthreads();                           // the shared arrays are free again
    }
}

// one block: totals of the block partials
__device__ __forceinline__ void sgd_final_body(const uint32_t *__restrict__ counts, const float *__restrict__ range, int nblocks,
                                               uint64_t *counters, float *range_out)
{
    __shared__ uint64_t sc[2][kSgdFinalThreads / kWave];
    __shared__ float sr[2][kSgdFinalThreads / kWave];
    uint64_t nnz = 0, nsat = 0;
    float lo = INFINITY, hi = -INFINITY;
    for (int b = threadIdx.x; b < nblocks; b += kSgdFinalThreads) {
        nnz += counts[b];
        nsat += counts[nblocks + b];
        lo = fminf(lo, range[2 * b]);
        hi = fmaxf(hi, range[2 * b + 1]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        nnz += __shfl_xor((unsigned long long)nnz, off, 64);
        nsat += __shfl_xor((unsigned long long)nsat, off, 64);
    }
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { sc[0][wave] = nnz; sc[1][wave] = nsat; sr[0][wave] = lo; sr[1][wave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kSgdFinalThreads / kWave; ++i) {
            nnz += sc[0][i]; nsat += sc[1][i];
            lo = fminf(lo, sr[0][i]); hi = fmaxf(hi, sr[1][i]);
        }
        if (counters) { counters[0] = nnz; counters[1] = nsat; }
        if (range_out) { range_out[0] = lo; range_out[1] = hi; }
    }
}

__global__ void __launch_bounds__(kSgdFinalThreads)
sgd_final_kernel(const uint32_t *__restrict__ counts, const float *__restrict__ range, int nblocks, uint64_t *counters,
                 float *range_out)
{
    sgd_final_body(counts, range, nblocks, counters, range_out);
}

// block t: the totals of tensor t of a batched launch
__global__ void __launch_bounds__(kSgdFinalThreads)
sgd_final_batch_kernel(const SgdBatch batch, const uint32_t *__restrict__ counts, const float *__restrict__ range, int nblocks)
{
    const SgdBatchItem &it = batch.item[blockIdx.x];
    if (!it.counters && !it.range) return;
    sgd_final_body(counts + (size_t)2 * blockIdx.x * nblocks, range + (size_t)2 * blockIdx.x * nblocks, nblocks, it.counters, it.range);
}

size_t ws_need_sgd_update(int num_cu, uint64_t n)
{
    const uint64_t groups = (n + 7) >> 3;
    const uint64_t blocks = std::min<uint64_t>(std::max<uint64_t>((groups + kSgdThreads - 1) / kSgdThreads, 1), (uint64_t)num_cu * 8);
    return (((size_t)blocks * 8 + 255) & ~(size_t)255) + (size_t)blocks * 8;
}

int sgd_update_batch(adapt_ctx *ctx, const SgdBatchItem *items, int count, adapt_sgd_params opt, int mode)
{
    if (!ctx || count < 0 || (count > 0 && !items) || (mode != ADAPT_SR && mode != ADAPT_RN_HALF_UP)) return ADAPT_EINVAL;
    if (!(opt.lr == opt.lr) || !(opt.l1 == opt.l1) || !(opt.l2 == opt.l2)) return ADAPT_EINVAL;
    for (int t = 0; t < count; ++t) {
        const SgdBatchItem &it = items[t];
        if ((it.es_g != 1 && it.es_g != 2) || it.wl < 2 || it.wl > 16 || it.es_q != (it.wl <= 8 ? 1 : 2) || it.fl < 0 || it.fl > 31 ||
            it.n > ((uint64_t)1 << 40))
            return ADAPT_EINVAL;
        if (it.n > 0 && (!it.w || !it.g || !it.q || !aligned16(it.w) || !aligned16(it.g) || !aligned16(it.q))) return ADAPT_EINVAL;
        if (((uintptr_t)it.counters & 7) || ((uintptr_t)it.g_sumsq & 7) || ((uintptr_t)it.range & 3)) return ADAPT_EINVAL;
    }
    // the grid of every launch, and the scratch of the largest, before anything is enqueued
    const uint64_t cap = (uint64_t)ctx->num_cu * 4;
    size_t need = 0;
    for (int base = 0; base < count; base += kUpdateMaxItems) {
        const int m = std::min(count - base, kUpdateMaxItems);
        uint64_t blocks = 0;
        for (int t = 0; t < m; ++t) blocks += std::max<uint64_t>((((items[base + t].n + 7) >> 3) + kSgdThreads - 1) / kSgdThreads, 1);
        const size_t grid = (size_t)std::min(blocks, cap);
        need = std::max(need, 2 * (((size_t)2 * m * grid * 4 + 255) & ~(size_t)255));
    }
    if (need > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    for (int base = 0; base < count; base += kUpdateMaxItems) {
        SgdBatch batch;
        batch.count = std::min(count - base, kUpdateMaxItems);
        uint64_t blocks = 0;
        for (int t = 0; t < batch.count; ++t) {
            batch.item[t] = items[base + t];
            blocks += std::max<uint64_t>((((items[base + t].n + 7) >> 3) + kSgdThreads - 1) / kSgdThreads, 1);
        }
        const int grid = (int)std::min(blocks, cap);
        const size_t part = ((size_t)2 * batch.count * grid * 4 + 255) & ~(size_t)255;
        uint32_t *counts = reinterpret_cast<uint32_t *>(scratch(ctx));
        float *range = reinterpret_cast<float *>(scratch(ctx) + part);
        hipLaunchKernelGGL(sgd_update_batch_kernel, dim3(grid), dim3(kSgdThreads), 0, ctx->stream, batch, opt.lr, (float)opt.l1,
                           (float)opt.l2, mode, counts, range);
        hipLaunchKernelGGL(sgd_final_batch_kernel, dim3(batch.count), dim3(kSgdFinalThreads), 0, ctx->stream, batch, counts, range, grid);
    }
    return hip_status(ctx, hipGetLastError());
}

}  // namespace adapt

using namespace adapt;

extern "C" int adapt_sgd_update_quantize(adapt_ctx *ctx, float *w, size_t n, const void *g, adapt_fmt fg,
                                         const uint64_t *g_sumsq, adapt_sgd_params opt, adapt_fmt fq, adapt_rng rng,
                                         void *q, uint64_t *counters, float *range)
{
    if (!ctx || !fmt_ok_wide(fg) || !fmt_ok_wide(fq) || (rng.mode != ADAPT_SR && rng.mode != ADAPT_RN_HALF_UP)) return ADAPT_EINVAL;
    if (n > 0 && (!w || !g || !q || !aligned16(w) || !aligned16(g) || !aligned16(q))) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if ((counters && ((uintptr_t)counters & 7)) || (g_sumsq && ((uintptr_t)g_sumsq & 7)) || (range && ((uintptr_t)range & 3)))
        return ADAPT_EINVAL;
    if (!(opt.lr == opt.lr) || !(opt.l1 == opt.l1) || !(opt.l2 == opt.l2)) return ADAPT_EINVAL;
    const uint64_t groups = ((uint64_t)n + 7) >> 3;
    uint64_t blocks = (groups + kSgdThreads - 1) / kSgdThreads;
    blocks = std::min<uint64_t>(std::max<uint64_t>(blocks, 1), (uint64_t)ctx->num_cu * 8);
    const int grid = (int)blocks;
    const size_t counts_bytes = ((size_t)grid * 8 + 255) & ~(size_t)255;
    if (counts_bytes + (size_t)grid * 8 > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    uint32_t *counts = reinterpret_cast<uint32_t *>(scratch(ctx));
    float *rpart = reinterpret_cast<float *>(scratch(ctx) + counts_bytes);
    SgdArgs a;
    a.w = w; a.g = g; a.q = q; a.g_sumsq = g_sumsq; a.n = n; a.lr = opt.lr; a.l1 = (float)opt.l1; a.l2 = (float)opt.l2;
    a.fl_g = fg.fl; a.wl = fq.wl; a.fl = fq.fl; a.mode = rng.mode; a.seed = rng.seed; a.stream = rng.stream;
#define ADAPT_SGD(G, Q) hipLaunchKernelGGL((sgd_update_quantize_kernel<G, Q>), dim3(grid), dim3(kSgdThreads), 0, ctx->stream, a, counts, rpart)
    switch (storage_bytes(fg) * 8 + storage_bytes(fq)) {
    case 1 * 8 + 1: ADAPT_SGD(int8_t, int8_t); break;
    case 1 * 8 + 2: ADAPT_SGD(int8_t, int16_t); break;
    case 1 * 8 + 4: ADAPT_SGD(int8_t, int32_t); break;
    case 2 * 8 + 1: ADAPT_SGD(int16_t, int8_t); break;
    case 2 * 8 + 2: ADAPT_SGD(int16_t, int16_t); break;
    case 2 * 8 + 4: ADAPT_SGD(int16_t, int32_t); break;
    case 4 * 8 + 1: ADAPT_SGD(int32_t, int8_t); break;
    case 4 * 8 + 2: ADAPT_SGD(int32_t, int16_t); break;
    default: ADAPT_SGD(int32_t, int32_t); break;
    }
#undef ADAPT_SGD
    if (counters || range)
        hipLaunchKernelGGL(sgd_final_kernel, dim3(1), dim3(kSgdFinalThreads), 0, ctx->stream, counts, rpart, grid, counters, range);
    return hip_status(ctx, hipGetLastError());
}
