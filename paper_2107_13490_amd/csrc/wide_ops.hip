// Element-wise steps of the chained training step for word lengths 17..32 (Sec. 3.3 bounds the precision that
// PushUp may ask for at 32 bits): the fitting requantization of 128-bit accumulators (and of any accumulators to
// codes above 16 bits).  The rules are those of the narrow kernels, evaluated in 128-bit integers; one element per
// thread and iteration, bound by HBM traffic (4-16 B read, 1-4 B written per element) at sizes where that matters.
#include <algorithm>

#include "common.hpp"
#include "context.hpp"
#include "fit.hpp"
#include "wide.hpp"

namespace adapt {

constexpr int kWoThreads = 256;

// part[block] = largest bit length of |acc[i]|; block 0 also clears the sum of squares that the next pass accumulates
template <typename AccT>
__global__ void __launch_bounds__(kWoThreads)
bitlen_max_kernel(const AccT *__restrict__ acc, const uint64_t n, uint64_t *__restrict__ part, unsigned long long *sumsq, int sumsq_words)
{
    uint64_t m = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kWoThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWoThreads) {
        const uint64_t b = (uint64_t)bit_length_128((i128)acc[i]);
        m = b > m ? b : m;
    }
    __shared__ uint64_t sm[kWoThreads / kWave];
    m = block_max_u64(m, sm, kWoThreads / kWave);
    if (threadIdx.x == 0) {
        part[blockIdx.x] = m;
        if (blockIdx.x == 0 && sumsq)
            for (int w = 0; w < sumsq_words; ++w) sumsq[w] = 0;
    }
}

// codes = requantize(acc, shift), shift = max(0, largest bit length - (wl - 1)); every block derives the shift from
// the partial maxima itself.  sumsq: one word (wl <= 16) or a 128-bit sum in two words, low first (wl > 16).
template <typename AccT, typename OutT>
__global__ void __launch_bounds__(kWoThreads) requant_fit_wide_kernel(const FitArgs a, int sumsq_words)
{
    __shared__ uint64_t sm[kWoThreads / kWave];
    __shared__ unsigned long long ss_sm[kWoThreads / kWave][2];
    uint64_t m = 0;
    for (int i = threadIdx.x; i < a.nparts; i += kWoThreads) m = a.part[i] > m ? a.part[i] : m;
    m = block_max_u64(m, sm, kWoThreads / kWave);
    const int shift = max(0, (int)m - (a.wl - 1));
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (a.shift_out) *a.shift_out = shift;
        if (a.e_out) *a.e_out = (a.e_in ? *a.e_in : 0) + a.e_add - shift;
    }
    const AccT *acc = static_cast<const AccT *>(a.acc);
    OutT *q = static_cast<OutT *>(a.q);
    u128 ss = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kWoThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kWoThreads) {
        const int c = requantize_wide_one((i128)acc[i], shift, a.wl, 0, rounding_bits_of(a.seed, a.stream, i, a.mode));
        q[i] = (OutT)c;
        ss += (u128)((long long)c * (long long)c);
    }
    if (a.sumsq) {
        ss = wave_sum_u128(ss);
        const int wave = threadIdx.x / kWave;
        if ((threadIdx.x & (kWave - 1)) == 0) { ss_sm[wave][0] = (unsigned long long)ss; ss_sm[wave][1] = (unsigned long long)(ss >> 64); }
        __syncthreads();
        if (threadIdx.x == 0) {
            u128 t = 0;
            for (int i = 0; i < kWoThreads / kWave; ++i) t += ((u128)ss_sm[i][1] << 64) | ss_sm[i][0];
            if (sumsq_words == 2) atomic_add_u128(a.sumsq, t);
            else if (t) atomicAdd(a.sumsq, (unsigned long long)t);
        }
    }
}

int requantize_fit_wide(adapt_ctx *ctx, const void *acc, int acc_bits, size_t n, int wl, adapt_rng rng, void *q, int32_t *shift,
                        uint64_t *sumsq, const long long *e_in, long long e_add, long long *e_out)
{
    if (!ctx || (acc_bits != 32 && acc_bits != 64 && acc_bits != 128) || wl < 2 || wl > 32) return ADAPT_EINVAL;
    if (rng.mode != ADAPT_SR && rng.mode != ADAPT_RN_HALF_UP) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if ((shift && ((uintptr_t)shift & 3)) || (sumsq && ((uintptr_t)sumsq & 7))) return ADAPT_EINVAL;
    if (n > 0 && (!acc || !q || !aligned16(acc) || !aligned16(q))) return ADAPT_EINVAL;
    const int grid = (int)std::min<uint64_t>(std::max<uint64_t>(((uint64_t)n + kWoThreads - 1) / kWoThreads, 1), (uint64_t)ctx->num_cu * 4);
    if ((size_t)grid * 8 > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    uint64_t *part = reinterpret_cast<uint64_t *>(scratch(ctx));
    unsigned long long *ss = reinterpret_cast<unsigned long long *>(sumsq);
    const int words = wl > 16 ? 2 : 1;
    FitArgs a;
    a.acc = acc; a.q = q; a.part = part; a.nparts = grid; a.n = n; a.wl = wl; a.mode = rng.mode; a.seed = rng.seed;
    a.stream = rng.stream; a.shift_out = shift; a.sumsq = ss; a.e_in = e_in; a.e_add = e_add; a.e_out = e_out;
    const dim3 g(grid), t(kWoThreads);
    if (acc_bits == 32) hipLaunchKernelGGL(bitlen_max_kernel<int32_t>, g, t, 0, ctx->stream, (const int32_t *)acc, (uint64_t)n, part, ss, words);
    else if (acc_bits == 64) hipLaunchKernelGGL(bitlen_max_kernel<int64_t>, g, t, 0, ctx->stream, (const int64_t *)acc, (uint64_t)n, part, ss, words);
    else hipLaunchKernelGGL(bitlen_max_kernel<i128>, g, t, 0, ctx->stream, (const i128 *)acc, (uint64_t)n, part, ss, words);
#define ADAPT_FITW(A, O) hipLaunchKernelGGL((requant_fit_wide_kernel<A, O>), g, t, 0, ctx->stream, a, words)
    if (wl > 16) {
        if (acc_bits == 32) ADAPT_FITW(int32_t, int32_t);
        else if (acc_bits == 64) ADAPT_FITW(int64_t, int32_t);
        else ADAPT_FITW(i128, int32_t);
    } else if (wl > 8) {
        ADAPT_FITW(i128, int16_t);
    } else {
        ADAPT_FITW(i128, int8_t);
    }
#undef ADAPT_FITW
    return hip_status(ctx, hipGetLastError());
}

}  // namespace adapt
