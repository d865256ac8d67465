// PushDown (Sec. 3.3 "The PushDown Operation", Alg. 3): KL divergence between the binned
// distribution of a tensor and of its <WL_c, FL_c> quantizations, for all candidate word
// lengths in one pass over the tensor.
//
// Three kernels per search, all on the context's stream, no host round trip:
//   range   min / max of the finite elements; the last block to finish derives the bin grid
//           (power-of-two width) and the per-candidate integer bin parameters ("plan");
//           it also clears the global histograms.
//   hist    one read of the tensor: reference bin + one bin per candidate for every element,
//           counted in LDS-private histograms (per wavefront replicas when they fit), then
//           flushed to global memory with integer atomics (order-independent, exact).
//   kld     fp64 KL sums over the bins, selection of the lowest WL with KL < eps.
#include <algorithm>

#include "common.hpp"
#include "context.hpp"

namespace adapt {

constexpr int kMaxCand = 15;
constexpr int kHistThreads = 1024;
constexpr int kRangeThreads = 256;
constexpr size_t kLdsBudget = 144 * 1024;

struct KldCand {
    int d;        // T >> d gives floor(x * 2^(FL_c + 16))
    int kind;     // 0: bin = (q >> s) - base   1: bin = (q << s) - base (32-bit)   2: 64-bit left shift
    int s;        // shift amount (kind 0: already includes the 16 guard bits, capped at 31)
    int base32;   // bin origin, saturated to +-2^30
    int bmax;     // bin of the largest code of the candidate, clamped to [0, nb-1]
    int pad;
    long long base64;
};

struct KldPlan {
    int degenerate;   // no finite element or min == max
    int e;            // bin width 2^e
    int nb;           // number of bins in use
    int ncand;
    float lo, hi;
    float base_f;     // floor(lo * 2^-e), exactly representable
    float tscale;     // 2^FLmax
    float tmin, tmax; // code range of the widest candidate
    long long base;
    KldCand cand[kMaxCand];
};

__device__ inline double floor_scaled(double v, int e) { return floor(ldexp(v, -e)); }

// Runs in one thread.  lo < hi are finite fp32 values.
__device__ void make_plan(KldPlan *plan, float lo, float hi, int wl_lo, int wl_hi, int il, int bins)
{
    plan->lo = lo;
    plan->hi = hi;
    plan->ncand = wl_hi - wl_lo + 1;
    const double dlo = lo, dhi = hi;
    // smallest e with floor(hi/2^e) - floor(lo/2^e) + 1 <= bins; the count is non-increasing in e
    int e = ilogb(dhi - dlo) - ilogb((double)bins) - 2;
    while (floor_scaled(dhi, e) - floor_scaled(dlo, e) + 1.0 > (double)bins) ++e;
    while (floor_scaled(dhi, e - 1) - floor_scaled(dlo, e - 1) + 1.0 <= (double)bins) --e;
    const double fbase = floor_scaled(dlo, e);
    const long long base = (long long)fbase;
    const int nb = (int)(floor_scaled(dhi, e) - fbase + 1.0);
    plan->e = e;
    plan->nb = nb;
    plan->base = base;
    plan->base_f = (float)fbase;
    const int flmax = wl_hi - il;
    plan->tscale = ldexpf(1.0f, flmax);
    plan->tmin = -ldexpf(1.0f, wl_hi - 1);
    plan->tmax = ldexpf(1.0f, wl_hi - 1) - 1.0f;
    const long long lim = 1ll << 30;
    for (int c = 0; c < plan->ncand; ++c) {
        KldCand k;
        const int wl = wl_lo + c, fl = wl - il;
        const long long qmax = (1ll << (wl - 1)) - 1;
        const int sh = fl + e;
        k.d = wl_hi - wl;
        k.base64 = base;
        k.base32 = (int)(base > lim ? lim : base < -lim ? -lim : base);
        k.pad = 0;
        long long braw;
        if (sh >= 0) {
            k.kind = 0;
            k.s = 16 + sh > 31 ? 31 : 16 + sh;
            braw = (qmax >> (sh > 62 ? 62 : sh)) - base;
        } else {
            const int L = -sh;
            if (L <= 14 && base >= -lim && base <= lim) {
                k.kind = 1;
                k.s = L;
            } else {
                k.kind = 2;
                k.s = L > 42 ? 42 : L;   // 2^42 exceeds |base| + nb, so the sign of q decides
            }
            braw = (long long)((unsigned long long)qmax << k.s) - base;
        }
        k.bmax = (int)(braw < 0 ? 0 : braw > nb - 1 ? nb - 1 : braw);
        plan->cand[c] = k;
    }
    plan->degenerate = 0;
}

// ---- kernel 1: range + plan + clearing of the global histograms --------------------------------
__global__ void __launch_bounds__(kRangeThreads)
kld_range_kernel(const float *__restrict__ w, uint64_t n, int wl_lo, int wl_hi, int il, int bins, KldPlan *plan,
                 float *partial /* [2*gridDim.x] */, uint32_t *ticket, uint32_t *ghist, uint64_t ghist_words)
{
    const uint64_t tid = (uint64_t)blockIdx.x * kRangeThreads + threadIdx.x;
    const uint64_t nthreads = (uint64_t)gridDim.x * kRangeThreads;
    for (uint64_t i = tid; i < ghist_words; i += nthreads) ghist[i] = 0;

    float lo = INFINITY, hi = -INFINITY;
    const uint64_t n4 = n >> 2;
    for (uint64_t i = tid; i < n4; i += nthreads) {
        const float4 v = reinterpret_cast<const float4 *>(w)[i];
        const float a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (fabsf(a[j]) < INFINITY) { lo = fminf(lo, a[j]); hi = fmaxf(hi, a[j]); }
    }
    if (tid == 0)
        for (uint64_t i = n4 << 2; i < n; ++i)
            if (fabsf(w[i]) < INFINITY) { lo = fminf(lo, w[i]); hi = fmaxf(hi, w[i]); }
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    __shared__ float slo[kRangeThreads / kWave], shi[kRangeThreads / kWave];
    __shared__ bool last;
    if ((threadIdx.x & (kWave - 1)) == 0) { slo[threadIdx.x / kWave] = lo; shi[threadIdx.x / kWave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kRangeThreads / kWave; ++i) { lo = fminf(lo, slo[i]); hi = fmaxf(hi, shi[i]); }
        partial[2 * blockIdx.x] = lo;
        partial[2 * blockIdx.x + 1] = hi;
        __threadfence();
        last = (atomicAdd(ticket, 1u) == gridDim.x - 1);
    }
    __syncthreads();
    if (!last) return;
    __threadfence();
    lo = INFINITY; hi = -INFINITY;
    for (uint32_t b = threadIdx.x; b < gridDim.x; b += kRangeThreads) {
        lo = fminf(lo, __hip_atomic_load(partial + 2 * b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        hi = fmaxf(hi, __hip_atomic_load(partial + 2 * b + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    if ((threadIdx.x & (kWave - 1)) == 0) { slo[threadIdx.x / kWave] = lo; shi[threadIdx.x / kWave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kRangeThreads / kWave; ++i) { lo = fminf(lo, slo[i]); hi = fmaxf(hi, shi[i]); }
        if (!(lo < hi)) {      // nothing finite (lo = +inf) or a single value
            plan->degenerate = 1;
            plan->ncand = wl_hi - wl_lo + 1;
            plan->e = 0; plan->nb = 0; plan->base = 0; plan->lo = lo; plan->hi = hi;
        } else {
            make_plan(plan, lo, hi, wl_lo, wl_hi, il, bins);
        }
        *ticket = 0;
    }
}

// ---- kernel 2: histograms -----------------------------------------------------------------------

// Bin of an fp32 value: floor(v * 2^-e) - base.  Scaling by a power of two and the difference
// of the two floored values are exact; only a complete underflow to zero loses the sign.
__device__ __forceinline__ int value_bin(float v, int e, float base_f)
{
    const float t = ldexpf(v, -e);
    float f = floorf(t);
    if (t == 0.0f && v < 0.0f) f = -1.0f;
    return (int)(f - base_f);
}

__device__ __forceinline__ int cand_bin(const KldCand &k, int T, int r, int nbm1)
{
    const int tr = (T >> k.d) + r;
    int b;
    if (k.kind == 0) {
        b = (tr >> k.s) - k.base32;
    } else if (k.kind == 1) {
        b = (int)((unsigned)(tr >> 16) << k.s) - k.base32;
    } else {
        const long long q = (long long)(tr >> 16);
        const long long b64 = (long long)((unsigned long long)q << k.s) - k.base64;
        b = (int)(b64 < 0 ? 0 : b64 > (long long)nbm1 ? (long long)nbm1 : b64);
    }
    return min(max(b, 0), k.bmax);
}

// LDS layout: replica-major, then row (0 = reference, 1 + c = candidate c) over [row0, row0+rows),
// `nb` counters per row.  USE_LDS = false counts straight into global memory (bins too large).
template <bool USE_LDS>
__global__ void __launch_bounds__(kHistThreads)
kld_hist_kernel(const float *__restrict__ w, uint64_t n, const KldPlan *__restrict__ plan_g, uint32_t *ghist,
                int bins, int row0, int rows, int replicas, int mode, uint64_t seed, uint64_t stream)
{
    extern __shared__ uint32_t lds[];
    __shared__ KldPlan plan;
    for (int i = threadIdx.x; i < (int)(sizeof(KldPlan) / 4); i += kHistThreads)
        reinterpret_cast<uint32_t *>(&plan)[i] = reinterpret_cast<const uint32_t *>(plan_g)[i];
    __syncthreads();
    if (plan.degenerate) return;
    const int nb = plan.nb, nbm1 = nb - 1, e = plan.e;
    const float base_f = plan.base_f, tscale = plan.tscale, tmin = plan.tmin, tmax = plan.tmax;
    const int c_begin = max(row0 - 1, 0), c_end = row0 + rows - 1;   // candidate range of this pass
    const bool do_ref = (row0 == 0);
    uint32_t *hist;
    int row_stride;
    if (USE_LDS) {
        const int words = rows * nb;
        for (int i = threadIdx.x; i < words * replicas; i += kHistThreads) lds[i] = 0;
        __syncthreads();
        hist = lds + ((threadIdx.x / kWave) % replicas) * words;
        row_stride = nb;
    } else {
        hist = ghist + (size_t)row0 * bins;
        row_stride = bins;
    }

    auto count = [&](float v, int r) {
        if (!(fabsf(v) < INFINITY)) return;
        if (do_ref) atomicAdd(&hist[value_bin(v, e, base_f)], 1u);
        const float yc = fminf(fmaxf(v * tscale, tmin), tmax);
        const int T = (int)floorf(yc * 65536.0f);
        for (int c = c_begin; c < c_end; ++c)
            atomicAdd(&hist[(c + 1 - row0) * row_stride + cand_bin(plan.cand[c], T, r, nbm1)], 1u);
    };

    const uint64_t full_groups = n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kHistThreads + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * kHistThreads;
    for (uint64_t g = first; g < full_groups; g += stride) {
        const float4 a = reinterpret_cast<const float4 *>(w)[2 * g];
        const float4 b = reinterpret_cast<const float4 *>(w)[2 * g + 1];
        int r[8];
        if (mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(seed, stream, g);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = 0x8000;
        }
        count(a.x, r[0]); count(a.y, r[1]); count(a.z, r[2]); count(a.w, r[3]);
        count(b.x, r[4]); count(b.y, r[5]); count(b.z, r[6]); count(b.w, r[7]);
    }
    if ((n & 7) && first == 0)
        for (uint64_t i = full_groups << 3; i < n; ++i) count(w[i], (int)rounding_bits_of(seed, stream, i, mode));

    if (USE_LDS) {
        __syncthreads();
        const int words = rows * nb;
        for (int i = threadIdx.x; i < words; i += kHistThreads) {
            uint32_t v = 0;
            for (int rep = 0; rep < replicas; ++rep) v += lds[rep * words + i];
            if (v) atomicAdd(&ghist[(size_t)(row0 + i / nb) * bins + (i % nb)], v);
        }
    }
}

// ---- kernel 3: KL sums and selection --------------------------------------------------------------
__device__ __forceinline__ double block_sum_f64(double v, double *red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int off = kHistThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

__global__ void __launch_bounds__(kHistThreads)
kld_final_kernel(const KldPlan *__restrict__ plan, const uint32_t *__restrict__ ghist, int bins, int wl_lo, int il,
                 double eps, double alpha_in, double *kld, int32_t *sel, long long *grid_out)
{
    __shared__ double red[kHistThreads];
    __shared__ double kl_s[kMaxCand];
    const int ncand = plan->ncand;
    const int nb = plan->nb;
    if (plan->degenerate) {
        if ((int)threadIdx.x < ncand) kld[threadIdx.x] = 0.0;
        if (threadIdx.x == 0) {
            sel[0] = wl_lo; sel[1] = wl_lo - il;
            if (grid_out) { grid_out[0] = 0; grid_out[1] = 0; grid_out[2] = 0; }
        }
        return;
    }
    double cnt = 0.0;
    for (int b = threadIdx.x; b < nb; b += kHistThreads) cnt += (double)ghist[b];
    const double nfin = block_sum_f64(cnt, red);          // exact: integers below 2^53
    const double alpha = alpha_in < 0.0 ? 1.0 / (double)nb : alpha_in;
    const double denom = nfin + alpha * (double)nb;
    for (int c = 0; c < ncand; ++c) {
        double acc = 0.0;
        const uint32_t *cp = ghist + (size_t)(c + 1) * bins;
        for (int b = threadIdx.x; b < nb; b += kHistThreads) {
            const double p = ((double)cp[b] + alpha) / denom;
            const double q = ((double)ghist[b] + alpha) / denom;
            if (p > 0.0) acc += (q > 0.0) ? p * log2(p / q) : (double)INFINITY;
        }
        const double kl = block_sum_f64(acc, red);
        if (threadIdx.x == 0) { kld[c] = kl; kl_s[c] = kl; }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int pick = ncand - 1;
        for (int c = 0; c < ncand; ++c)
            if (kl_s[c] < eps) { pick = c; break; }
        sel[0] = wl_lo + pick;
        sel[1] = wl_lo + pick - il;
        if (grid_out) { grid_out[0] = plan->e; grid_out[1] = plan->base; grid_out[2] = nb; }
    }
}

static int search_one(adapt_ctx *ctx, const float *w, uint64_t n, int wl_lo, int wl_hi, int il, int bins, double eps,
                      double alpha, int mode, uint64_t seed, uint64_t stream, double *kld, int32_t *sel,
                      uint32_t *hist, int64_t *grid)
{
    const int ncand = wl_hi - wl_lo + 1;
    const int rows = ncand + 1;
    // workspace: plan | range partials | histograms (unless the caller supplied them)
    char *ws = scratch(ctx);
    const size_t plan_bytes = (sizeof(KldPlan) + 255) & ~(size_t)255;
    const int range_grid = (int)std::min<uint64_t>((uint64_t)ctx->num_cu * 4, std::max<uint64_t>(1, (n / 4 + kRangeThreads - 1) / kRangeThreads));
    const size_t partial_bytes = ((size_t)range_grid * 8 + 255) & ~(size_t)255;
    const size_t hist_words = (size_t)rows * bins;
    size_t need = plan_bytes + partial_bytes + (hist ? 0 : hist_words * 4);
    if (need > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    KldPlan *plan = reinterpret_cast<KldPlan *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan_bytes);
    uint32_t *ghist = hist ? hist : reinterpret_cast<uint32_t *>(ws + plan_bytes + partial_bytes);

    hipLaunchKernelGGL(kld_range_kernel, dim3(range_grid), dim3(kRangeThreads), 0, ctx->stream, w, n, wl_lo, wl_hi, il,
                       bins, plan, partial, ticket(ctx, 1), ghist, (uint64_t)hist_words);

    if (n > 0) {
        // enough elements per block to amortise the flush of the block's histograms
        const uint64_t per_block = 16384;
        const int hist_grid = (int)std::min<uint64_t>((uint64_t)ctx->num_cu, std::max<uint64_t>(1, (n + per_block - 1) / per_block));
        const size_t row_bytes = (size_t)bins * 4;
        if (row_bytes <= kLdsBudget) {
            const int rows_per_pass = (int)std::min<size_t>(rows, kLdsBudget / row_bytes);
            for (int row0 = 0; row0 < rows; row0 += rows_per_pass) {
                const int r = std::min(rows_per_pass, rows - row0);
                const int replicas = (int)std::min<size_t>(kHistThreads / kWave, kLdsBudget / (r * row_bytes));
                const size_t lds = (size_t)replicas * r * row_bytes;
                hipLaunchKernelGGL(kld_hist_kernel<true>, dim3(hist_grid), dim3(kHistThreads), lds, ctx->stream, w, n,
                                   plan, ghist, bins, row0, r, replicas, mode, seed, stream);
            }
        } else {
            hipLaunchKernelGGL(kld_hist_kernel<false>, dim3(hist_grid), dim3(kHistThreads), 0, ctx->stream, w, n, plan,
                               ghist, bins, 0, rows, 1, mode, seed, stream);
        }
    }
    hipLaunchKernelGGL(kld_final_kernel, dim3(1), dim3(kHistThreads), 0, ctx->stream, plan, ghist, bins, wl_lo, il, eps,
                       alpha, kld, sel, reinterpret_cast<long long *>(grid));
    return hip_status(ctx, hipGetLastError());
}

static int check_search_args(int wl_lo, int wl_hi, int il, int bins, double eps, double alpha, int mode)
{
    if (wl_lo < 2 || wl_hi > 16 || wl_lo > wl_hi) return ADAPT_EINVAL;
    if (il < 1 || wl_lo - il < 0 || wl_hi - il > 31) return ADAPT_EINVAL;
    if (bins < 2 || bins > 65536) return ADAPT_EINVAL;
    if (mode != ADAPT_SR && mode != ADAPT_RN_HALF_UP) return ADAPT_EINVAL;
    if (eps != eps || alpha != alpha) return ADAPT_EINVAL;
    return ADAPT_OK;
}

static hipError_t allow_big_lds()
{
    static hipError_t done = hipFuncSetAttribute(reinterpret_cast<const void *>(&kld_hist_kernel<true>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
    return done;
}

}  // namespace adapt

using namespace adapt;

extern "C" int adapt_kld_precision_search(adapt_ctx *ctx, const float *w, size_t n, int wl_lo, int wl_hi, int il,
                                          int bins, double eps, double alpha, adapt_rng rng, double *kld, int32_t *sel,
                                          uint32_t *hist, int64_t *grid)
{
    if (!ctx || !kld || !sel) return ADAPT_EINVAL;
    if (int s = check_search_args(wl_lo, wl_hi, il, bins, eps, alpha, rng.mode)) return s;
    if (n > 0 && (!w || !aligned16(w))) return ADAPT_EINVAL;
    if (n >= ((uint64_t)1 << 60)) return ADAPT_EINVAL;
    if (((uintptr_t)kld & 7) || ((uintptr_t)sel & 3) || ((uintptr_t)hist & 3) || ((uintptr_t)grid & 7)) return ADAPT_EINVAL;
    if (allow_big_lds() != hipSuccess) return hip_status(ctx, allow_big_lds());
    return search_one(ctx, w, n, wl_lo, wl_hi, il, bins, eps, alpha, rng.mode, rng.seed, rng.stream, kld, sel, hist, grid);
}

extern "C" int adapt_kld_precision_search_batched(adapt_ctx *ctx, const adapt_kld_item *items, int count, int wl_lo,
                                                  int wl_hi, double eps, double alpha, int mode, uint64_t seed,
                                                  double *kld, int32_t *sel)
{
    if (!ctx || count < 0 || (count > 0 && (!items || !kld || !sel))) return ADAPT_EINVAL;
    if (((uintptr_t)kld & 7) || ((uintptr_t)sel & 3)) return ADAPT_EINVAL;
    for (int t = 0; t < count; ++t) {
        if (int s = check_search_args(wl_lo, wl_hi, items[t].il, items[t].bins, eps, alpha, mode)) return s;
        if (items[t].n > 0 && (!items[t].w || !aligned16(items[t].w))) return ADAPT_EINVAL;
        if (items[t].n >= ((uint64_t)1 << 60)) return ADAPT_EINVAL;
    }
    if (allow_big_lds() != hipSuccess) return hip_status(ctx, allow_big_lds());
    const int ncand = wl_hi - wl_lo + 1;
    for (int t = 0; t < count; ++t) {
        const int s = search_one(ctx, items[t].w, items[t].n, wl_lo, wl_hi, items[t].il, items[t].bins, eps, alpha, mode,
                                 seed, items[t].stream, kld + (size_t)t * ncand, sel + 2 * t, nullptr, nullptr);
        if (s != ADAPT_OK) return s;
    }
    return ADAPT_OK;
}
