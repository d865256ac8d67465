// PushDown (Sec. 3.3 "The PushDown Operation", Alg. 3): KL divergence between the binned
// distribution of a tensor and of its <WL_c, FL_c> quantizations, for all candidate word
// lengths in one pass over the tensor.
//
// Four launches per search (per batch of searches in the batched form), all on the context's stream, no host round trip (kernel boundaries
// order the phases; only the small final kernel uses a device-wide fence):
//   range    per-block min / max of the finite elements.
//   hist     every block first reduces the range partials and derives the bin grid (power-of-two
//            width) and the per-candidate integer bin parameters (the "plan"; block 0 also stores
//            it for the later kernels), then reads its share of the tensor once: reference bin +
//            one bin per candidate for every element, counted in LDS histograms, and written to the block's own slab with plain stores.
//   sum      blocks of (256 bins, row): add the slabs of one row.
//   final    blocks of (256 bins, candidate): partial KL sums in fp64; the last block to finish adds
//            the partial sums in a fixed order and picks the lowest WL with KL < eps.
// All counts are integers, so the result does not depend on the order of accumulation.
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "common.hpp"
#include "context.hpp"

namespace adapt {

constexpr int kMaxCand = 31;                      // candidate word lengths 2..32
constexpr int kHistMaxThreads = 1024;
constexpr int kRangeThreads = 256;
constexpr size_t kLdsBudget = 156 * 1024;      // dynamic LDS of a block; 160 KB per CU less the static part
constexpr int kPrivWords = 1024;                  // counters of one coarse candidate's private table
constexpr int kChunk = 256;                       // bins per block of the final kernel

struct KldCand {
    int d;        // T >> d gives floor(x * 2^(FL_c + 16))
    int kind;     // 0: bin = (q >> s) - base   1: bin = (q << s) - base (32-bit)   2: 64-bit left shift
    int s;        // shift amount (kind 0: includes the 16 guard bits, capped at 31)
    int lo;       // bin origin, saturated to +-2^30 ("base32")
    int hi;       // lo + bin of the largest code of the candidate (already clamped to [0, nb-1])
    int bmax;
    long long base64;
    // Candidates whose codes are coarser than the bins populate few bins, and the LDS atomics of a
    // wavefront would serialise on them: they are counted by code, in lane-private LDS counters
    // (index (q - qmin) * 2^rsh + lane mod 2^rsh, q clamped to [qmin, qmax]), and mapped to bins once
    // per block.
    int coarse, qmin, qmax, rsh;
};

struct KldPlan {
    int degenerate;   // no finite element or min == max
    int e;            // bin width 2^e
    int nb;           // number of bins in use
    int ncand;
    float lo, hi;
    float base_f;     // floor(lo * 2^-e), exactly representable
    float tscale;     // 2^(FLmax + 16)
    float tmin, tmax; // code range of the widest candidate, times 2^16
    int wide;         // candidates above 16 bits: the scaled value needs 48 bits (fp64 scaling, 64-bit integer forms)
    double tscale_d, tmin_d, tmax_d;
    long long base;
    KldCand cand[kMaxCand];
};

// floor(v * 2^-e) for |e| < 1000 and v an fp32 value held in a double: the power of two is built
// from its exponent bits and the product is exact (no overflow or underflow in that range).
__device__ inline double floor_scaled(double v, int e) { return floor(v * __longlong_as_double((long long)(1023 - e) << 52)); }
__device__ inline int exponent_of(double v) { return (int)((__double_as_longlong(v) >> 52) & 0x7ff) - 1023; }   // normal v > 0

// Bin grid from the range: runs in one thread.  lo < hi are finite fp32 values.
__device__ void make_grid(KldPlan *plan, float lo, float hi, int wl_hi, int il, int bins)
{
    const double dlo = lo, dhi = hi;
    // smallest e with floor(hi/2^e) - floor(lo/2^e) + 1 <= bins; the count is non-increasing in e
    int e = exponent_of(dhi - dlo) - exponent_of((double)bins) - 2;
    while (floor_scaled(dhi, e) - floor_scaled(dlo, e) + 1.0 > (double)bins) ++e;
    while (floor_scaled(dhi, e - 1) - floor_scaled(dlo, e - 1) + 1.0 <= (double)bins) --e;
    const double fbase = floor_scaled(dlo, e);
    plan->e = e;
    plan->nb = (int)(floor_scaled(dhi, e) - fbase + 1.0);
    plan->base = (long long)fbase;
    plan->base_f = (float)fbase;
    plan->lo = lo;
    plan->hi = hi;
    const int flmax = wl_hi - il;
    plan->tscale = ldexpf(1.0f, flmax + 16);
    plan->tmin = -ldexpf(1.0f, wl_hi - 1 + 16);
    plan->tmax = (ldexpf(1.0f, wl_hi - 1) - 1.0f) * 65536.0f;
    plan->wide = wl_hi > 16;
    plan->tscale_d = ldexp(1.0, flmax + 16);
    plan->tmin_d = -ldexp(1.0, wl_hi - 1 + 16);
    plan->tmax_d = (ldexp(1.0, wl_hi - 1) - 1.0) * 65536.0;
    plan->degenerate = 0;
}

// Parameters of candidate c: runs in one thread per candidate after make_grid.
__device__ void make_candidate(KldPlan *plan, int c, int wl_lo, int wl_hi, int il)
{
    KldCand k;
    const int e = plan->e, nb = plan->nb;
    const long long base = plan->base;
    const int wl = wl_lo + c, fl = wl - il;
    const long long qmax = (1ll << (wl - 1)) - 1;
    const int sh = fl + e;
    const long long lim = 1ll << 30;
    k.d = wl_hi - wl;
    k.base64 = base;
    k.lo = (int)(base > lim ? lim : base < -lim ? -lim : base);
    long long braw;
    if (sh >= 0) {
        k.kind = 0;
        const int cap = plan->wide ? 63 : 31;               // beyond the width of the scaled value only its sign is left
        k.s = 16 + sh > cap ? cap : 16 + sh;
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
    k.hi = k.lo + k.bmax;
    // Codes coarser than the bins (kind 1) populate few bins: count them by code.  Only the codes
    // whose bins fall inside the row matter (the others clamp to its ends, as their neighbours do).
    k.coarse = 0; k.qmin = 0; k.qmax = 0; k.rsh = 0;
    if (k.kind == 1) {
        const int qa = k.lo >> k.s, qb = -((-k.hi) >> k.s);          // floor(lo / 2^s), ceil(hi / 2^s)
        const int qlo = qa > -(int)(qmax + 1) ? qa : -(int)(qmax + 1), qhi = qb < (int)qmax ? qb : (int)qmax;
        const int ncodes = qhi - qlo + 1;
        if (ncodes >= 1 && ncodes <= kPrivWords) {
            k.coarse = 1; k.qmin = qlo; k.qmax = qhi;
            while (k.rsh < 6 && (ncodes << (k.rsh + 1)) <= kPrivWords) ++k.rsh;
        }
    }
    plan->cand[c] = k;
}

// Position of a block inside the (sub-)grid of one tensor's search: the single-tensor kernels take
// it from blockIdx / gridDim, the batched kernels from the batch table.
struct BlockGeo { unsigned bx, by, gx, gy; };

// ---- kernel 1: per-block range of the finite elements -----------------------------------------------
__device__ __forceinline__ void kld_range_body(const float *__restrict__ w, uint64_t n, float *partial /* [2*gx] */,
                                               const BlockGeo geo)
{
    const uint64_t tid = (uint64_t)geo.bx * kRangeThreads + threadIdx.x;
    const uint64_t nthreads = (uint64_t)geo.gx * kRangeThreads;
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
    if ((threadIdx.x & (kWave - 1)) == 0) { slo[threadIdx.x / kWave] = lo; shi[threadIdx.x / kWave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kRangeThreads / kWave; ++i) { lo = fminf(lo, slo[i]); hi = fmaxf(hi, shi[i]); }
        partial[2 * geo.bx] = lo;
        partial[2 * geo.bx + 1] = hi;
    }
}

__global__ void __launch_bounds__(kRangeThreads)
kld_range_kernel(const float *__restrict__ w, uint64_t n, float *partial /* [2*gridDim.x] */)
{
    kld_range_body(w, n, partial, BlockGeo{blockIdx.x, 0, gridDim.x, 1});
}

// ---- kernel 2: plan + histograms ------------------------------------------------------------------------

// Bin of an fp32 value: floor(v * 2^-e) - base.  Scaling by a power of two and the difference
// of the two floored values are exact; only a complete underflow to zero loses the sign.
__device__ __forceinline__ int value_bin(float v, int e, float base_f)
{
    const float t = ldexpf(v, -e);
    const float f = (t == 0.0f && v < 0.0f) ? -1.0f : floorf(t);
    return (int)(f - base_f);
}

// Adds the 8 elements of a group to candidate k's row.  x = bin + k.lo of the candidate's code for
// an element with scaled value T and rounding bits r; `inc` is 0 for non-finite elements (their
// clamped bin is a valid address).  The branch on the candidate's kind is uniform and outside
// the element loop, so the loop bodies are straight-line code.
// bin + k.lo of code q (the value that count_candidate computes from T and r), clamped into the row
__device__ __forceinline__ int bin_of_code(const KldCand &k, int q)
{
    if (k.kind == 0) return min(max(q >> (k.s - 16), k.lo), k.hi);
    if (k.kind == 1) return min(max((int)((unsigned)q << k.s), k.lo), k.hi);
    const long long b64 = (long long)((unsigned long long)(long long)q << k.s) - k.base64;
    return (int)(b64 < 0 ? 0 : b64 > (long long)k.bmax ? (long long)k.bmax : b64) + k.lo;
}

// min(max(x, lo), hi) for lo <= hi in one instruction (the median of the three)
__device__ __forceinline__ int clamp_i32(int x, int lo, int hi)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
    return r;
}

// `park` is a lane-private LDS word that takes the (zero) additions of the elements that are counted elsewhere: zeros
// and non-finite elements.  An atomic addition of 0 still takes its turn at the counter's address, and the zeros of
// a pruned tensor would queue up there.
// TT: int for candidates up to 16 bits, long long above (the scaled value has up to 48 bits)
template <typename TT>
__device__ __forceinline__ int clamp_tt(TT x, int lo, int hi)
{
    if (sizeof(TT) == 4) return clamp_i32((int)x, lo, hi);
    return (int)(x < (TT)lo ? (TT)lo : x > (TT)hi ? (TT)hi : x);
}

template <typename TT>
__device__ __forceinline__ void count_candidate_by_code(const KldCand &k, uint32_t *priv, uint32_t *park, int lane, const TT (&T)[8],
                                                        const int (&r)[8], const uint32_t (&inc)[8])
{
    const int sub = lane & ((1 << k.rsh) - 1);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int q = clamp_tt<TT>(((T[j] >> k.d) + (TT)r[j]) >> 16, k.qmin, k.qmax);
        atomicAdd(inc[j] ? &priv[((q - k.qmin) << k.rsh) + sub] : park, inc[j]);
    }
}

// USE_LDS: row and park are LDS words; else row is global memory and the skipped elements are predicated off
template <bool USE_LDS>
__device__ __forceinline__ void count_one(uint32_t *row, uint32_t *park, int x, uint32_t inc)
{
    if (USE_LDS) atomicAdd(inc ? &row[x] : park, inc);
    else if (inc) atomicAdd(&row[x], inc);
}

template <bool USE_LDS, typename TT>
__device__ __forceinline__ void count_candidate(const KldCand &k, uint32_t *row, uint32_t *park, const TT (&T)[8], const int (&r)[8],
                                                const uint32_t (&inc)[8])
{
    typedef typename std::make_unsigned<TT>::type UT;
    if (k.kind == 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const TT x = ((T[j] >> k.d) + (TT)r[j]) >> k.s;
            count_one<USE_LDS>(row, park, clamp_tt<TT>(x, k.lo, k.hi), inc[j]);
        }
    } else if (k.kind == 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const TT x = (TT)((UT)(((T[j] >> k.d) + (TT)r[j]) >> 16) << k.s);
            count_one<USE_LDS>(row, park, clamp_tt<TT>(x, k.lo, k.hi), inc[j]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const long long q = (long long)(((T[j] >> k.d) + r[j]) >> 16);
            const long long b64 = (long long)((unsigned long long)q << k.s) - k.base64;
            const int x = (int)(b64 < 0 ? 0 : b64 > (long long)k.bmax ? (long long)k.bmax : b64) + k.lo;
            count_one<USE_LDS>(row, park, x, inc[j]);
        }
    }
}

__global__ void zero_words_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// LDS layout: row (0 = reference, 1 + c = candidate c) over [row0, row0+rows), `nb` counters per row.  Every block writes its counts (zeros included) to its own slab
// slabs[block][row][bins] with plain stores: device-wide atomics on shared counters are far
// slower than that on this GPU.  USE_LDS = false (bins too large for LDS) counts with atomics
// straight into the block's slab, which the host has cleared.
template <bool USE_LDS, bool WIDE = false>
__device__ __forceinline__ void kld_hist_body(const float *__restrict__ w, uint64_t n, const float *__restrict__ range_partial,
                                              int range_blocks, int wl_lo, int wl_hi, int il, int bins, KldPlan *plan_out,
                                              uint32_t *tickets, uint32_t *slabs, int total_rows, int rows_per_group, int mode,
                                              uint64_t seed, uint64_t stream, const BlockGeo geo)
{
    // geo.by selects a group of histogram rows: small tensors are spread over more CUs by
    // letting several blocks count different candidates of the same elements
    const int row0 = geo.by * rows_per_group;
    const int rows = min(rows_per_group, total_rows - row0);
    extern __shared__ uint32_t lds[];
    __shared__ KldPlan plan;
    __shared__ float slo[kHistMaxThreads / kWave], shi[kHistMaxThreads / kWave];
    __shared__ int row_off[kMaxCand];          // word offset of the candidate's row minus its bin origin
    __shared__ int priv_off[kMaxCand];         // word offset of a coarse candidate's private table, else -1
    __shared__ uint32_t park_words[kWave];     // where the additions of skipped elements go, one word per lane
    uint32_t *park = &park_words[threadIdx.x & (kWave - 1)];
    const int nthreads = blockDim.x, nwaves = nthreads / kWave;
    const int ncand = wl_hi - wl_lo + 1;

    // ---- plan (identical in every block) ----
    {
        float lo = INFINITY, hi = -INFINITY;
        for (int b = threadIdx.x; b < range_blocks; b += nthreads) {
            lo = fminf(lo, range_partial[2 * b]);
            hi = fmaxf(hi, range_partial[2 * b + 1]);
        }
        lo = wave_min_f32(lo);
        hi = wave_max_f32(hi);
        if ((threadIdx.x & (kWave - 1)) == 0) { slo[threadIdx.x / kWave] = lo; shi[threadIdx.x / kWave] = hi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int i = 1; i < nwaves; ++i) { lo = fminf(lo, slo[i]); hi = fmaxf(hi, shi[i]); }
            plan.ncand = ncand;
            if (!(lo < hi)) {      // nothing finite (lo = +inf) or a single value
                plan.degenerate = 1;
                plan.e = 0; plan.nb = 0; plan.base = 0; plan.lo = lo; plan.hi = hi;
            } else {
                make_grid(&plan, lo, hi, wl_hi, il, bins);
            }
        }
        __syncthreads();
        if (!plan.degenerate && (int)threadIdx.x < ncand) make_candidate(&plan, threadIdx.x, wl_lo, wl_hi, il);
        __syncthreads();
        if (geo.bx == 0 && geo.by == 0) {
            for (int i = threadIdx.x; i < (int)(sizeof(KldPlan) / 4); i += nthreads)
                reinterpret_cast<uint32_t *>(plan_out)[i] = reinterpret_cast<const uint32_t *>(&plan)[i];
            if (threadIdx.x == 0) tickets[0] = 0;      // the ticket of the final kernel
        }
    }
    if (plan.degenerate) return;

    const int nb = plan.nb, e = plan.e;
    const float base_f = plan.base_f, tscale = plan.tscale, tmin = plan.tmin, tmax = plan.tmax;
    const int c_begin = max(row0 - 1, 0), c_end = row0 + rows - 1;   // candidate range of this pass
    const bool do_ref = (row0 == 0);
    uint32_t *hist;
    int row_stride;
    if (USE_LDS) {
        // rows, padded to a multiple of 4 words, then one private table per coarse candidate of this block
        const int rows_words = (rows * nb + 3) & ~3;
        int ncoarse = 0;
        for (int c = c_begin; c < c_end; ++c) ncoarse += plan.cand[c].coarse;
        const int total = rows_words + ncoarse * kPrivWords;
        for (int i = threadIdx.x; i < total / 4; i += nthreads) reinterpret_cast<uint4 *>(lds)[i] = make_uint4(0, 0, 0, 0);
        if (threadIdx.x == 0) {
            int next = rows_words;
            for (int c = c_begin; c < c_end; ++c) {
                priv_off[c] = plan.cand[c].coarse ? next : -1;
                next += plan.cand[c].coarse ? kPrivWords : 0;
            }
        }
        hist = lds;
        row_stride = nb;
    } else {
        if ((int)threadIdx.x >= c_begin && (int)threadIdx.x < c_end) priv_off[threadIdx.x] = -1;
        hist = slabs + ((size_t)geo.bx * total_rows + row0) * bins;
        row_stride = bins;
    }
    if ((int)threadIdx.x >= c_begin && (int)threadIdx.x < c_end)
        row_off[threadIdx.x] = (threadIdx.x + 1 - row0) * row_stride - plan.cand[threadIdx.x].lo;
    __syncthreads();

    // Zeros (pruned weights, Sec. 3.4) all land in one counter of every row, where the LDS atomics of a wavefront
    // would serialise: each thread counts its zeros in a register and the block adds the total to the rows once.
    // A zero has code 0 under every candidate, whatever its rounding bits.
    uint32_t nzero = 0;
    // One group = 8 consecutive elements of one thread (one Philox block).  A pass takes G groups into registers,
    // counts the reference row, then visits the candidates one after the other: a candidate's parameters are read
    // (and made wavefront-uniform) once per pass, and its kind is one uniform branch around 8 G straight-line elements.
    auto count_groups = [&](auto gtag, const float (&v)[decltype(gtag)::value][8], const int (&r)[decltype(gtag)::value][8],
                            const int (&cnt)[decltype(gtag)::value]) {
        constexpr int G = decltype(gtag)::value;
        typedef typename std::conditional<WIDE, long long, int>::type TT;
        TT T[G][8];
        uint32_t inc[G][8];
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool zero = v[u][j] == 0.0f;
                const bool fin = j < cnt[u] && fabsf(v[u][j]) < INFINITY;
                nzero += (fin && zero) ? 1u : 0u;
                inc[u][j] = (fin && !zero) ? 1u : 0u;
                if (WIDE) T[u][j] = (TT)floor(fmin(fmax((double)v[u][j] * plan.tscale_d, plan.tmin_d), plan.tmax_d));
                else T[u][j] = (TT)(int)floorf(fminf(fmaxf(v[u][j] * tscale, tmin), tmax));      // NaN -> tmin
                // (the clamp only acts when a caller-supplied range does not bound the tensor)
            }
        if (do_ref) {
#pragma unroll
            for (int u = 0; u < G; ++u)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    count_one<USE_LDS>(hist, park, inc[u][j] ? min(max(value_bin(v[u][j], e, base_f), 0), nb - 1) : 0, inc[u][j]);
        }
        for (int c = c_begin; c < c_end; ++c) {
            KldCand k;
            k.d = __builtin_amdgcn_readfirstlane(plan.cand[c].d);
            k.kind = __builtin_amdgcn_readfirstlane(plan.cand[c].kind);
            k.s = __builtin_amdgcn_readfirstlane(plan.cand[c].s);
            k.lo = __builtin_amdgcn_readfirstlane(plan.cand[c].lo);
            k.hi = __builtin_amdgcn_readfirstlane(plan.cand[c].hi);
            k.bmax = __builtin_amdgcn_readfirstlane(plan.cand[c].bmax);
            k.base64 = plan.cand[c].base64;
            k.coarse = 0;
            k.qmin = __builtin_amdgcn_readfirstlane(plan.cand[c].qmin);
            k.qmax = __builtin_amdgcn_readfirstlane(plan.cand[c].qmax);
            k.rsh = __builtin_amdgcn_readfirstlane(plan.cand[c].rsh);
            const int poff = __builtin_amdgcn_readfirstlane(priv_off[c]), roff = __builtin_amdgcn_readfirstlane(row_off[c]);
            if (USE_LDS && poff >= 0) {
#pragma unroll
                for (int u = 0; u < G; ++u) count_candidate_by_code<TT>(k, lds + poff, park, threadIdx.x & (kWave - 1), T[u], r[u], inc[u]);
            } else {
#pragma unroll
                for (int u = 0; u < G; ++u) count_candidate<USE_LDS, TT>(k, hist + roff, park, T[u], r[u], inc[u]);
            }
        }
    };
    auto rounding_of = [&](uint64_t g, int (&r)[8]) {
        if (mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(seed, stream, g);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = 0x8000;
        }
    };

    constexpr int kPass = 4;
    const uint64_t full_groups = n >> 3;
    const uint64_t first = (uint64_t)geo.bx * nthreads + threadIdx.x;
    const uint64_t stride = (uint64_t)geo.gx * nthreads;
    uint64_t g = first;
    for (; g + (kPass - 1) * stride < full_groups; g += kPass * stride) {
        float v[kPass][8];
        int r[kPass][8], cnt[kPass];
#pragma unroll
        for (int u = 0; u < kPass; ++u) {
            const float4 a = reinterpret_cast<const float4 *>(w)[2 * (g + u * stride)];
            const float4 b = reinterpret_cast<const float4 *>(w)[2 * (g + u * stride) + 1];
            v[u][0] = a.x; v[u][1] = a.y; v[u][2] = a.z; v[u][3] = a.w; v[u][4] = b.x; v[u][5] = b.y; v[u][6] = b.z; v[u][7] = b.w;
            cnt[u] = 8;
        }
#pragma unroll
        for (int u = 0; u < kPass; ++u) rounding_of(g + u * stride, r[u]);
        count_groups(std::integral_constant<int, kPass>{}, v, r, cnt);
    }
    // the last groups of the thread (fewer than kPass): a pass of two, then single groups
    if (g + stride < full_groups) {
        float v[2][8];
        int r[2][8];
        const int cnt[2] = {8, 8};
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float4 a = reinterpret_cast<const float4 *>(w)[2 * (g + u * stride)];
            const float4 b = reinterpret_cast<const float4 *>(w)[2 * (g + u * stride) + 1];
            v[u][0] = a.x; v[u][1] = a.y; v[u][2] = a.z; v[u][3] = a.w; v[u][4] = b.x; v[u][5] = b.y; v[u][6] = b.z; v[u][7] = b.w;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) rounding_of(g + u * stride, r[u]);
        count_groups(std::integral_constant<int, 2>{}, v, r, cnt);
        g += 2 * stride;
    }
    for (; g < full_groups; g += stride) {
        const float4 a = reinterpret_cast<const float4 *>(w)[2 * g];
        const float4 b = reinterpret_cast<const float4 *>(w)[2 * g + 1];
        const float v[1][8] = {{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
        int r[1][8];
        const int cnt[1] = {8};
        rounding_of(g, r[0]);
        count_groups(std::integral_constant<int, 1>{}, v, r, cnt);
    }
    if ((n & 7) && first == 0) {
        float v[1][8];
        int r[1][8];
        const int cnt[1] = {(int)(n & 7)};
        for (int j = 0; j < 8; ++j) {
            const uint64_t i = (full_groups << 3) + j;
            v[0][j] = j < cnt[0] ? w[i] : 0.0f;
            r[0][j] = (int)rounding_bits_of(seed, stream, i, mode);
        }
        count_groups(std::integral_constant<int, 1>{}, v, r, cnt);
    }

    // the block's zeros: one addition per row
    __shared__ uint32_t zero_total;
    if (threadIdx.x == 0) zero_total = 0;
    __syncthreads();
    nzero = wave_sum_u32(nzero);
    if ((threadIdx.x & (kWave - 1)) == 0 && nzero) atomicAdd(&zero_total, nzero);
    __syncthreads();
    if (zero_total) {
        if (do_ref && threadIdx.x == 0) atomicAdd(&hist[min(max(value_bin(0.0f, e, base_f), 0), nb - 1)], zero_total);
        if ((int)threadIdx.x >= c_begin && (int)threadIdx.x < c_end)
            atomicAdd(&hist[row_off[threadIdx.x] + bin_of_code(plan.cand[threadIdx.x], 0)], zero_total);
    }

    if (USE_LDS) {
        __syncthreads();
        // coarse candidates: per-code counts (summed over the lane-private copies) into the bins of the row
        bool any = false;
        for (int c = c_begin; c < c_end; ++c) {
            if (priv_off[c] < 0) continue;
            any = true;
            const KldCand &k = plan.cand[c];
            const uint32_t *priv = lds + priv_off[c];
            for (int i = threadIdx.x; i < kPrivWords; i += nthreads) {
                const uint32_t v = priv[i];
                if (v) atomicAdd(&hist[row_off[c] + bin_of_code(k, (i >> k.rsh) + k.qmin)], v);
            }
        }
        if (any) __syncthreads();
        // slab rows are 16-byte aligned when bins % 4 == 0; otherwise every counter is written singly
        const int nb4 = (bins % 4 == 0) ? nb / 4 : 0;
        for (int row = 0; row < rows; ++row) {
            uint32_t *dst = slabs + ((size_t)geo.bx * total_rows + row0 + row) * bins;
            const uint32_t *src = lds + row * nb;
            for (int q = threadIdx.x; q < nb4; q += nthreads)
                reinterpret_cast<uint4 *>(dst)[q] = make_uint4(src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]);
            for (int b = 4 * nb4 + threadIdx.x; b < nb; b += nthreads) dst[b] = src[b];
        }
    }
}

template <bool USE_LDS, bool WIDE = false>
__global__ void __launch_bounds__(kHistMaxThreads)
kld_hist_kernel(const float *__restrict__ w, uint64_t n, const float *__restrict__ range_partial, int range_blocks,
                int wl_lo, int wl_hi, int il, int bins, KldPlan *plan_out, uint32_t *tickets, uint32_t *slabs, int total_rows,
                int rows_per_group, int mode, uint64_t seed, uint64_t stream)
{
    kld_hist_body<USE_LDS, WIDE>(w, n, range_partial, range_blocks, wl_lo, wl_hi, il, bins, plan_out, tickets, slabs, total_rows,
                           rows_per_group, mode, seed, stream, BlockGeo{blockIdx.x, blockIdx.y, gridDim.x, gridDim.y});
}

// ---- kernel 3: slab sums, partial KL sums, selection ---------------------------------------------------------
// With the same smoothing and the same total on both sides,
//   KL = sum_b P(b) log2(P(b)/Q(b)) = (1/D) sum_b (cp_b + alpha) log2((cp_b + alpha)/(cq_b + alpha)),
// D = n_finite + alpha nb, so bins with cp_b == cq_b contribute nothing and need no logarithm.
// Two launches (a device-wide fence per block, which a single launch would need, empties the caches the slab
// loads live on).  Sum: block (x, row) adds bins [x*kChunk, (x+1)*kChunk) of one row over the slabs into
// sums[row][bins].  Final: block (x, c) forms the terms of candidate c on its bins and their sum part[c][x]
// (block (x, 0) also part[ncand][x], the sum of reference counts); the last block of the search to finish
// (a ticket) adds them in a fixed order and selects.
// The region of a search in the scratch: ticket | part | sums.
struct KlRegion {
    uint32_t *tickets;      // [0]: blocks of the final kernel that have finished
    double *part;           // [(ncand + 1) * nchunks]
    uint32_t *sums;         // [rows * bins]
};
__host__ __device__ inline size_t kl_region_bytes(int ncand, int nchunks, int bins)
{
    auto a256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    return a256((size_t)(nchunks + 1) * 4) + a256((size_t)(ncand + 1) * nchunks * 8) + a256((size_t)(ncand + 1) * bins * 4);
}
__host__ __device__ inline KlRegion kl_region(char *base, int ncand, int nchunks)
{
    auto a256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    KlRegion r;
    r.tickets = reinterpret_cast<uint32_t *>(base);
    r.part = reinterpret_cast<double *>(base + a256((size_t)(nchunks + 1) * 4));
    r.sums = reinterpret_cast<uint32_t *>(base + a256((size_t)(nchunks + 1) * 4) + a256((size_t)(ncand + 1) * nchunks * 8));
    return r;
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);      // the same tree in every lane
    return v;
}

// kernel 3a, block (x, row): sums[row][b] = sum over the slabs, one thread per bin, eight loads in flight
__device__ __forceinline__ void kld_sum_body(const KldPlan *__restrict__ plan, const uint32_t *__restrict__ slabs, int nslabs,
                                             int rows, int bins, uint32_t *__restrict__ sums, uint32_t *hist_out, const BlockGeo geo)
{
    const int row = geo.by;
    const int b = geo.bx * kChunk + threadIdx.x;
    const int nb = plan->degenerate ? 0 : plan->nb;
    const size_t slab_words = (size_t)rows * bins;
    uint32_t u = 0;
    if (b < nb) {
        // a slab index past the end is redirected to slab 0 and its value dropped, so the loads carry no branches
        const uint32_t *p = slabs + (size_t)row * bins + b;
        for (int s0 = 0; s0 < nslabs; s0 += 8) {
            uint32_t t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = p[s0 + i < nslabs ? (size_t)(s0 + i) * slab_words : 0];
#pragma unroll
            for (int i = 0; i < 8; ++i) u += s0 + i < nslabs ? t[i] : 0u;
        }
    }
    if (b < bins) {
        __hip_atomic_store(sums + (size_t)row * bins + b, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (hist_out) hist_out[(size_t)row * bins + b] = u;
    }
}

// kernel 3b, block (x, y): terms of the candidates y, y + gy, ... on bins [x*kChunk, (x+1)*kChunk), each summed over
// the chunk in a fixed order (lanes, then wavefronts); the blocks with y = 0 also sum the chunk's reference counts.
// gy = number of candidates: one logarithm per thread (small searches, where latency counts); gy = 1: every
// candidate in turn (batches of large searches, where the device-wide fence of 13 times as many tickets costs more
// than it saves).  The last block of the search to finish adds the chunks in a fixed order and selects.
__device__ __forceinline__ void kld_final_body(const KldPlan *__restrict__ plan, int rows, int bins, double alpha_in,
                                               const KlRegion reg, int wl_lo, int il, double eps, double *kld, int32_t *sel,
                                               long long *grid_out, const BlockGeo geo)
{
    const int x = geo.bx, nchunks = geo.gx, ncand = rows - 1;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int b = x * kChunk + threadIdx.x;
    const int nb = plan->degenerate ? 0 : plan->nb;
    __shared__ double red[kMaxCand + 1][kChunk / kWave];
    const double alpha = alpha_in < 0.0 ? 1.0 / (double)(nb > 0 ? nb : 1) : alpha_in;
    const uint32_t uq = b < nb ? __hip_atomic_load(reg.sums + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    for (int c = geo.by; c < ncand; c += geo.gy) {
        const uint32_t up = b < nb ? __hip_atomic_load(reg.sums + (size_t)(c + 1) * bins + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : uq;
        double term = 0.0;
        if (up != uq) {
            const double pp = (double)up + alpha, qq = (double)uq + alpha;
            if (pp > 0.0) term = (qq > 0.0) ? pp * log2(pp / qq) : (double)INFINITY;
        }
        term = wave_sum_f64(term);
        if (lane == 0) red[c][wave] = term;
    }
    if (geo.by == 0) {
        const double cnt = wave_sum_f64((double)uq);      // exact
        if (lane == 0) red[ncand][wave] = cnt;
    }
    __syncthreads();
    __shared__ bool last_block;
    if (threadIdx.x == 0) {
        auto put = [&](int c) {
            double t = red[c][0];
#pragma unroll
            for (int i = 1; i < kChunk / kWave; ++i) t += red[c][i];
            __hip_atomic_store(reg.part + (size_t)c * nchunks + x, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        for (int c = geo.by; c < ncand; c += geo.gy) put(c);
        if (geo.by == 0) put(ncand);
        // release this block's partial sums, acquire everyone else's
        last_block = __hip_atomic_fetch_add(reg.tickets, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == geo.gx * geo.gy - 1;
    }
    __syncthreads();
    if (!last_block) return;

    __shared__ double kl_s[kMaxCand];
    if ((int)threadIdx.x < ncand) {
        const int cc = threadIdx.x;
        double total = 0.0, nfin = 0.0;
        for (int i = 0; i < nchunks; ++i) {
            total += __hip_atomic_load(reg.part + (size_t)cc * nchunks + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            nfin += __hip_atomic_load(reg.part + (size_t)ncand * nchunks + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // exact
        }
        const double kl = nb > 0 ? total / (nfin + alpha * (double)nb) : 0.0;
        kld[cc] = kl;
        kl_s[cc] = kl;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    int pick = plan->degenerate ? 0 : ncand - 1;
    if (!plan->degenerate)
        for (int i = 0; i < ncand; ++i)
            if (kl_s[i] < eps) { pick = i; break; }
    sel[0] = wl_lo + pick;
    sel[1] = wl_lo + pick - il;
    if (grid_out) {
        grid_out[0] = plan->degenerate ? 0 : plan->e;
        grid_out[1] = plan->degenerate ? 0 : plan->base;
        grid_out[2] = plan->degenerate ? 0 : plan->nb;
    }
}

__global__ void __launch_bounds__(kChunk)
kld_sum_kernel(const KldPlan *__restrict__ plan, const uint32_t *__restrict__ slabs, int nslabs, int rows, int bins, char *region,
               uint32_t *hist_out)
{
    kld_sum_body(plan, slabs, nslabs, rows, bins, kl_region(region, rows - 1, gridDim.x).sums, hist_out,
                 BlockGeo{blockIdx.x, blockIdx.y, gridDim.x, gridDim.y});
}

__global__ void __launch_bounds__(kChunk)
kld_final_kernel(const KldPlan *__restrict__ plan, int rows, int bins, double alpha_in, char *region, int wl_lo, int il, double eps,
                 double *kld, int32_t *sel, long long *grid_out)
{
    kld_final_body(plan, rows, bins, alpha_in, kl_region(region, rows - 1, gridDim.x), wl_lo, il, eps, kld, sel, grid_out,
                   BlockGeo{blockIdx.x, blockIdx.y, gridDim.x, gridDim.y});
}

// ---- batched form: the three phases of up to kKldBatchMax searches, one launch per phase --------------------
constexpr int kKldBatchMax = 24;
struct KldBatchItem {
    const float *w;
    const float *range;       // device (min, max) of the finite elements, or null: the range pass computes it
    uint64_t n, stream;
    double *kld;
    int32_t *sel;
    unsigned long long off_plan, off_range, off_klpart, off_slabs;      // byte offsets into the scratch
    int il, bins, range_blocks, hist_x, groups, rows_per_group, nchunks;
};
struct KldBatch {
    KldBatchItem item[kKldBatchMax];
    // first block of each tensor in the four launches (ascending)
    unsigned first_range[kKldBatchMax], first_hist[kKldBatchMax], first_sum[kKldBatchMax], first_final[kKldBatchMax];
    int count, wl_lo, wl_hi, mode;
    int final_y;              // blocks per chunk of the final launch: the number of candidates, or 1
    unsigned long long seed;
    double eps, alpha;
    char *ws;
};

// the tensor a block belongs to: every lane compares one table entry, the wavefront votes
#define ADAPT_KLD_FIND(field)                                                                             \
    const int lane_ = threadIdx.x & (kWave - 1);                                                          \
    const unsigned first_ = lane_ < b.count ? b.field[lane_ < kKldBatchMax ? lane_ : 0] : 0xffffffffu;    \
    const int t = __popcll(__ballot(blockIdx.x >= first_)) - 1;                                           \
    const KldBatchItem &it = b.item[t];                                                                   \
    const unsigned l = blockIdx.x - b.field[t]

__global__ void __launch_bounds__(kRangeThreads)
kld_range_batched_kernel(const KldBatch b)
{
    ADAPT_KLD_FIND(first_range);
    kld_range_body(it.w, it.n, reinterpret_cast<float *>(b.ws + it.off_range), BlockGeo{l, 0, (unsigned)it.range_blocks, 1});
}

template <bool WIDE>
__global__ void __launch_bounds__(kHistMaxThreads)
kld_hist_batched_kernel(const KldBatch b)
{
    ADAPT_KLD_FIND(first_hist);
    const int rows = b.wl_hi - b.wl_lo + 2;
    kld_hist_body<true, WIDE>(it.w, it.n, it.range ? it.range : reinterpret_cast<const float *>(b.ws + it.off_range),
                        it.range ? 1 : it.range_blocks, b.wl_lo, b.wl_hi,
                        it.il, it.bins, reinterpret_cast<KldPlan *>(b.ws + it.off_plan),
                        reinterpret_cast<uint32_t *>(b.ws + it.off_klpart), reinterpret_cast<uint32_t *>(b.ws + it.off_slabs), rows,
                        it.rows_per_group, b.mode, b.seed, it.stream,
                        BlockGeo{l % (unsigned)it.hist_x, l / (unsigned)it.hist_x, (unsigned)it.hist_x, (unsigned)it.groups});
}

__global__ void __launch_bounds__(kChunk)
kld_sum_batched_kernel(const KldBatch b)
{
    ADAPT_KLD_FIND(first_sum);
    const int ncand = b.wl_hi - b.wl_lo + 1;
    kld_sum_body(reinterpret_cast<const KldPlan *>(b.ws + it.off_plan), reinterpret_cast<const uint32_t *>(b.ws + it.off_slabs),
                 it.hist_x, ncand + 1, it.bins, kl_region(b.ws + it.off_klpart, ncand, it.nchunks).sums, nullptr,
                 BlockGeo{l % (unsigned)it.nchunks, l / (unsigned)it.nchunks, (unsigned)it.nchunks, (unsigned)(ncand + 1)});
}

__global__ void __launch_bounds__(kChunk)
kld_final_batched_kernel(const KldBatch b)
{
    ADAPT_KLD_FIND(first_final);
    const int ncand = b.wl_hi - b.wl_lo + 1;
    kld_final_body(reinterpret_cast<const KldPlan *>(b.ws + it.off_plan), ncand + 1, it.bins, b.alpha,
                   kl_region(b.ws + it.off_klpart, ncand, it.nchunks), b.wl_lo, it.il, b.eps, it.kld, it.sel, nullptr,
                   BlockGeo{l % (unsigned)it.nchunks, l / (unsigned)it.nchunks, (unsigned)it.nchunks, (unsigned)b.final_y});
}

static int search_one(adapt_ctx *ctx, const float *w, uint64_t n, int wl_lo, int wl_hi, int il, int bins, double eps,
                      double alpha, int mode, uint64_t seed, uint64_t stream, double *kld, int32_t *sel,
                      uint32_t *hist, int64_t *grid, const float *range = nullptr /* device (min, max) or null */)
{
    const int ncand = wl_hi - wl_lo + 1;
    const int rows = ncand + 1;
    // small tensors: many small blocks; large tensors: one big block per CU (more wavefronts share
    // one set of LDS histograms)
    const int threads = n >= ((uint64_t)1 << 20) ? 1024 : n >= ((uint64_t)1 << 16) ? 512 : 256;
    const uint64_t per_block = (uint64_t)threads * 8;
    const int hist_grid = (int)std::min<uint64_t>((uint64_t)ctx->num_cu, std::max<uint64_t>(1, (n + per_block - 1) / per_block));
    // workspace: plan | range partials | KL partials | slabs
    char *ws = scratch(ctx);
    const int nchunks = (bins + kChunk - 1) / kChunk;
    const size_t klpart_bytes = kl_region_bytes(ncand, nchunks, bins);
    const size_t plan_bytes = (sizeof(KldPlan) + 255) & ~(size_t)255;
    const int range_grid = (int)std::min<uint64_t>((uint64_t)ctx->num_cu * 4, std::max<uint64_t>(1, (n / 4 + kRangeThreads - 1) / kRangeThreads));
    const size_t partial_bytes = ((size_t)range_grid * 8 + 255) & ~(size_t)255;
    const size_t hist_words = (size_t)rows * bins;
    const size_t need = plan_bytes + partial_bytes + klpart_bytes + (size_t)hist_grid * hist_words * 4;
    if (need > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    KldPlan *plan = reinterpret_cast<KldPlan *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan_bytes);
    char *klpart = ws + plan_bytes + partial_bytes;
    uint32_t *slabs = reinterpret_cast<uint32_t *>(ws + plan_bytes + partial_bytes + klpart_bytes);

    // a range the caller already holds (from the pass that produced the tensor) stands in for the
    // range partials: one pair
    const float *range_src = range ? range : partial;
    const int range_count = range ? 1 : range_grid;
    if (!range) hipLaunchKernelGGL(kld_range_kernel, dim3(range_grid), dim3(kRangeThreads), 0, ctx->stream, w, n, partial);

    const size_t row_bytes = (size_t)bins * 4;
    // a row plus, for a candidate counted by code, its private table
    const size_t per_row = row_bytes + kPrivWords * 4;
    if (per_row + 16 <= kLdsBudget) {
        // rows per block: as many as LDS holds, fewer when the tensor alone cannot fill the GPU
        int rows_per_group = (int)std::min<size_t>(rows, kLdsBudget / per_row);
        const int want_groups = std::max(1, (2 * ctx->num_cu + hist_grid - 1) / hist_grid);
        rows_per_group = std::max(1, std::min(rows_per_group, (rows + want_groups - 1) / want_groups));
        const int groups = (rows + rows_per_group - 1) / rows_per_group;
        // one set of LDS histograms per block: per-wavefront replicas were measured no faster
        const size_t lds = (size_t)rows_per_group * per_row + 16;
        if (wl_hi > 16)
            hipLaunchKernelGGL((kld_hist_kernel<true, true>), dim3(hist_grid, groups), dim3(threads), lds, ctx->stream, w, n, range_src,
                               range_count, wl_lo, wl_hi, il, bins, plan, reinterpret_cast<uint32_t *>(klpart), slabs, rows, rows_per_group,
                               mode, seed, stream);
        else
            hipLaunchKernelGGL((kld_hist_kernel<true, false>), dim3(hist_grid, groups), dim3(threads), lds, ctx->stream, w, n, range_src,
                               range_count, wl_lo, wl_hi, il, bins, plan, reinterpret_cast<uint32_t *>(klpart), slabs, rows, rows_per_group,
                               mode, seed, stream);
    } else {
        const size_t zw = (size_t)hist_grid * hist_words;
        hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)std::min<size_t>((zw + 255) / 256, (size_t)ctx->num_cu * 8)),
                           dim3(256), 0, ctx->stream, slabs, zw);
        if (wl_hi > 16)
            hipLaunchKernelGGL((kld_hist_kernel<false, true>), dim3(hist_grid, 1), dim3(threads), 0, ctx->stream, w, n, range_src, range_count,
                               wl_lo, wl_hi, il, bins, plan, reinterpret_cast<uint32_t *>(klpart), slabs, rows, rows, mode, seed, stream);
        else
            hipLaunchKernelGGL((kld_hist_kernel<false, false>), dim3(hist_grid, 1), dim3(threads), 0, ctx->stream, w, n, range_src, range_count,
                               wl_lo, wl_hi, il, bins, plan, reinterpret_cast<uint32_t *>(klpart), slabs, rows, rows, mode, seed, stream);
    }
    hipLaunchKernelGGL(kld_sum_kernel, dim3(nchunks, rows), dim3(kChunk), 0, ctx->stream, plan, slabs, hist_grid, rows, bins, klpart,
                       hist);
    hipLaunchKernelGGL(kld_final_kernel, dim3(nchunks, ncand), dim3(kChunk), 0, ctx->stream, plan, rows, bins, alpha, klpart, wl_lo, il,
                       eps, kld, sel, reinterpret_cast<long long *>(grid));
    return hip_status(ctx, hipGetLastError());
}

static int check_search_args(int wl_lo, int wl_hi, int il, int bins, double eps, double alpha, int mode)
{
    if (wl_lo < 2 || wl_hi > 32 || wl_lo > wl_hi) return ADAPT_EINVAL;
    if (il < 1 || wl_lo - il < 0 || wl_hi - il > 31) return ADAPT_EINVAL;
    if (bins < 2 || bins > 65536) return ADAPT_EINVAL;
    if (mode != ADAPT_SR && mode != ADAPT_RN_HALF_UP) return ADAPT_EINVAL;
    if (eps != eps || alpha != alpha) return ADAPT_EINVAL;
    return ADAPT_OK;
}

static hipError_t allow_hist_lds(adapt_ctx *ctx)
{
    hipError_t e = allow_big_lds(ctx, reinterpret_cast<const void *>(&kld_hist_kernel<true, false>), kLdsBudget);
    if (e == hipSuccess) e = allow_big_lds(ctx, reinterpret_cast<const void *>(&kld_hist_kernel<true, true>), kLdsBudget);
    if (e == hipSuccess) e = allow_big_lds(ctx, reinterpret_cast<const void *>(&kld_hist_batched_kernel<false>), kLdsBudget);
    if (e == hipSuccess) e = allow_big_lds(ctx, reinterpret_cast<const void *>(&kld_hist_batched_kernel<true>), kLdsBudget);
    return e;
}

// Searches on items[0 .. count): consecutive tensors are packed into batches (at most kKldBatchMax
// tensors, as many as the workspace holds) that run their three phases in one launch each; a tensor
// whose histogram rows do not fit LDS takes the single-tensor path.
static int search_batch(adapt_ctx *ctx, const adapt_kld_item *items, const float *const *ranges, int count, int wl_lo, int wl_hi,
                        double eps, double alpha, int mode, uint64_t seed, double *kld, int32_t *sel)
{
    const int ncand = wl_hi - wl_lo + 1, rows = ncand + 1;
    auto a256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    int t0 = 0;
    while (t0 < count) {
        const size_t per_row0 = (size_t)items[t0].bins * 4 + kPrivWords * 4;
        if (per_row0 + 16 > kLdsBudget) {
            const int st = search_one(ctx, items[t0].w, items[t0].n, wl_lo, wl_hi, items[t0].il, items[t0].bins, eps, alpha, mode,
                                      seed, items[t0].stream, kld + (size_t)t0 * ncand, sel + 2 * t0, nullptr, nullptr,
                                      ranges ? ranges[t0] : nullptr);
            if (st != ADAPT_OK) return st;
            ++t0;
            continue;
        }
        // block size of the histogram launch: large blocks when the batch holds a large tensor
        int threads = 512;
        for (int m = 0; m < kKldBatchMax && t0 + m < count; ++m)
            if (items[t0 + m].n >= ((uint64_t)1 << 20)) threads = 1024;
        KldBatch b;
        b.count = 0; b.wl_lo = wl_lo; b.wl_hi = wl_hi; b.mode = mode; b.seed = seed; b.eps = eps; b.alpha = alpha;
        b.ws = scratch(ctx);
        size_t off = 0, lds_max = 0;
        unsigned nr = 0, nh = 0, nsum = 0, nf = 0;
        // The batch as a whole fills the GPU once (a full set of rows leaves room for one block per CU): every block
        // clears and flushes its histogram rows, and the final phase reads the slabs back, so a tensor gets blocks
        // in proportion to its share of the elements rather than as many as it could use alone.
        uint64_t batch_elems = 0, batch_blocks = 0;
        const uint64_t per_block = (uint64_t)threads * 8;
        for (int m = 0; m < kKldBatchMax && t0 + m < count; ++m) batch_elems += items[t0 + m].n;
        // a chunk's candidates share a block when the batch is large (see kld_final_body)
        b.final_y = batch_elems >= ((uint64_t)1 << 21) ? 1 : ncand;
        // the launch ends with its most loaded block: no block takes more than `load` elements, and `load` is chosen so
        // that the blocks of all tensors (each rounded up) still number at most one per CU
        int batch_count = 0;
        for (int m = 0; m < kKldBatchMax && t0 + m < count; ++m) ++batch_count;
        const uint64_t spare = (uint64_t)std::max(1, ctx->num_cu - batch_count);
        const uint64_t load = std::max<uint64_t>(1, (batch_elems + spare - 1) / spare);
        auto blocks_of = [&](uint64_t n) {
            const uint64_t by_size = std::max<uint64_t>(1, (n + per_block - 1) / per_block);
            const uint64_t by_share = std::max<uint64_t>(1, (n + load - 1) / load);
            return (int)std::min<uint64_t>((uint64_t)ctx->num_cu, std::min(by_size, by_share));
        };
        for (int m = 0; m < kKldBatchMax && t0 + m < count; ++m) batch_blocks += (uint64_t)blocks_of(items[t0 + m].n);
        // Every group of rows repeats the per-element work that the rows share (rounding bits, scaled values), so the rows
        // are split over several blocks only when the batch leaves CUs idle.
        const int want_groups = (int)std::max<uint64_t>(1, (2 * (uint64_t)ctx->num_cu + batch_blocks - 1) / std::max<uint64_t>(batch_blocks, 1));
        while (b.count < kKldBatchMax && t0 + b.count < count) {
            const adapt_kld_item &src = items[t0 + b.count];
            const size_t row_bytes = (size_t)src.bins * 4, per_row = row_bytes + kPrivWords * 4;
            if (per_row + 16 > kLdsBudget) break;
            KldBatchItem it;
            it.w = src.w; it.n = src.n; it.stream = src.stream; it.il = src.il; it.bins = src.bins;
            it.range = ranges ? ranges[t0 + b.count] : nullptr;
            it.kld = kld + (size_t)(t0 + b.count) * ncand;
            it.sel = sel + 2 * (t0 + b.count);
            it.hist_x = blocks_of(src.n);
            it.range_blocks = it.range ? 0 : (int)std::min<uint64_t>((uint64_t)ctx->num_cu * 4, std::max<uint64_t>(1, (src.n / 4 + kRangeThreads - 1) / kRangeThreads));
            it.nchunks = (src.bins + kChunk - 1) / kChunk;
            int rpg = (int)std::min<size_t>(rows, kLdsBudget / per_row);
            rpg = std::max(1, std::min(rpg, (rows + want_groups - 1) / want_groups));      // a small batch splits the candidates
            it.rows_per_group = rpg;
            it.groups = (rows + rpg - 1) / rpg;
            const size_t need = a256(sizeof(KldPlan)) + a256((size_t)it.range_blocks * 8) + kl_region_bytes(ncand, it.nchunks, src.bins) +
                                a256((size_t)it.hist_x * rows * src.bins * 4);
            if (off + need > scratch_bytes(ctx)) {
                if (b.count == 0) return ADAPT_EWORKSPACE;
                break;
            }
            it.off_plan = off;
            it.off_range = it.off_plan + a256(sizeof(KldPlan));
            it.off_klpart = it.off_range + a256((size_t)it.range_blocks * 8);
            it.off_slabs = it.off_klpart + kl_region_bytes(ncand, it.nchunks, src.bins);
            off += need;
            b.first_range[b.count] = nr; b.first_hist[b.count] = nh; b.first_sum[b.count] = nsum; b.first_final[b.count] = nf;
            nr += (unsigned)it.range_blocks;
            nh += (unsigned)(it.hist_x * it.groups);
            nsum += (unsigned)(it.nchunks * rows);
            nf += (unsigned)(it.nchunks * b.final_y);
            lds_max = std::max(lds_max, (size_t)rpg * per_row + 16);
            b.item[b.count++] = it;
        }
        for (int i = b.count; i < kKldBatchMax; ++i) { b.first_range[i] = b.first_hist[i] = b.first_sum[i] = b.first_final[i] = 0xffffffffu; }
        if (nr) hipLaunchKernelGGL(kld_range_batched_kernel, dim3(nr), dim3(kRangeThreads), 0, ctx->stream, b);
        if (wl_hi > 16) hipLaunchKernelGGL(kld_hist_batched_kernel<true>, dim3(nh), dim3(threads), lds_max, ctx->stream, b);
        else hipLaunchKernelGGL(kld_hist_batched_kernel<false>, dim3(nh), dim3(threads), lds_max, ctx->stream, b);
        hipLaunchKernelGGL(kld_sum_batched_kernel, dim3(nsum), dim3(kChunk), 0, ctx->stream, b);
        hipLaunchKernelGGL(kld_final_batched_kernel, dim3(nf), dim3(kChunk), 0, ctx->stream, b);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return hip_status(ctx, e);
        t0 += b.count;
    }
    return ADAPT_OK;
}

// upper bounds of what search_one / one batch of search_batch lay out in the scratch
static size_t need_of_tensor(int num_cu, uint64_t n, int ncand, int bins)
{
    auto a256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    const int threads = n >= ((uint64_t)1 << 20) ? 1024 : n >= ((uint64_t)1 << 16) ? 512 : 256;
    const uint64_t per_block = (uint64_t)threads * 8;
    const uint64_t hist_grid = std::min<uint64_t>((uint64_t)num_cu, std::max<uint64_t>(1, (n + per_block - 1) / per_block));
    const uint64_t range_grid = std::min<uint64_t>((uint64_t)num_cu * 4, std::max<uint64_t>(1, (n / 4 + kRangeThreads - 1) / kRangeThreads));
    const size_t nchunks = (size_t)(bins + kChunk - 1) / kChunk;
    return a256(sizeof(KldPlan)) + a256((size_t)range_grid * 8) + kl_region_bytes(ncand, (int)nchunks, bins) +
           a256((size_t)hist_grid * (size_t)(ncand + 1) * (size_t)bins * 4);
}

size_t ws_need_kld_search(int num_cu, uint64_t n, int wl_lo, int wl_hi, int bins)
{
    return need_of_tensor(num_cu, n, wl_hi - wl_lo + 1, bins);
}

size_t ws_need_kld_search_batched(int num_cu, const adapt_kld_item *items, int count, int wl_lo, int wl_hi)
{
    size_t worst = 0;
    for (int t0 = 0; t0 < count; t0 += kKldBatchMax) {
        size_t sum = 0;
        for (int t = t0; t < count && t < t0 + kKldBatchMax; ++t) sum += need_of_tensor(num_cu, items[t].n, wl_hi - wl_lo + 1, items[t].bins);
        worst = std::max(worst, sum);
    }
    return worst;
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
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if (((uintptr_t)kld & 7) || ((uintptr_t)sel & 3) || ((uintptr_t)hist & 3) || ((uintptr_t)grid & 7)) return ADAPT_EINVAL;
    if (hipError_t e = allow_hist_lds(ctx); e != hipSuccess) return hip_status(ctx, e);
    return search_one(ctx, w, n, wl_lo, wl_hi, il, bins, eps, alpha, rng.mode, rng.seed, rng.stream, kld, sel, hist, grid);
}

extern "C" int adapt_kld_precision_search_ranged(adapt_ctx *ctx, const float *w, size_t n, const float *range, int wl_lo,
                                                 int wl_hi, int il, int bins, double eps, double alpha, adapt_rng rng,
                                                 double *kld, int32_t *sel, uint32_t *hist, int64_t *grid)
{
    if (!ctx || !kld || !sel || !range || ((uintptr_t)range & 3)) return ADAPT_EINVAL;
    if (int s = check_search_args(wl_lo, wl_hi, il, bins, eps, alpha, rng.mode)) return s;
    if (n > 0 && (!w || !aligned16(w))) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if (((uintptr_t)kld & 7) || ((uintptr_t)sel & 3) || ((uintptr_t)hist & 3) || ((uintptr_t)grid & 7)) return ADAPT_EINVAL;
    if (hipError_t e = allow_hist_lds(ctx); e != hipSuccess) return hip_status(ctx, e);
    return search_one(ctx, w, n, wl_lo, wl_hi, il, bins, eps, alpha, rng.mode, rng.seed, rng.stream, kld, sel, hist, grid, range);
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
        if (items[t].n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    }
    if (hipError_t e = allow_hist_lds(ctx); e != hipSuccess) return hip_status(ctx, e);
    return search_batch(ctx, items, nullptr, count, wl_lo, wl_hi, eps, alpha, mode, seed, kld, sel);
}

extern "C" int adapt_kld_precision_search_batched_ranged(adapt_ctx *ctx, const adapt_kld_item *items, const float *const *ranges,
                                                         int count, int wl_lo, int wl_hi, double eps, double alpha, int mode,
                                                         uint64_t seed, double *kld, int32_t *sel)
{
    if (!ctx || count < 0 || (count > 0 && (!items || !ranges || !kld || !sel))) return ADAPT_EINVAL;
    if (((uintptr_t)kld & 7) || ((uintptr_t)sel & 3)) return ADAPT_EINVAL;
    for (int t = 0; t < count; ++t) {
        if (int s = check_search_args(wl_lo, wl_hi, items[t].il, items[t].bins, eps, alpha, mode)) return s;
        if (items[t].n > 0 && (!items[t].w || !aligned16(items[t].w))) return ADAPT_EINVAL;
        if (items[t].n > ((uint64_t)1 << 40) || ((uintptr_t)ranges[t] & 3)) return ADAPT_EINVAL;
    }
    if (hipError_t e = allow_hist_lds(ctx); e != hipSuccess) return hip_status(ctx, e);
    return search_batch(ctx, items, ranges, count, wl_lo, wl_hi, eps, alpha, mode, seed, kld, sel);
}
