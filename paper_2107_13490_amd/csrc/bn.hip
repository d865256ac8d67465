// Fixed-point batch normalisation, global average pooling and the merge of two gradient tensors: the
// element-wise steps that the chained training step (Alg. 1) needs on the residual networks of
// Sec. 4.1.  The paper does not say how these are done on fixed-point codes; the rules implemented:
//
//   forward    per channel k over the m rows of the convolution output y (codes, NHWC so a row is one
//              position): S1 = sum y, S2 = sum y^2 as exact integers; mean = S1/m,
//              var = max(S2/m - mean*mean, 0), sig = sqrt(var + eps 4^FL_y), alpha = gamma 2^FL_o / sig,
//              off = beta 2^FL_o - mean alpha in fp64 (one correctly rounded operation at a time, no
//              contraction); FA = clamp(30 - E, 0, 30) with max |alpha| = f 2^E, 1/2 <= f < 1;
//              A = rint(alpha 2^FA) (|A| <= 2^30), B = rint(off 2^FA) (|B| <= 2^61);
//              out = requantize(A y + B [+ shortcut on that grid], FA) to <WL_o,FL_o>, SR, optional ReLU
//   backward   D1 = sum dz, D2 = sum dz y (exact); dgamma = (D2 - mean D1)/sig, dbeta = D1;
//              c1 = D1/m, c2 = dgamma/(m sig); P = alpha, Q = -(alpha c2), R = alpha (mean c2 - c1);
//              FB from max(|P|,|Q|) like FA; exact acc = P^ dz + Q^ y + R^ stored in WL bits with the
//              fitting shift: exponent e + FB - shift + FL_o - FL_y
//   update     gamma and beta each step against their gradient divided by its 2-norm over the channels
//              (the rule of Sec. 3.3 "Dealing with Fixed-Points Limited Range" for weights)
//   pooling    mean over the h*w (a power of two) positions: integer sum, requantize by log2(h*w)
//   merge      exact sum of two gradient tensors on the finer of their grids, fitting shift; exponents
//              more than 40 apart: the far smaller tensor is left out
//
// All element-wise kernels read every input once and write every output once in 8- or 16-byte accesses
// (HBM-bound); the statistics kernels keep a thread's eight channels in registers when the channel count
// divides the thread stride, and fall back to LDS atomics otherwise.
#include <algorithm>
#include <cmath>

#include "common.hpp"
#include "context.hpp"
#include "fit.hpp"
#include "update_batch.hpp"
#include "wide.hpp"

// every fp64 operation of the coefficient kernels is rounded on its own: no fused multiply-adds
#pragma clang fp contract(off)

namespace adapt {

constexpr int kBnThreads = 256;
constexpr int kBnMaxChannels = 4096;

struct BnHeader {
    int32_t channels, fl_y, fl_o, fa, fb, pad[3];
    unsigned long long rows;
};
constexpr size_t kBnHeaderBytes = 64;
static_assert(sizeof(BnHeader) <= kBnHeaderBytes, "header");

// state: header | mean[K] sig[K] alpha[K] (fp64) | B[K] R[K] (int64) | A[K] P[K] Q[K] (int32)
struct BnState {
    BnHeader *h;
    double *mean, *sig, *alpha;
    long long *B, *R;
    int32_t *A, *P, *Q;
};
__host__ __device__ inline size_t bn_state_bytes(int k) { return kBnHeaderBytes + (size_t)k * (3 * 8 + 2 * 8 + 3 * 4); }
__host__ __device__ inline BnState bn_state(void *p, int k)
{
    char *c = static_cast<char *>(p);
    BnState s;
    s.h = reinterpret_cast<BnHeader *>(c);
    s.mean = reinterpret_cast<double *>(c + kBnHeaderBytes);
    s.sig = s.mean + k;
    s.alpha = s.sig + k;
    s.B = reinterpret_cast<long long *>(s.alpha + k);
    s.R = s.B + k;
    s.A = reinterpret_cast<int32_t *>(s.R + k);
    s.P = s.A + k;
    s.Q = s.P + k;
    return s;
}

// ---- per-channel sums -----------------------------------------------------------------------------------
// MODE 0: (sum y, sum y^2); MODE 1: (sum dz, sum dz*y).  One group = 8 consecutive elements = 8 consecutive
// channels of one row (channels % 8 == 0).  REG: the thread stride in groups is a multiple of channels/8, so a
// thread meets the same eight channels every time and sums them in registers.
template <typename TA, typename TB, int MODE, bool REG>
__global__ void __launch_bounds__(kBnThreads)
bn_sums_kernel(const TA *__restrict__ a, const TB *__restrict__ b, uint64_t groups, int channels, long long *__restrict__ partial)
{
    extern __shared__ long long lsum[];          // [2 * channels]
    for (int i = threadIdx.x; i < 2 * channels; i += kBnThreads) lsum[i] = 0;
    __syncthreads();
    const uint32_t cg = (uint32_t)channels >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kBnThreads;
    if (REG) {
        long long s1[8], s2[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0;
        for (uint64_t g = first; g < groups; g += stride) {
            int x[8], y[8];
            load_codes8<TA>(a, g, x);
            if (MODE == 1) load_codes8<TB>(b, g, y);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s1[e] += x[e];
                s2[e] += (long long)(MODE == 1 ? x[e] * y[e] : x[e] * x[e]);
            }
        }
        if (first < groups) {
            const uint32_t c0 = (uint32_t)(first % cg) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                atomicAdd(reinterpret_cast<unsigned long long *>(&lsum[c0 + e]), (unsigned long long)s1[e]);
                atomicAdd(reinterpret_cast<unsigned long long *>(&lsum[channels + c0 + e]), (unsigned long long)s2[e]);
            }
        }
    } else {
        for (uint64_t g = first; g < groups; g += stride) {
            int x[8], y[8];
            load_codes8<TA>(a, g, x);
            if (MODE == 1) load_codes8<TB>(b, g, y);
            const uint32_t c0 = (uint32_t)(g % cg) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                atomicAdd(reinterpret_cast<unsigned long long *>(&lsum[c0 + e]), (unsigned long long)(long long)x[e]);
                atomicAdd(reinterpret_cast<unsigned long long *>(&lsum[channels + c0 + e]),
                          (unsigned long long)(long long)(MODE == 1 ? x[e] * y[e] : x[e] * x[e]));
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * channels; i += kBnThreads) partial[(size_t)blockIdx.x * 2 * channels + i] = lsum[i];
}

// clamp(30 - E, 0, 30) for vmax = f 2^E, 1/2 <= f < 1; 30 for vmax = 0 or infinite
__device__ inline int coef_exponent(double vmax)
{
    if (!(vmax > 0.0) || vmax == (double)INFINITY) return 30;
    int e;
    (void)frexp(vmax, &e);
    return min(max(30 - e, 0), 30);
}

__device__ inline long long rint_clamped(double v, int sh, double lim)
{
    const double t = rint(ldexp(v, sh));
    return (long long)fmin(fmax(t, -lim), lim);      // NaN -> -lim (the callers' inputs are finite)
}

// block-wide maximum of doubles >= 0 (all threads get it)
__device__ inline double block_max_f64(double v, double *sm)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & (kWave - 1)) == 0) sm[threadIdx.x / kWave] = v;
    __syncthreads();
    v = sm[0];
    for (int i = 1; i < (int)blockDim.x / kWave; ++i) v = fmax(v, sm[i]);
    __syncthreads();
    return v;
}

// The totals may have been written by other blocks of the same launch (the merged totals + coefficients kernels):
// they are read at device scope, past this compute unit's cache.
__device__ __forceinline__ long long total_at(const long long *tot, int i)
{
    return __hip_atomic_load(tot + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One block: statistics and forward coefficients from the totals.
__device__ __forceinline__ void bn_coef_fwd_body(const long long *tot /* [2 * channels] */, int channels, unsigned long long rows, int fl_y,
                                                 int fl_o, const float *__restrict__ gamma, const float *__restrict__ beta, double eps,
                                                 void *state, const double *__restrict__ s2d)
{
    __shared__ double sm[16];
    const BnState st = bn_state(state, channels);
    const double m = (double)rows;
    double amax = 0.0;
    for (int k = threadIdx.x; k < channels; k += blockDim.x) {
        const long long s1 = total_at(tot, k);
        const double mean = (double)s1 / m;
        const double ex2 = (s2d ? s2d[k] : (double)total_at(tot, channels + k)) / m;
        const double var = fmax(ex2 - mean * mean, 0.0);
        const double sig = sqrt(var + ldexp(eps, 2 * fl_y));
        const double alpha = ldexp((double)gamma[k], fl_o) / sig;
        st.mean[k] = mean;
        st.sig[k] = sig;
        st.alpha[k] = alpha;
        amax = fmax(amax, fabs(alpha));
    }
    amax = block_max_f64(amax, sm);
    const int fa = coef_exponent(amax);
    for (int k = threadIdx.x; k < channels; k += blockDim.x) {
        const double alpha = st.alpha[k];
        const double off = ldexp((double)beta[k], fl_o) - st.mean[k] * alpha;
        st.A[k] = (int32_t)rint_clamped(alpha, fa, 1073741824.0);
        st.B[k] = rint_clamped(off, fa, 2305843009213693952.0);
    }
    if (threadIdx.x == 0) {
        st.h->channels = channels; st.h->fl_y = fl_y; st.h->fl_o = fl_o; st.h->fa = fa; st.h->fb = 0; st.h->rows = rows;
    }
}

__global__ void __launch_bounds__(1024)
bn_coef_fwd_kernel(const long long *tot, int channels, unsigned long long rows, int fl_y, int fl_o, const float *__restrict__ gamma,
                   const float *__restrict__ beta, double eps, void *state,
                   const double *__restrict__ s2d = nullptr /* sums of squares beyond 64 bits, as their nearest doubles */)
{
    bn_coef_fwd_body(tot, channels, rows, fl_y, fl_o, gamma, beta, eps, state, s2d);
}

// One block: from the totals of (sum dz, sum dz*y) the parameter gradients and the backward coefficients.
__device__ __forceinline__ void bn_coef_bwd_body(const long long *tot /* [2 * channels] */, int channels, void *state,
                                                 double *__restrict__ dgamma, double *__restrict__ dbeta, const double *__restrict__ d2d)
{
    __shared__ double sm[16];
    const BnState st = bn_state(state, channels);
    const double m = (double)st.h->rows;
    double pmax = 0.0;
    for (int k = threadIdx.x; k < channels; k += blockDim.x) {
        const long long d1 = total_at(tot, k);
        const double d2 = d2d ? d2d[k] : (double)total_at(tot, channels + k);
        const double mean = st.mean[k], sig = st.sig[k], alpha = st.alpha[k];
        const double dg = (d2 - mean * (double)d1) / sig;
        const double c1 = (((double)d1) / (m));
        const double c2 = dg / (m * sig);
        const double q = -((alpha) * (c2));
        const double r = alpha * (mean * c2 - c1);
        dgamma[k] = dg;
        dbeta[k] = (double)d1;
        // Q and R wait in the slots of their codes until the common exponent is known
        reinterpret_cast<double *>(st.R)[k] = r;
        reinterpret_cast<double *>(st.B)[k] = q;       // B is not needed after the forward pass
        pmax = fmax(pmax, fmax(fabs(alpha), fabs(q)));
    }
    pmax = block_max_f64(pmax, sm);
    const int fb = coef_exponent(pmax);
    for (int k = threadIdx.x; k < channels; k += blockDim.x) {
        const double q = reinterpret_cast<const double *>(st.B)[k], r = reinterpret_cast<const double *>(st.R)[k];
        st.P[k] = (int32_t)rint_clamped(st.alpha[k], fb, 1073741824.0);
        st.Q[k] = (int32_t)rint_clamped(q, fb, 1073741824.0);
        st.R[k] = rint_clamped(r, fb, 2305843009213693952.0);
    }
    if (threadIdx.x == 0) st.h->fb = fb;
}

__global__ void __launch_bounds__(1024)
bn_coef_bwd_kernel(const long long *tot, int channels, void *state, double *__restrict__ dgamma, double *__restrict__ dbeta,
                   const double *__restrict__ d2d = nullptr /* sums of products beyond 64 bits */)
{
    bn_coef_bwd_body(tot, channels, state, dgamma, dbeta, d2d);
}

// Totals and coefficients in one launch.  Totals of the block partials partial[nparts][2 * channels] of a statistics
// launch: a block takes 8 columns, 32 threads per column each add every 32nd partial (independent loads), LDS
// combines them.  The block that finishes last (a ticket, zero before the launch and zero again after it) goes on
// with the coefficients.
struct BnCoefArgs {
    int channels, fl_y, fl_o;
    unsigned long long rows;
    const float *gamma, *beta;
    double eps;
    void *state;
    double *dgamma, *dbeta;
};

template <bool BWD>
__global__ void __launch_bounds__(256)
bn_total_coef_kernel(const long long *__restrict__ partial, int nparts, long long *totals, uint32_t *ticket, const BnCoefArgs c)
{
    __shared__ long long sm[32][8];
    __shared__ bool last;
    const int width = 2 * c.channels;
    const int col8 = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int col = blockIdx.x * 8 + col8;
    long long acc = 0;
    if (col < width)
        for (int r = rl; r < nparts; r += 32) acc += partial[(size_t)r * width + col];
    sm[rl][col8] = acc;
    __syncthreads();
    if (threadIdx.x < 8 && col < width) {
        long long t = 0;
#pragma unroll
        for (int i = 0; i < 32; ++i) t += sm[i][threadIdx.x];
        __hip_atomic_store(totals + col, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();                               // the block's totals are issued before its ticket
    if (threadIdx.x == 0) {
        // release this block's totals, acquire everyone else's
        last = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
        if (last) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);      // for the next launch
    }
    __syncthreads();
    if (!last) return;
    if (BWD) bn_coef_bwd_body(totals, c.channels, c.state, c.dgamma, c.dbeta, nullptr);
    else bn_coef_fwd_body(totals, c.channels, c.rows, c.fl_y, c.fl_o, c.gamma, c.beta, c.eps, c.state, nullptr);
}

// ---- forward: out = requantize(A y + B [+ shortcut], FA) ---------------------------------------------------
struct BnApplyArgs {
    const void *y, *res;
    void *out;
    const void *state;
    uint64_t groups;
    int channels, wl, relu, mode, has_res, fl_res;
    uint64_t seed, stream;
};

template <typename TY, typename TR, typename TO>
__global__ void __launch_bounds__(kBnThreads) bn_apply_kernel(const BnApplyArgs a)
{
    extern __shared__ long long coef[];          // B[channels] then A[channels] (int32)
    const BnState st = bn_state(const_cast<void *>(a.state), a.channels);
    int32_t *la = reinterpret_cast<int32_t *>(coef + a.channels);
    for (int i = threadIdx.x; i < a.channels; i += kBnThreads) { coef[i] = st.B[i]; la[i] = st.A[i]; }
    __syncthreads();
    const int fa = st.h->fa;
    const int rsh = st.h->fl_o + fa - a.fl_res;                  // alignment of the shortcut: left shift, or floor
    const uint32_t cg = (uint32_t)a.channels >> 3;
    const TY *y = static_cast<const TY *>(a.y);
    const TR *res = static_cast<const TR *>(a.res);
    TO *out = static_cast<TO *>(a.out);
    const uint64_t first = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kBnThreads;
    for (uint64_t g = first; g < a.groups; g += stride) {
        int x[8], s[8], code[8];
        load_codes8<TY>(y, g, x);
        if (a.has_res) load_codes8<TR>(res, g, s);
        uint32_t r[8];
        if (a.mode == ADAPT_SR) {
            const u32x4 blk = rounding_block(a.seed, a.stream, g);
            r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
            r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
        }
        const uint32_t c0 = (uint32_t)(g % cg) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            long long acc = (long long)la[c0 + e] * x[e] + coef[c0 + e];
            if (a.has_res) acc += rsh >= 0 ? (long long)((unsigned long long)(long long)s[e] << rsh) : ((long long)s[e] >> -rsh);
            code[e] = requantize_one(acc, fa, a.wl, a.relu, r[e]);
        }
        store_codes8<TO>(out, g, code);
    }
}

// ---- backward: acc = P dz + Q y + R, fitted ----------------------------------------------------------------
struct BnBwdArgs {
    const void *dz, *y;
    void *dy;
    const void *state;
    uint64_t groups;
    int channels, wl, mode;
    uint64_t seed, stream;
    uint64_t *part;
    int nparts;
    int32_t *shift_out;
    const long long *e_in;
    long long *e_out;
};

template <typename TD, typename TY, typename TO, bool FIT>
__global__ void __launch_bounds__(kBnThreads) bn_bwd_kernel(const BnBwdArgs a)
{
    extern __shared__ long long coef[];          // R[channels], then P[channels], Q[channels] (int32)
    __shared__ uint64_t sm[kBnThreads / kWave];
    const BnState st = bn_state(const_cast<void *>(a.state), a.channels);
    int32_t *lp = reinterpret_cast<int32_t *>(coef + a.channels), *lq = lp + a.channels;
    for (int i = threadIdx.x; i < a.channels; i += kBnThreads) { coef[i] = st.R[i]; lp[i] = st.P[i]; lq[i] = st.Q[i]; }
    int shift = 0;
    if (FIT) {
        uint64_t m = 0;
        for (int i = threadIdx.x; i < a.nparts; i += kBnThreads) m = a.part[i] > m ? a.part[i] : m;
        m = block_max_u64(m, sm, kBnThreads / kWave);
        shift = fit_shift_of(m, a.wl);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.shift_out) *a.shift_out = shift;
            if (a.e_out) *a.e_out = (a.e_in ? *a.e_in : 0) + st.h->fb - shift + st.h->fl_o - st.h->fl_y;
        }
    } else {
        __syncthreads();
    }
    const int qhi = (1 << (a.wl - 1)) - 1, qlo = -(1 << (a.wl - 1));
    const uint32_t cg = (uint32_t)a.channels >> 3;
    const TD *dz = static_cast<const TD *>(a.dz);
    const TY *y = static_cast<const TY *>(a.y);
    TO *dy = static_cast<TO *>(a.dy);
    uint64_t mx = 0;
    const uint64_t first = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kBnThreads;
    for (uint64_t g = first; g < a.groups; g += stride) {
        int d[8], x[8];
        load_codes8<TD>(dz, g, d);
        load_codes8<TY>(y, g, x);
        const uint32_t c0 = (uint32_t)(g % cg) * 8;
        long long acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = (long long)lp[c0 + e] * d[e] + (long long)lq[c0 + e] * x[e] + coef[c0 + e];
        if (!FIT) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t v = magnitude(acc[e]);
                mx = v > mx ? v : mx;
            }
        } else {
            uint32_t r[8];
            if (a.mode == ADAPT_SR) {
                const u32x4 blk = rounding_block(a.seed, a.stream, g);
                r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
                r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = 0x8000u;
            }
            int code[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) code[e] = fit_one(acc[e], shift, r[e], qlo, qhi);
            store_codes8<TO>(dy, g, code);
        }
    }
    if (!FIT) {
        mx = block_max_u64(mx, sm, kBnThreads / kWave);
        if (threadIdx.x == 0) a.part[blockIdx.x] = mx;
    }
}


// ---- word lengths 17..32 (int32 codes) ------------------------------------------------------------------------
// The same rules with wider integers: sums of squares and of products reach 85 bits and are kept in 128, their
// totals enter the fp64 formulas as their nearest doubles; A y + B + shortcut and P dz + Q y + R are formed in 128
// bits.  One element per thread and iteration, storage width chosen at run time: these paths are for correctness
// (a layer that PushUp took above 16 bits), not for speed.
__device__ __forceinline__ long long code_at(const void *p, int es, uint64_t i)
{
    return es == 1 ? (long long)static_cast<const int8_t *>(p)[i] : es == 2 ? (long long)static_cast<const int16_t *>(p)[i]
                                                                            : (long long)static_cast<const int32_t *>(p)[i];
}
__device__ __forceinline__ void code_put(void *p, int es, uint64_t i, int v)
{
    if (es == 1) static_cast<int8_t *>(p)[i] = (int8_t)v;
    else if (es == 2) static_cast<int16_t *>(p)[i] = (int16_t)v;
    else static_cast<int32_t *>(p)[i] = v;
}
// nearest double of a signed 128-bit integer given as two words
__device__ __forceinline__ double i128_to_double(unsigned long long lo, unsigned long long hi)
{
    if (!(hi >> 63)) return u128_to_double(lo, hi);
    const u128 m = (u128)0 - (((u128)hi << 64) | lo);
    return -u128_to_double((unsigned long long)m, (unsigned long long)(m >> 64));
}

// partial[block][channel][4]: first sum, unused, second sum (low word, high word).  A block takes a run of rows.
__global__ void __launch_bounds__(kBnThreads)
bn_sums_wide_kernel(const void *__restrict__ a, int es_a, const void *__restrict__ b, int es_b, int mode, uint64_t rows, int channels,
                    unsigned long long *__restrict__ partial)
{
    const uint64_t per = (rows + gridDim.x - 1) / gridDim.x;
    const uint64_t r0 = (uint64_t)blockIdx.x * per, r1 = r0 + per < rows ? r0 + per : rows;
    for (int c = threadIdx.x; c < channels; c += kBnThreads) {
        long long s1 = 0;
        i128 s2 = 0;
        for (uint64_t r = r0; r < r1; ++r) {
            const long long x = code_at(a, es_a, r * channels + c);
            const long long y = mode == 1 ? code_at(b, es_b, r * channels + c) : x;
            s1 += x;
            s2 += (i128)(x * y);
        }
        unsigned long long *dst = partial + ((size_t)blockIdx.x * channels + c) * 4;
        dst[0] = (unsigned long long)s1;
        dst[1] = 0;
        dst[2] = (unsigned long long)s2;
        dst[3] = (unsigned long long)((u128)s2 >> 64);
    }
}

// totals over the blocks: tot[c] = first sum (64 bits suffice), second[c] = nearest double of the second sum
__global__ void __launch_bounds__(64)
bn_total_wide_kernel(const unsigned long long *__restrict__ partial, int nparts, int channels, long long *__restrict__ tot,
                     double *__restrict__ second)
{
    const int c = blockIdx.x * 64 + threadIdx.x;
    if (c >= channels) return;
    long long s1 = 0;
    i128 s2 = 0;
    for (int p = 0; p < nparts; ++p) {
        const unsigned long long *src = partial + ((size_t)p * channels + c) * 4;
        s1 += (long long)src[0];
        s2 += (i128)(((u128)src[3] << 64) | src[2]);
    }
    tot[c] = s1;
    second[c] = i128_to_double((unsigned long long)s2, (unsigned long long)((u128)s2 >> 64));
}

struct BnWideArgs {
    const void *x, *y;            // forward: y codes, shortcut or null; backward: dz codes, y codes
    void *out;
    const void *state;
    uint64_t n;
    int es_x, es_y, es_o, channels, wl, relu, mode, fl_res;
    uint64_t seed, stream;
    uint64_t *part;
    int nparts;
    int32_t *shift_out;
    const long long *e_in;
    long long *e_out;
};

__global__ void __launch_bounds__(kBnThreads) bn_apply_wide_kernel(const BnWideArgs a)
{
    const BnState st = bn_state(const_cast<void *>(a.state), a.channels);
    const int fa = st.h->fa;
    const int rsh = st.h->fl_o + fa - a.fl_res;
    for (uint64_t i = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kBnThreads) {
        const int c = (int)(i % (uint64_t)a.channels);
        i128 acc = (i128)st.A[c] * (i128)code_at(a.x, a.es_x, i) + (i128)st.B[c];
        if (a.y) {
            const long long s = code_at(a.y, a.es_y, i);
            acc += rsh >= 0 ? (i128)((u128)(i128)s << rsh) : (i128)(s >> (-rsh > 63 ? 63 : -rsh));
        }
        code_put(a.out, a.es_o, i, requantize_wide_one(acc, fa, a.wl, a.relu, rounding_bits_of(a.seed, a.stream, i, a.mode)));
    }
}

// PASS 0: the largest bit length of acc = P dz + Q y + R per block; PASS 1: the fitted codes
template <int PASS>
__global__ void __launch_bounds__(kBnThreads) bn_bwd_wide_kernel(const BnWideArgs a)
{
    __shared__ uint64_t sm[kBnThreads / kWave];
    const BnState st = bn_state(const_cast<void *>(a.state), a.channels);
    int shift = 0;
    if (PASS == 1) {
        uint64_t m = 0;
        for (int i = threadIdx.x; i < a.nparts; i += kBnThreads) m = a.part[i] > m ? a.part[i] : m;
        m = block_max_u64(m, sm, kBnThreads / kWave);
        shift = max(0, (int)m - (a.wl - 1));
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.shift_out) *a.shift_out = shift;
            if (a.e_out) *a.e_out = (a.e_in ? *a.e_in : 0) + st.h->fb - shift + st.h->fl_o - st.h->fl_y;
        }
    }
    uint64_t mx = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kBnThreads) {
        const int c = (int)(i % (uint64_t)a.channels);
        const i128 acc = (i128)st.P[c] * (i128)code_at(a.x, a.es_x, i) + (i128)st.Q[c] * (i128)code_at(a.y, a.es_y, i) + (i128)st.R[c];
        if (PASS == 0) {
            const uint64_t bl = (uint64_t)bit_length_128(acc);
            mx = bl > mx ? bl : mx;
        } else {
            code_put(a.out, a.es_o, i, requantize_wide_one(acc, shift, a.wl, 0, rounding_bits_of(a.seed, a.stream, i, a.mode)));
        }
    }
    if (PASS == 0) {
        mx = block_max_u64(mx, sm, kBnThreads / kWave);
        if (threadIdx.x == 0) a.part[blockIdx.x] = mx;
    }
}

// global average pooling of codes of any width: one thread per (sample, channel)
__global__ void __launch_bounds__(kBnThreads)
gap_fwd_wide_kernel(const void *__restrict__ a, int es, void *__restrict__ out, uint32_t n, uint32_t hw, uint32_t c, int sh, int wl, int mode,
                    uint64_t seed, uint64_t stream)
{
    const uint64_t total = (uint64_t)n * c;
    for (uint64_t i = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; i < total; i += (uint64_t)gridDim.x * kBnThreads) {
        const uint64_t s = i / c, ch = i - s * c;
        i128 acc = 0;
        for (uint32_t p = 0; p < hw; ++p) acc += (i128)code_at(a, es, (s * hw + p) * c + ch);
        code_put(out, es, i, requantize_wide_one(acc, sh, wl, 0, rounding_bits_of(seed, stream, i, mode)));
    }
}

__global__ void __launch_bounds__(kBnThreads)
gap_bwd_wide_kernel(const int32_t *__restrict__ dout, int32_t *__restrict__ da, uint64_t total, uint32_t hw, uint32_t c)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; i < total; i += (uint64_t)gridDim.x * kBnThreads) {
        const uint64_t pos = i / c;
        da[i] = dout[(pos / hw) * c + (i - pos * c)];
    }
}

// ---- update of gamma and beta -------------------------------------------------------------------------------
__device__ __forceinline__ void bn_update_body(float *gamma, float *beta, const double *__restrict__ dgamma,
                                               const double *__restrict__ dbeta, int channels, float lr)
{
    // the squares are formed by all threads, a chunk at a time; the two sums run in channel order (the order fixes
    // the rounding) on one lane each
    constexpr int kChunk = 2048;
    __shared__ double sq[2][kChunk];
    __shared__ double nrm[2];
    const bool summer = (threadIdx.x & 63) == 0 && threadIdx.x < 128;
    double t = 0.0;
    for (int base = 0; base < channels; base += kChunk) {
        const int len = channels - base < kChunk ? channels - base : kChunk;
        for (int k = threadIdx.x; k < len; k += blockDim.x) {
            sq[0][k] = dgamma[base + k] * dgamma[base + k];
            sq[1][k] = dbeta[base + k] * dbeta[base + k];
        }
        __syncthreads();
        if (summer) {
            const double *d = sq[threadIdx.x >> 6];
            int k = 0;
            for (; k + 8 <= len; k += 8) {
                const double v0 = d[k], v1 = d[k + 1], v2 = d[k + 2], v3 = d[k + 3], v4 = d[k + 4], v5 = d[k + 5], v6 = d[k + 6], v7 = d[k + 7];
                t = t + v0; t = t + v1; t = t + v2; t = t + v3; t = t + v4; t = t + v5; t = t + v6; t = t + v7;
            }
            for (; k < len; ++k) t = t + d[k];
        }
        __syncthreads();
    }
    if (summer) nrm[threadIdx.x >> 6] = sqrt(t);
    __syncthreads();
    for (int k = threadIdx.x; k < channels; k += blockDim.x) {
        if (nrm[0] > 0.0 && nrm[0] < (double)INFINITY) gamma[k] = __builtin_fmaf(-lr, (float)((dgamma[k]) / (nrm[0])), gamma[k]);
        if (nrm[1] > 0.0 && nrm[1] < (double)INFINITY) beta[k] = __builtin_fmaf(-lr, (float)((dbeta[k]) / (nrm[1])), beta[k]);
    }
}

__global__ void __launch_bounds__(1024)
bn_update_kernel(float *gamma, float *beta, const double *__restrict__ dgamma, const double *__restrict__ dbeta, int channels, float lr)
{
    bn_update_body(gamma, beta, dgamma, dbeta, channels, lr);
}

// block t: layer t of a chained step
struct BnUpdateBatch {
    BnUpdateItem item[kUpdateMaxItems];
};
__global__ void __launch_bounds__(1024) bn_update_batch_kernel(const BnUpdateBatch b, float lr)
{
    const BnUpdateItem &it = b.item[blockIdx.x];
    bn_update_body(it.gamma, it.beta, it.dgamma, it.dbeta, it.channels, lr);
}

// ---- global average pooling ----------------------------------------------------------------------------------
// out[n, c] = requantize(sum over hw positions, log2 hw); one thread per 8 channels of one sample
template <typename T>
__global__ void __launch_bounds__(kBnThreads)
gap_fwd_kernel(const T *__restrict__ a, T *__restrict__ out, uint32_t n, uint32_t hw, uint32_t cg, int sh, int wl, int mode,
               uint64_t seed, uint64_t stream)
{
    const uint32_t total = n * cg;
    for (uint32_t i = blockIdx.x * kBnThreads + threadIdx.x; i < total; i += gridDim.x * kBnThreads) {
        const uint32_t s = i / cg, c = i - s * cg;
        long long acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0;
        for (uint32_t p = 0; p < hw; ++p) {
            int x[8];
            load_codes8<T>(a, ((uint64_t)s * hw + p) * cg + c, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += x[e];
        }
        int code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) code[e] = requantize_one(acc[e], sh, wl, 0, rounding_bits_of(seed, stream, (uint64_t)i * 8 + e, mode));
        store_codes8<T>(out, i, code);
    }
}

// da[n, p, c] = dout[n, c]
template <typename T>
__global__ void __launch_bounds__(kBnThreads)
gap_bwd_kernel(const T *__restrict__ dout, T *__restrict__ da, uint64_t groups, uint32_t hw, uint32_t cg)
{
    for (uint64_t g = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; g < groups; g += (uint64_t)gridDim.x * kBnThreads) {
        const uint64_t pos = g / cg;
        const uint32_t c = (uint32_t)(g - pos * cg);
        int x[8];
        load_codes8<T>(dout, (pos / hw) * cg + c, x);
        store_codes8<T>(da, g, x);
    }
}

// ---- merge of two gradient tensors ---------------------------------------------------------------------------
struct MergeArgs {
    const void *a, *b;
    void *out;
    const long long *e_a, *e_b;
    long long *e_out;
    int32_t *shift_out;
    uint64_t n;
    int wl, mode;
    uint64_t seed, stream;
    uint64_t *part;
    int nparts;
};

constexpr int kMergeMaxGap = 40;

// alignment of the two tensors: left shifts (or -1: the tensor is left out) and the exponent of the sum
__device__ __forceinline__ void merge_plan(const MergeArgs &a, int &sa, int &sb, long long &e)
{
    const long long ea = a.e_a ? *a.e_a : 0;
    if (!a.b) { sa = 0; sb = -1; e = ea; return; }
    const long long eb = a.e_b ? *a.e_b : 0;
    if (ea - eb > kMergeMaxGap) { sa = -1; sb = 0; e = eb; }
    else if (eb - ea > kMergeMaxGap) { sa = 0; sb = -1; e = ea; }
    else { e = ea > eb ? ea : eb; sa = (int)(e - ea); sb = (int)(e - eb); }
}

template <typename TA, typename TB, typename TO, bool FIT>
__global__ void __launch_bounds__(kBnThreads) merge_kernel(const MergeArgs a)
{
    __shared__ uint64_t sm[kBnThreads / kWave];
    int sa, sb;
    long long e;
    merge_plan(a, sa, sb, e);
    int shift = 0;
    if (FIT) {
        uint64_t m = 0;
        for (int i = threadIdx.x; i < a.nparts; i += kBnThreads) m = a.part[i] > m ? a.part[i] : m;
        m = block_max_u64(m, sm, kBnThreads / kWave);
        shift = fit_shift_of(m, a.wl);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.shift_out) *a.shift_out = shift;
            if (a.e_out) *a.e_out = e - shift;
        }
    }
    const int qhi = (1 << (a.wl - 1)) - 1, qlo = -(1 << (a.wl - 1));
    const TA *pa = static_cast<const TA *>(a.a);
    const TB *pb = static_cast<const TB *>(a.b);
    TO *out = static_cast<TO *>(a.out);
    auto sum_of = [&](int x, int y) {
        long long s = 0;
        if (sa >= 0) s += (long long)((unsigned long long)(long long)x << sa);
        if (sb >= 0) s += (long long)((unsigned long long)(long long)y << sb);
        return s;
    };
    uint64_t mx = 0;
    const uint64_t groups = a.n >> 3;
    const uint64_t first = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kBnThreads;
    for (uint64_t g = first; g < groups; g += stride) {
        int x[8], y[8];
        load_codes8<TA>(pa, g, x);
        if (a.b) load_codes8<TB>(pb, g, y);
        else {
#pragma unroll
            for (int i = 0; i < 8; ++i) y[i] = 0;
        }
        if (!FIT) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint64_t v = magnitude(sum_of(x[i], y[i]));
                mx = v > mx ? v : mx;
            }
        } else {
            uint32_t r[8];
            if (a.mode == ADAPT_SR) {
                const u32x4 blk = rounding_block(a.seed, a.stream, g);
                r[0] = blk.x & 0xffffu; r[1] = blk.x >> 16; r[2] = blk.y & 0xffffu; r[3] = blk.y >> 16;
                r[4] = blk.z & 0xffffu; r[5] = blk.z >> 16; r[6] = blk.w & 0xffffu; r[7] = blk.w >> 16;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = 0x8000u;
            }
            int code[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) code[i] = fit_one(sum_of(x[i], y[i]), shift, r[i], qlo, qhi);
            store_codes8<TO>(out, g, code);
        }
    }
    if ((a.n & 7) && first == 0)
        for (uint64_t i = groups << 3; i < a.n; ++i) {
            const long long s = sum_of((int)pa[i], a.b ? (int)pb[i] : 0);
            if (!FIT) { const uint64_t v = magnitude(s); mx = v > mx ? v : mx; }
            else out[i] = (TO)fit_one(s, shift, rounding_bits_of(a.seed, a.stream, i, a.mode), qlo, qhi);
        }
    if (!FIT) {
        mx = block_max_u64(mx, sm, kBnThreads / kWave);
        if (threadIdx.x == 0) a.part[blockIdx.x] = mx;
    }
}


// the merge for tensors above 16 bits: the aligned sum in 128 bits (a gap of 40 on 32-bit codes passes 64)
template <int PASS>
__global__ void __launch_bounds__(kBnThreads) merge_wide_kernel(const MergeArgs a, int es_a, int es_b, int es_o)
{
    __shared__ uint64_t sm[kBnThreads / kWave];
    int sa, sb;
    long long e;
    merge_plan(a, sa, sb, e);
    int shift = 0;
    if (PASS == 1) {
        uint64_t m = 0;
        for (int i = threadIdx.x; i < a.nparts; i += kBnThreads) m = a.part[i] > m ? a.part[i] : m;
        m = block_max_u64(m, sm, kBnThreads / kWave);
        shift = max(0, (int)m - (a.wl - 1));
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.shift_out) *a.shift_out = shift;
            if (a.e_out) *a.e_out = e - shift;
        }
    }
    uint64_t mx = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kBnThreads + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * kBnThreads) {
        i128 s = 0;
        if (sa >= 0) s += (i128)((u128)(i128)code_at(a.a, es_a, i) << sa);
        if (sb >= 0 && a.b) s += (i128)((u128)(i128)code_at(a.b, es_b, i) << sb);
        if (PASS == 0) {
            const uint64_t bl = (uint64_t)bit_length_128(s);
            mx = bl > mx ? bl : mx;
        } else {
            code_put(a.out, es_o, i, requantize_wide_one(s, shift, a.wl, 0, rounding_bits_of(a.seed, a.stream, i, a.mode)));
        }
    }
    if (PASS == 0) {
        mx = block_max_u64(mx, sm, kBnThreads / kWave);
        if (threadIdx.x == 0) a.part[blockIdx.x] = mx;
    }
}

static int bn_grid(const adapt_ctx *ctx, uint64_t groups)
{
    const uint64_t blocks = (groups + kBnThreads - 1) / kBnThreads;
    return (int)std::min<uint64_t>(std::max<uint64_t>(blocks, 1), (uint64_t)ctx->num_cu * 8);
}
// blocks of the statistics launch: each flushes 2 * channels sums, so fewer and longer-running ones
static int sums_grid(const adapt_ctx *ctx, uint64_t groups, int channels, bool &reg)
{
    int grid = (int)std::min<uint64_t>(std::max<uint64_t>((groups + kBnThreads * 4 - 1) / (kBnThreads * 4), 1), (uint64_t)ctx->num_cu * 2);
    const uint64_t cg = (uint64_t)channels / 8;
    // register sums need a thread stride (grid * threads groups) that is a multiple of channels / 8
    reg = false;
    if (cg <= kBnThreads && kBnThreads % cg == 0) reg = true;
    else if ((uint64_t)grid * kBnThreads % cg == 0) reg = true;
    return grid;
}
static bool rng_ok(adapt_rng r) { return r.mode == ADAPT_SR || r.mode == ADAPT_RN_HALF_UP; }

size_t ws_need_bn(int num_cu, int channels)
{
    return (size_t)num_cu * 2 * 2 * (size_t)channels * 8 + (size_t)2 * channels * 8 + (size_t)num_cu * 8 * 8 + 256;
}

}  // namespace adapt

using namespace adapt;

extern "C" size_t adapt_bn_state_bytes(int channels)
{
    return channels > 0 && channels <= kBnMaxChannels ? ((bn_state_bytes(channels) + 255) & ~(size_t)255) : 0;
}

template <int MODE>
static int launch_sums(adapt_ctx *ctx, const void *a, int es_a, const void *b, int es_b, uint64_t groups, int channels, long long *partial,
                       int &grid)
{
    bool reg;
    grid = sums_grid(ctx, groups, channels, reg);
    const size_t lds = (size_t)2 * channels * 8;
    const dim3 g(grid), t(kBnThreads);
#define ADAPT_SUMS(TA, TB)                                                                                                          \
    do {                                                                                                                            \
        if (reg) hipLaunchKernelGGL((bn_sums_kernel<TA, TB, MODE, true>), g, t, lds, ctx->stream, (const TA *)a, (const TB *)b, groups, channels, partial); \
        else hipLaunchKernelGGL((bn_sums_kernel<TA, TB, MODE, false>), g, t, lds, ctx->stream, (const TA *)a, (const TB *)b, groups, channels, partial);    \
    } while (0)
    if (es_a == 1 && es_b == 1) ADAPT_SUMS(int8_t, int8_t);
    else if (es_a == 1) ADAPT_SUMS(int8_t, int16_t);
    else if (es_b == 1) ADAPT_SUMS(int16_t, int8_t);
    else ADAPT_SUMS(int16_t, int16_t);
#undef ADAPT_SUMS
    return ADAPT_OK;
}

extern "C" int adapt_bn_forward(adapt_ctx *ctx, const void *y, adapt_fmt fy, size_t rows, int channels, const float *gamma,
                                const float *beta, double eps, const void *res, adapt_fmt fres, adapt_fmt fo, adapt_rng rng, int relu,
                                void *out, void *state)
{
    if (!ctx || !fmt_ok_wide(fy) || !fmt_ok_wide(fo) || !rng_ok(rng) || !(eps >= 0.0) || (res && !fmt_ok_wide(fres))) return ADAPT_EINVAL;
    if (channels < 8 || channels > kBnMaxChannels || (channels & 7)) return ADAPT_EUNSUPPORTED;
    if (rows < 1 || rows > ((size_t)1 << 23)) return ADAPT_EUNSUPPORTED;         // sums of squares stay below 2^53
    if (!y || !out || !state || !gamma || !beta || !aligned16(y) || !aligned16(out) || ((uintptr_t)state & 63) || (res && !aligned16(res)))
        return ADAPT_EINVAL;
    const uint64_t groups = (uint64_t)rows * channels / 8;
    if (ws_need_bn(ctx->num_cu, channels) > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    long long *partial = reinterpret_cast<long long *>(scratch(ctx));
    if (fy.wl > 16 || fo.wl > 16 || (res && fres.wl > 16)) {      // int32 codes somewhere: the 128-bit kernels
        const int gridw = (int)std::min<uint64_t>(rows, (uint64_t)ctx->num_cu);
        long long *tot = partial + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels;
        double *second = reinterpret_cast<double *>(tot + channels);
        hipLaunchKernelGGL(bn_sums_wide_kernel, dim3(gridw), dim3(kBnThreads), 0, ctx->stream, y, storage_bytes(fy), y, storage_bytes(fy), 0,
                           (uint64_t)rows, channels, reinterpret_cast<unsigned long long *>(partial));
        hipLaunchKernelGGL(bn_total_wide_kernel, dim3((channels + 63) / 64), dim3(64), 0, ctx->stream,
                           reinterpret_cast<const unsigned long long *>(partial), gridw, channels, tot, second);
        hipLaunchKernelGGL(bn_coef_fwd_kernel, dim3(1), dim3(1024), 0, ctx->stream, tot, channels, (unsigned long long)rows, fy.fl, fo.fl,
                           gamma, beta, eps, state, second);
        BnWideArgs w = {};
        w.x = y; w.y = res; w.out = out; w.state = state; w.n = (uint64_t)rows * channels; w.es_x = storage_bytes(fy);
        w.es_y = res ? storage_bytes(fres) : 1; w.es_o = storage_bytes(fo); w.channels = channels; w.wl = fo.wl; w.relu = relu != 0;
        w.mode = rng.mode; w.fl_res = res ? fres.fl : 0; w.seed = rng.seed; w.stream = rng.stream;
        hipLaunchKernelGGL(bn_apply_wide_kernel, dim3(bn_grid(ctx, w.n)), dim3(kBnThreads), 0, ctx->stream, w);
        return hip_status(ctx, hipGetLastError());
    }
    int grid;
    launch_sums<0>(ctx, y, storage_bytes(fy), y, storage_bytes(fy), groups, channels, partial, grid);
    long long *totals = partial + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels;
    BnCoefArgs ca = {};
    ca.channels = channels; ca.fl_y = fy.fl; ca.fl_o = fo.fl; ca.rows = (unsigned long long)rows; ca.gamma = gamma; ca.beta = beta;
    ca.eps = eps; ca.state = state;
    hipLaunchKernelGGL(bn_total_coef_kernel<false>, dim3((2 * channels + 7) / 8), dim3(256), 0, ctx->stream, partial, grid, totals,
                       ticket(ctx, 0), ca);
    BnApplyArgs a;
    a.y = y; a.res = res; a.out = out; a.state = state; a.groups = groups; a.channels = channels; a.wl = fo.wl; a.relu = relu != 0;
    a.mode = rng.mode; a.has_res = res != nullptr; a.fl_res = res ? fres.fl : 0; a.seed = rng.seed; a.stream = rng.stream;
    const size_t lds = (size_t)channels * 12;
    const dim3 g(bn_grid(ctx, groups)), t(kBnThreads);
    const int sel = (storage_bytes(fy) == 2) * 4 + ((res ? storage_bytes(fres) : 1) == 2) * 2 + (storage_bytes(fo) == 2);
#define ADAPT_APPLY(TY, TR, TO) hipLaunchKernelGGL((bn_apply_kernel<TY, TR, TO>), g, t, lds, ctx->stream, a)
    switch (sel) {
    case 0: ADAPT_APPLY(int8_t, int8_t, int8_t); break;
    case 1: ADAPT_APPLY(int8_t, int8_t, int16_t); break;
    case 2: ADAPT_APPLY(int8_t, int16_t, int8_t); break;
    case 3: ADAPT_APPLY(int8_t, int16_t, int16_t); break;
    case 4: ADAPT_APPLY(int16_t, int8_t, int8_t); break;
    case 5: ADAPT_APPLY(int16_t, int8_t, int16_t); break;
    case 6: ADAPT_APPLY(int16_t, int16_t, int8_t); break;
    default: ADAPT_APPLY(int16_t, int16_t, int16_t); break;
    }
#undef ADAPT_APPLY
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_bn_backward(adapt_ctx *ctx, const void *dz, int wl_dz, const void *y, adapt_fmt fy, size_t rows, int channels,
                                 void *state, int wl_out, adapt_rng rng, void *dy, double *dgamma, double *dbeta, int32_t *shift,
                                 const int64_t *e_in, int64_t *e_out)
{
    if (!ctx || !fmt_ok_wide(fy) || wl_dz < 2 || wl_dz > 32 || wl_out < 2 || wl_out > 32 || !rng_ok(rng)) return ADAPT_EINVAL;
    if (channels < 8 || channels > kBnMaxChannels || (channels & 7)) return ADAPT_EUNSUPPORTED;
    if (rows < 1 || rows > ((size_t)1 << 23)) return ADAPT_EUNSUPPORTED;
    if (!dz || !y || !dy || !state || !dgamma || !dbeta || !aligned16(dz) || !aligned16(y) || !aligned16(dy) || ((uintptr_t)state & 63))
        return ADAPT_EINVAL;
    if (((uintptr_t)dgamma & 7) || ((uintptr_t)dbeta & 7) || ((uintptr_t)shift & 3) || ((uintptr_t)e_in & 7) || ((uintptr_t)e_out & 7))
        return ADAPT_EINVAL;
    const uint64_t groups = (uint64_t)rows * channels / 8;
    if (ws_need_bn(ctx->num_cu, channels) > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    long long *partial = reinterpret_cast<long long *>(scratch(ctx));
    const int es_d = storage_bytes(adapt_fmt{wl_dz, 0}), es_y = storage_bytes(fy), es_o = storage_bytes(adapt_fmt{wl_out, 0});
    if (es_d == 4 || es_y == 4 || es_o == 4) {                     // int32 codes somewhere: the 128-bit kernels
        const int gridw = (int)std::min<uint64_t>(rows, (uint64_t)ctx->num_cu);
        long long *tot = partial + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels;
        double *second = reinterpret_cast<double *>(tot + channels);
        hipLaunchKernelGGL(bn_sums_wide_kernel, dim3(gridw), dim3(kBnThreads), 0, ctx->stream, dz, es_d, y, es_y, 1, (uint64_t)rows, channels,
                           reinterpret_cast<unsigned long long *>(partial));
        hipLaunchKernelGGL(bn_total_wide_kernel, dim3((channels + 63) / 64), dim3(64), 0, ctx->stream,
                           reinterpret_cast<const unsigned long long *>(partial), gridw, channels, tot, second);
        hipLaunchKernelGGL(bn_coef_bwd_kernel, dim3(1), dim3(1024), 0, ctx->stream, tot, channels, state, dgamma, dbeta, second);
        BnWideArgs w = {};
        w.x = dz; w.y = y; w.out = dy; w.state = state; w.n = (uint64_t)rows * channels; w.es_x = es_d; w.es_y = es_y; w.es_o = es_o;
        w.channels = channels; w.wl = wl_out; w.mode = rng.mode; w.seed = rng.seed; w.stream = rng.stream; w.shift_out = shift;
        w.e_in = reinterpret_cast<const long long *>(e_in); w.e_out = reinterpret_cast<long long *>(e_out);
        const int gridp = (int)std::min<uint64_t>(std::max<uint64_t>((w.n + kBnThreads - 1) / kBnThreads, 1), (uint64_t)ctx->num_cu * 4);
        w.part = reinterpret_cast<uint64_t *>(scratch(ctx) + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels * 8 + (size_t)2 * channels * 8);
        w.nparts = gridp;
        hipLaunchKernelGGL(bn_bwd_wide_kernel<0>, dim3(gridp), dim3(kBnThreads), 0, ctx->stream, w);
        hipLaunchKernelGGL(bn_bwd_wide_kernel<1>, dim3(bn_grid(ctx, w.n)), dim3(kBnThreads), 0, ctx->stream, w);
        return hip_status(ctx, hipGetLastError());
    }
    int grid;
    launch_sums<1>(ctx, dz, es_d, y, es_y, groups, channels, partial, grid);
    long long *totals = partial + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels;
    BnCoefArgs ca = {};
    ca.channels = channels; ca.state = state; ca.dgamma = dgamma; ca.dbeta = dbeta;
    hipLaunchKernelGGL(bn_total_coef_kernel<true>, dim3((2 * channels + 7) / 8), dim3(256), 0, ctx->stream, partial, grid, totals,
                       ticket(ctx, 0), ca);
    BnBwdArgs a;
    a.dz = dz; a.y = y; a.dy = dy; a.state = state; a.groups = groups; a.channels = channels; a.wl = wl_out; a.mode = rng.mode;
    a.seed = rng.seed; a.stream = rng.stream; a.shift_out = shift;
    a.e_in = reinterpret_cast<const long long *>(e_in); a.e_out = reinterpret_cast<long long *>(e_out);
    const int grid1 = (int)std::min<uint64_t>(std::max<uint64_t>((groups + kBnThreads - 1) / kBnThreads, 1), (uint64_t)ctx->num_cu * 4);
    a.part = reinterpret_cast<uint64_t *>(scratch(ctx) + (size_t)ctx->num_cu * 2 * 2 * (size_t)channels * 8 + (size_t)2 * channels * 8);
    a.nparts = grid1;
    const size_t lds = (size_t)channels * 16;
    const dim3 t(kBnThreads), g2(bn_grid(ctx, groups));
    const int sel = (es_d == 2) * 4 + (es_y == 2) * 2 + (es_o == 2);
#define ADAPT_BWD(TD, TY, TO)                                                                                     \
    do {                                                                                                          \
        hipLaunchKernelGGL((bn_bwd_kernel<TD, TY, TO, false>), dim3(grid1), t, lds, ctx->stream, a);              \
        hipLaunchKernelGGL((bn_bwd_kernel<TD, TY, TO, true>), g2, t, lds, ctx->stream, a);                        \
    } while (0)
    switch (sel) {
    case 0: ADAPT_BWD(int8_t, int8_t, int8_t); break;
    case 1: ADAPT_BWD(int8_t, int8_t, int16_t); break;
    case 2: ADAPT_BWD(int8_t, int16_t, int8_t); break;
    case 3: ADAPT_BWD(int8_t, int16_t, int16_t); break;
    case 4: ADAPT_BWD(int16_t, int8_t, int8_t); break;
    case 5: ADAPT_BWD(int16_t, int8_t, int16_t); break;
    case 6: ADAPT_BWD(int16_t, int16_t, int8_t); break;
    default: ADAPT_BWD(int16_t, int16_t, int16_t); break;
    }
#undef ADAPT_BWD
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_bn_update(adapt_ctx *ctx, float *gamma, float *beta, const double *dgamma, const double *dbeta, int channels,
                               double lr)
{
    if (!ctx || !gamma || !beta || !dgamma || !dbeta || channels < 1 || channels > kBnMaxChannels || !(lr == lr)) return ADAPT_EINVAL;
    if (((uintptr_t)dgamma & 7) || ((uintptr_t)dbeta & 7)) return ADAPT_EINVAL;
    hipLaunchKernelGGL(bn_update_kernel, dim3(1), dim3(1024), 0, ctx->stream, gamma, beta, dgamma, dbeta, channels, (float)lr);
    return hip_status(ctx, hipGetLastError());
}

namespace adapt {
int bn_update_batch(adapt_ctx *ctx, const BnUpdateItem *items, int count, double lr)
{
    if (!ctx || count < 0 || (count > 0 && !items) || !(lr == lr)) return ADAPT_EINVAL;
    for (int t = 0; t < count; ++t) {
        const BnUpdateItem &it = items[t];
        if (!it.gamma || !it.beta || !it.dgamma || !it.dbeta || it.channels < 1 || it.channels > kBnMaxChannels) return ADAPT_EINVAL;
        if (((uintptr_t)it.dgamma & 7) || ((uintptr_t)it.dbeta & 7)) return ADAPT_EINVAL;
    }
    for (int base = 0; base < count; base += kUpdateMaxItems) {
        BnUpdateBatch b;
        const int m = std::min(count - base, kUpdateMaxItems);
        for (int t = 0; t < m; ++t) b.item[t] = items[base + t];
        hipLaunchKernelGGL(bn_update_batch_kernel, dim3(m), dim3(1024), 0, ctx->stream, b, (float)lr);
    }
    return hip_status(ctx, hipGetLastError());
}
}  // namespace adapt

extern "C" int adapt_gap_fwd(adapt_ctx *ctx, const void *a, adapt_fmt f, int n, int hw, int c, adapt_rng rng, void *out)
{
    if (!ctx || !fmt_ok_wide(f) || !rng_ok(rng) || n < 0 || hw < 1 || c < 1) return ADAPT_EINVAL;
    if ((hw & (hw - 1)) || (c & 7) || hw > (1 << 20) || (uint64_t)n * c >= ((uint64_t)1 << 31)) return ADAPT_EUNSUPPORTED;
    if (n == 0) return ADAPT_OK;
    if (!a || !out || !aligned16(a) || !aligned16(out)) return ADAPT_EINVAL;
    int sh = 0;
    while ((1 << sh) < hw) ++sh;
    if (f.wl > 16) {
        hipLaunchKernelGGL(gap_fwd_wide_kernel, dim3(bn_grid(ctx, (uint64_t)n * c)), dim3(kBnThreads), 0, ctx->stream, a, 4, out, (uint32_t)n,
                           (uint32_t)hw, (uint32_t)c, sh, f.wl, rng.mode, rng.seed, rng.stream);
        return hip_status(ctx, hipGetLastError());
    }
    const uint32_t cg = (uint32_t)c / 8;
    const dim3 g(bn_grid(ctx, (uint64_t)n * cg)), t(kBnThreads);
    if (storage_bytes(f) == 1)
        hipLaunchKernelGGL(gap_fwd_kernel<int8_t>, g, t, 0, ctx->stream, (const int8_t *)a, (int8_t *)out, (uint32_t)n, (uint32_t)hw, cg, sh,
                           f.wl, rng.mode, rng.seed, rng.stream);
    else
        hipLaunchKernelGGL(gap_fwd_kernel<int16_t>, g, t, 0, ctx->stream, (const int16_t *)a, (int16_t *)out, (uint32_t)n, (uint32_t)hw, cg,
                           sh, f.wl, rng.mode, rng.seed, rng.stream);
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_gap_bwd(adapt_ctx *ctx, const void *dout, int wl, int n, int hw, int c, void *da)
{
    if (!ctx || wl < 2 || wl > 32 || n < 0 || hw < 1 || c < 1) return ADAPT_EINVAL;
    if ((hw & (hw - 1)) || (c & 7)) return ADAPT_EUNSUPPORTED;
    if (n == 0) return ADAPT_OK;
    if (!dout || !da || !aligned16(dout) || !aligned16(da)) return ADAPT_EINVAL;
    if (wl > 16) {
        const uint64_t total = (uint64_t)n * hw * c;
        hipLaunchKernelGGL(gap_bwd_wide_kernel, dim3(bn_grid(ctx, total)), dim3(kBnThreads), 0, ctx->stream, (const int32_t *)dout,
                           (int32_t *)da, total, (uint32_t)hw, (uint32_t)c);
        return hip_status(ctx, hipGetLastError());
    }
    const uint32_t cg = (uint32_t)c / 8;
    const uint64_t groups = (uint64_t)n * hw * cg;
    const dim3 g(bn_grid(ctx, groups)), t(kBnThreads);
    if (wl <= 8) hipLaunchKernelGGL(gap_bwd_kernel<int8_t>, g, t, 0, ctx->stream, (const int8_t *)dout, (int8_t *)da, groups, (uint32_t)hw, cg);
    else hipLaunchKernelGGL(gap_bwd_kernel<int16_t>, g, t, 0, ctx->stream, (const int16_t *)dout, (int16_t *)da, groups, (uint32_t)hw, cg);
    return hip_status(ctx, hipGetLastError());
}

extern "C" int adapt_grad_add(adapt_ctx *ctx, const void *a, int wl_a, const int64_t *e_a, const void *b, int wl_b, const int64_t *e_b,
                              size_t n, int wl_out, adapt_rng rng, void *out, int32_t *shift, int64_t *e_out)
{
    if (!ctx || wl_a < 2 || wl_a > 32 || wl_out < 2 || wl_out > 32 || (b && (wl_b < 2 || wl_b > 32)) || !rng_ok(rng)) return ADAPT_EINVAL;
    if (n > ((uint64_t)1 << 40)) return ADAPT_EINVAL;
    if (((uintptr_t)e_a & 7) || ((uintptr_t)e_b & 7) || ((uintptr_t)e_out & 7) || ((uintptr_t)shift & 3)) return ADAPT_EINVAL;
    if (n > 0 && (!a || !out || !aligned16(a) || !aligned16(out) || (b && !aligned16(b)))) return ADAPT_EINVAL;
    const uint64_t groups = ((uint64_t)n + 7) >> 3;
    const int grid1 = (int)std::min<uint64_t>(std::max<uint64_t>((groups + kBnThreads - 1) / kBnThreads, 1), (uint64_t)ctx->num_cu * 4);
    if ((size_t)grid1 * 8 > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    MergeArgs m;
    m.a = a; m.b = b; m.out = out; m.e_a = reinterpret_cast<const long long *>(e_a); m.e_b = reinterpret_cast<const long long *>(e_b);
    m.e_out = reinterpret_cast<long long *>(e_out); m.shift_out = shift; m.n = n; m.wl = wl_out; m.mode = rng.mode; m.seed = rng.seed;
    m.stream = rng.stream; m.part = reinterpret_cast<uint64_t *>(scratch(ctx)); m.nparts = grid1;
    const dim3 t(kBnThreads), g2(bn_grid(ctx, groups));
    if (wl_a > 16 || wl_out > 16 || (b && wl_b > 16)) {             // int32 codes somewhere: sums in 128 bits
        const int ea = storage_bytes(adapt_fmt{wl_a, 0}), eb = b ? storage_bytes(adapt_fmt{wl_b, 0}) : 1, eo = storage_bytes(adapt_fmt{wl_out, 0});
        hipLaunchKernelGGL(merge_wide_kernel<0>, dim3(grid1), t, 0, ctx->stream, m, ea, eb, eo);
        hipLaunchKernelGGL(merge_wide_kernel<1>, dim3(bn_grid(ctx, (uint64_t)n)), t, 0, ctx->stream, m, ea, eb, eo);
        return hip_status(ctx, hipGetLastError());
    }
    const int sel = (wl_a > 8) * 4 + ((b ? wl_b : 8) > 8) * 2 + (wl_out > 8);
#define ADAPT_MERGE(TA, TB, TO)                                                                               \
    do {                                                                                                      \
        hipLaunchKernelGGL((merge_kernel<TA, TB, TO, false>), dim3(grid1), t, 0, ctx->stream, m);             \
        hipLaunchKernelGGL((merge_kernel<TA, TB, TO, true>), g2, t, 0, ctx->stream, m);                       \
    } while (0)
    switch (sel) {
    case 0: ADAPT_MERGE(int8_t, int8_t, int8_t); break;
    case 1: ADAPT_MERGE(int8_t, int8_t, int16_t); break;
    case 2: ADAPT_MERGE(int8_t, int16_t, int8_t); break;
    case 3: ADAPT_MERGE(int8_t, int16_t, int16_t); break;
    case 4: ADAPT_MERGE(int16_t, int8_t, int8_t); break;
    case 5: ADAPT_MERGE(int16_t, int8_t, int16_t); break;
    case 6: ADAPT_MERGE(int16_t, int16_t, int8_t); break;
    default: ADAPT_MERGE(int16_t, int16_t, int16_t); break;
    }
#undef ADAPT_MERGE
    return hip_status(ctx, hipGetLastError());
}
