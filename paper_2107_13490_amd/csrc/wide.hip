// Contractions with word lengths 17..32 (Sec. 3.3 bounds the precision that PushUp may ask for at
// 32 bits).  An operand above 16 bits is held as int32 codes and split into parts that the two-limb
// int8 MFMA kernels of this library take; an operand of at most 16 bits stays as it is.
//   17..23 bits: the signed low byte and what is left above it, a = a1 2^8 + a0 with |a1| <= 2^(wl-9), a code of
//                wl - 7 <= 16 bits: the byte stays one limb in the kernels, so a pair of such operands costs nine
//                int8 products (4 + 2 + 2 + 1) instead of the sixteen of two 16-bit parts each;
//   24..31 bits: two 16-bit parts, a = a1 2^16 + a0 with a0 the signed low half-word (so a1 =
//                (a + 2^15) >> 16 stays within 16 bits: |a1| <= 2^14);
//   32 bits:     there a1 could reach 2^15, so three parts of 11 bits, a = a2 2^22 + a1 2^11 + a0,
//                a0, a1 in [0, 2047], a2 = a >> 22 in [-512, 511], each a 12-bit code.
// Every pair of parts is one exact contraction (int32 or int64 sums, by the accumulator bound of that
// pair); the partial results are added at their weights 2^(bits_a i + bits_b j) in 128-bit integers,
// and the requantizing rule of the contraction epilogue (or the exact 128-bit sum) is applied once at
// the end.  Four contractions for two operands of up to 31 bits, nine for two of 32, two or three
// when one operand is narrow: the cost of precision above 16 bits on hardware whose matrix cores
// multiply bytes.
//
// The host code below composes the library's own entry points; the three kernels here are bound by
// HBM traffic (split: 4 B read, 6 B written per code; accumulate: 4-8 B read, 16 B read and written
// per output and part pair; finish: 16 B read, 1-4 B written per output).
#include <algorithm>
#include <functional>

#include "common.hpp"
#include "context.hpp"
#include "wide.hpp"

namespace adapt {

constexpr int kWideThreads = 256;
constexpr int kPartBits = 11;


__global__ void __launch_bounds__(kWideThreads)
split3_kernel(const int32_t *__restrict__ a, int16_t *__restrict__ p0, int16_t *__restrict__ p1, int16_t *__restrict__ p2, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads) {
        const int32_t v = a[i];
        p0[i] = (int16_t)(v & 2047);
        p1[i] = (int16_t)((v >> kPartBits) & 2047);
        p2[i] = (int16_t)(v >> (2 * kPartBits));
    }
}

// codes of at most 31 bits: signed low half-word and what is left above it
__global__ void __launch_bounds__(kWideThreads)
split2_kernel(const int32_t *__restrict__ a, int16_t *__restrict__ p0, int16_t *__restrict__ p1, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads) {
        const int32_t v = a[i];
        const int32_t lo = (int32_t)(int16_t)(v & 0xffff);
        p0[i] = (int16_t)lo;
        p1[i] = (int16_t)((v - lo) >> 16);
    }
}

// codes of at most 23 bits: signed low byte (an int8 tensor) and what is left above it
__global__ void __launch_bounds__(kWideThreads)
split_byte_kernel(const int32_t *__restrict__ a, int8_t *__restrict__ p0, int16_t *__restrict__ p1, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads) {
        const int32_t v = a[i];
        const int32_t lo = (int32_t)(int8_t)(v & 0xff);
        p0[i] = (int8_t)lo;
        p1[i] = (int16_t)((v - lo) >> 8);
    }
}

// acc[i] (+)= c[i] * 2^sh
template <typename CT>
__global__ void __launch_bounds__(kWideThreads)
acc128_kernel(const CT *__restrict__ c, int sh, i128 *__restrict__ acc, uint64_t n, int first)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads) {
        const i128 v = (i128)((u128)(i128)c[i] << sh);
        acc[i] = first ? v : acc[i] + v;
    }
}

template <typename OutT>
__global__ void __launch_bounds__(kWideThreads)
finish128_kernel(const i128 *__restrict__ acc, OutT *__restrict__ out, uint64_t n, int shift, int wl, int relu, int mode, uint64_t seed,
                 uint64_t stream)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads)
        out[i] = (OutT)requantize_wide_one(acc[i], shift, wl, relu, rounding_bits_of(seed, stream, i, mode));
}

// With room for one exact output buffer per pair of parts, the partial results are combined in one pass instead of
// one accumulation pass per pair: out = requantize(sum_p c_p 2^sh_p) (or the 128-bit sum itself).
struct PairSet {
    const void *c[9];
    int sh[9];
    int is32[9];
    int count;
};

template <typename OutT, bool RAW>
__global__ void __launch_bounds__(kWideThreads)
combine_kernel(const PairSet ps, OutT *__restrict__ out, uint64_t n, int shift, int wl, int relu, int mode, uint64_t seed, uint64_t stream)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kWideThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kWideThreads) {
        i128 s = 0;
        for (int p = 0; p < ps.count; ++p) {
            const long long v = ps.is32[p] ? (long long)static_cast<const int32_t *>(ps.c[p])[i] : static_cast<const long long *>(ps.c[p])[i];
            s += (i128)((u128)(i128)v << ps.sh[p]);
        }
        if (RAW) reinterpret_cast<i128 *>(out)[i] = s;
        else out[i] = (OutT)requantize_wide_one(s, shift, wl, relu, rounding_bits_of(seed, stream, i, mode));
    }
}

static int wide_grid(const adapt_ctx *ctx, uint64_t n)
{
    return (int)std::min<uint64_t>(std::max<uint64_t>((n + kWideThreads - 1) / kWideThreads, 1), (uint64_t)ctx->num_cu * 8);
}

static size_t a256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t ws_need_wide(uint64_t elems_a, bool wide_a, uint64_t elems_b, bool wide_b, uint64_t outputs, bool raw)
{
    return (wide_a ? 3 * a256(elems_a * 2) : 0) + (wide_b ? 3 * a256(elems_b * 2) : 0) + a256(outputs * 8) + (raw ? 0 : a256(outputs * 16));
}

// The parts an operand of format f is split into: their formats (lowest first) and the weight step in bits; returns
// the number of parts (1: the operand as it is)
int wide_parts(adapt_fmt f, adapt_fmt fmt[3], int *step)
{
    if (f.wl <= 16) { fmt[0] = f; *step = 0; return 1; }
    if (f.wl <= 23) { fmt[0] = adapt_fmt{8, 0}; fmt[1] = adapt_fmt{f.wl - 7, 0}; *step = 8; return 2; }
    if (f.wl <= 31) { fmt[0] = fmt[1] = adapt_fmt{16, 0}; *step = 16; return 2; }
    fmt[0] = fmt[1] = fmt[2] = adapt_fmt{12, 0};
    *step = kPartBits;
    return 3;
}

// One operand of a wide contraction: its parts (pointers, formats) after the split
struct WideOperand {
    const void *part[3];
    adapt_fmt fmt[3];
    int parts;
    int bits;          // weight of part i: 2^(bits * i)
};

int wide_contraction(adapt_ctx *ctx, const void *a, adapt_fmt fa, uint64_t elems_a, const void *b, adapt_fmt fb, uint64_t elems_b,
                     uint64_t outputs, int64_t k_total, void *out, adapt_epilogue ep, const SubContraction &sub)
{
    if (!fmt_ok_wide(fa) || !fmt_ok_wide(fb)) return ADAPT_EINVAL;
    if (!ep.raw && (!fmt_ok_wide(ep.fmt) || (ep.rng.mode != ADAPT_SR && ep.rng.mode != ADAPT_RN_HALF_UP))) return ADAPT_EINVAL;
    if (outputs == 0) return ADAPT_OK;
    const bool wide_a = fa.wl > 16, wide_b = fb.wl > 16;
    // buffers of this call at the end of the workspace; the contractions of the parts see the rest
    const size_t keep = (size_t)1 << 20;
    adapt_fmt pf[3];
    int step;
    const int npairs = wide_parts(fa, pf, &step) * wide_parts(fb, pf, &step);
    // one output buffer per pair and a single combining pass, when the workspace has room for that beside what a
    // part contraction of this size may itself need (taken as twice the minimal tail); else one buffer and a pass per pair
    const size_t tail_min = ws_need_wide(elems_a, wide_a, elems_b, wide_b, outputs, ep.raw != 0);
    const size_t tail_all = (wide_a ? 3 * a256(elems_a * 2) : 0) + (wide_b ? 3 * a256(elems_b * 2) : 0) + (size_t)npairs * a256(outputs * 8);
    const bool all_pairs = tail_all + tail_min + keep <= scratch_bytes(ctx);
    const size_t tail = all_pairs ? tail_all : tail_min;
    if (tail + keep > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    const size_t saved = ctx->ws_bytes;
    char *base = ctx->ws + saved - tail;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base + off; off += a256(bytes); return p; };
    WideOperand A, B;
    auto prepare = [&](WideOperand &o, const void *p, adapt_fmt f, uint64_t elems, bool wide) {
        if (!wide) {
            o.parts = 1; o.bits = 0; o.part[0] = p; o.fmt[0] = f;
            return;
        }
        o.parts = wide_parts(f, o.fmt, &o.bits);
        int16_t *q[3] = {nullptr, nullptr, nullptr};
        for (int i = 0; i < o.parts; ++i) {
            q[i] = reinterpret_cast<int16_t *>(take(elems * 2));      // (the byte part of the 8-bit split uses half of its room)
            o.part[i] = q[i];
        }
        if (o.bits == 8)
            hipLaunchKernelGGL(split_byte_kernel, dim3(wide_grid(ctx, elems)), dim3(kWideThreads), 0, ctx->stream,
                               static_cast<const int32_t *>(p), reinterpret_cast<int8_t *>(q[0]), q[1], elems);
        else if (o.parts == 2)
            hipLaunchKernelGGL(split2_kernel, dim3(wide_grid(ctx, elems)), dim3(kWideThreads), 0, ctx->stream,
                               static_cast<const int32_t *>(p), q[0], q[1], elems);
        else
            hipLaunchKernelGGL(split3_kernel, dim3(wide_grid(ctx, elems)), dim3(kWideThreads), 0, ctx->stream,
                               static_cast<const int32_t *>(p), q[0], q[1], q[2], elems);
    };
    prepare(A, a, fa, elems_a, wide_a);
    prepare(B, b, fb, elems_b, wide_b);
    adapt_epilogue ex = {};
    ex.raw = 1;
    ex.fmt = adapt_fmt{8, 0};
    ex.rng.mode = ADAPT_RN_HALF_UP;
    int status = ADAPT_OK;
    const size_t off_parts = off;
    if (all_pairs) {
        PairSet ps = {};
        ctx->ws_bytes = saved - tail;                  // what the part contractions may use
        for (int i = 0; i < A.parts && status == ADAPT_OK; ++i)
            for (int j = 0; j < B.parts && status == ADAPT_OK; ++j) {
                void *cp = take(outputs * 8);
                status = sub(A.part[i], A.fmt[i], B.part[j], B.fmt[j], cp, ex);
                ps.c[ps.count] = cp;
                ps.sh[ps.count] = A.bits * i + B.bits * j;
                ps.is32[ps.count] = adapt_acc_bits(k_total, A.fmt[i], B.fmt[j]) == 32;
                ++ps.count;
            }
        ctx->ws_bytes = saved;
        if (status == ADAPT_EWORKSPACE && tail_all >= tail_min) {      // a part contraction wanted more scratch: the frugal way
            status = ADAPT_OK;
            off = off_parts;
        } else {
            if (status != ADAPT_OK) return status;
            const int shift = ep.raw ? 0 : fa.fl + fb.fl - ep.fmt.fl;
            const dim3 g(wide_grid(ctx, outputs)), t(kWideThreads);
#define ADAPT_COMBINE(T, RAW) hipLaunchKernelGGL((combine_kernel<T, RAW>), g, t, 0, ctx->stream, ps, static_cast<T *>(out), outputs, shift, \
                                                 (int)ep.fmt.wl, ep.relu != 0, (int)ep.rng.mode, ep.rng.seed, ep.rng.stream)
            if (ep.raw) ADAPT_COMBINE(long long, true);
            else if (ep.fmt.wl <= 8) ADAPT_COMBINE(int8_t, false);
            else if (ep.fmt.wl <= 16) ADAPT_COMBINE(int16_t, false);
            else ADAPT_COMBINE(int32_t, false);
#undef ADAPT_COMBINE
            return hip_status(ctx, hipGetLastError());
        }
    }
    void *c = take(outputs * 8);
    i128 *acc = ep.raw ? static_cast<i128 *>(out) : reinterpret_cast<i128 *>(take(outputs * 16));
    ctx->ws_bytes = saved - tail;                      // what the part contractions may use
    bool first = true;
    for (int i = 0; i < A.parts && status == ADAPT_OK; ++i)
        for (int j = 0; j < B.parts && status == ADAPT_OK; ++j) {
            status = sub(A.part[i], A.fmt[i], B.part[j], B.fmt[j], c, ex);
            if (status != ADAPT_OK) break;
            const int sh = A.bits * i + B.bits * j;
            const int bits = adapt_acc_bits(k_total, A.fmt[i], B.fmt[j]);
            const dim3 g(wide_grid(ctx, outputs)), t(kWideThreads);
            if (bits == 32) hipLaunchKernelGGL(acc128_kernel<int32_t>, g, t, 0, ctx->stream, static_cast<const int32_t *>(c), sh, acc, outputs, first ? 1 : 0);
            else hipLaunchKernelGGL(acc128_kernel<int64_t>, g, t, 0, ctx->stream, static_cast<const int64_t *>(c), sh, acc, outputs, first ? 1 : 0);
            first = false;
        }
    ctx->ws_bytes = saved;
    if (status != ADAPT_OK) return status;
    if (!ep.raw) {
        const int shift = fa.fl + fb.fl - ep.fmt.fl;
        const dim3 g(wide_grid(ctx, outputs)), t(kWideThreads);
        if (ep.fmt.wl <= 8)
            hipLaunchKernelGGL(finish128_kernel<int8_t>, g, t, 0, ctx->stream, acc, static_cast<int8_t *>(out), outputs, shift, ep.fmt.wl,
                               ep.relu != 0, ep.rng.mode, ep.rng.seed, ep.rng.stream);
        else if (ep.fmt.wl <= 16)
            hipLaunchKernelGGL(finish128_kernel<int16_t>, g, t, 0, ctx->stream, acc, static_cast<int16_t *>(out), outputs, shift, ep.fmt.wl,
                               ep.relu != 0, ep.rng.mode, ep.rng.seed, ep.rng.stream);
        else
            hipLaunchKernelGGL(finish128_kernel<int32_t>, g, t, 0, ctx->stream, acc, static_cast<int32_t *>(out), outputs, shift, ep.fmt.wl,
                               ep.relu != 0, ep.rng.mode, ep.rng.seed, ep.rng.stream);
    }
    return hip_status(ctx, hipGetLastError());
}

}  // namespace adapt
