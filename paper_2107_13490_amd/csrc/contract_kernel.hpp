// Integer contractions of the quantized layers (ForwardPass / backward pass of Alg. 1):
// GEMM and implicit-GEMM convolution forward, data gradient and weight gradient, exact over
// the integers, on the int8 MFMA units of gfx950.
//
// One kernel template serves all four: the output O[m][n] (n is the contiguous output
// dimension) is computed as sum_k ACT[m][k] * WGT[n][k], where ACT ("m side") and WGT
// ("n side") are gathered on the fly from the operands:
//
//   op      m            n          k            ACT[m][k]                      WGT[n][k]
//   gemm    row of C     col of C   K            A                              B
//   fwd     (n,p,q)      kout       (r,s,c)      x[n,p*st+r-pad,q*st+s-pad,c]   w[kout,r,s,c]
//   dgrad   (n,h,w)      c          (r,s,kout)   dy[n,(h+pad-r)/st,(w+pad-s)/st,kout]   w[kout,r,s,c]
//   wgrad   kout         (r,s,c)    (n,p,q)      dy[n,p,q,kout]                 x[n,p*st+r-pad,q*st+s-pad,c]
//
// Tiles of ACT and WGT are staged in LDS and fed to v_mfma_i32_32x32x32_i8 with WGT as the row
// operand, so that a lane ends up holding 16 consecutive n for one m: the requantizing
// epilogue then needs one Philox block per 8 outputs and issues 16-byte stores.
//
// 9..16-bit operands are split on load into two int8 limbs; the four limb products accumulate in
// three int32 accumulators (hi*hi, cross, lo*lo) that the epilogue recombines in 64 bits.
//   balanced split (word lengths up to 15): a = 256*hi + lo with lo = the low byte read as a signed
//     int8 and hi = (a + 128) >> 8, which stays in [-64, 64] for |a| <= 2^14: nothing to correct.
//   offset split (word length 16, where the balanced hi would reach +128): a = 256*hi + (lo - 128) + 128
//     with hi = a >> 8 and lo - 128 = (a & 255) ^ 0x80, both in [-128,127] for every int16 a; the
//     "+128" offsets are undone in the epilogue from the row sums of both operands:
//       sum a*b = sum a'b' + 128 (sum a' + sum b') + 16384 * K,   a' = a - 128.
// An operand's limb mode: 1 = int8 storage, one limb; 2 = int16 storage, offset split; 3 = int16
// storage, balanced split.
#pragma once
#include <cmath>
#include <cstdlib>
#include <cstdio>
#include <algorithm>
#include <type_traits>

#include "common.hpp"
#include "context.hpp"

namespace adapt {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// OP_DGRAD_S2: the data gradient of a stride-2 convolution with its rows visited in parity-class order (see
// ContractArgs::dg_classes); a separate instantiation so that the plain data-gradient kernels keep their registers
enum { OP_GEMM = 0, OP_FWD = 1, OP_DGRAD = 2, OP_WGRAD = 3, OP_DGRAD_S2 = 4 };
constexpr bool is_dgrad(int op) { return op == OP_DGRAD || op == OP_DGRAD_S2; }
enum { LOAD_SCALAR = 0, LOAD_VEC = 1, LOAD_ROWS = 2 };
enum { OUT_RAW32 = 0, OUT_RAW64 = 1, OUT_Q8 = 2, OUT_Q16 = 3 };

constexpr int kThreads = 256;
constexpr unsigned kXcds = 8;      // accelerator dies, each with its own L2

// unsigned division by a run-time constant (Granlund-Montgomery round-up method), n < 2^31
struct FastDiv {
    uint32_t d, m, s;
};
static FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    f.s = l;
    f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    const uint32_t t = __umulhi(n, f.m);
    return (t + n) >> f.s;      // n < 2^31 and t < 2^32: t + n can wrap only for n >= 2^31
}

struct ContractArgs {
    const void *act, *wgt;
    void *out;
    int M, N, K;
    int act_es, wgt_es;          // element size in bytes (1: int8, 2: int16)
    int balanced;                // every int16 operand has a word length of at most 15: balanced limb split
    int fast;                    // two limbs, requantized output: the sums are small enough for 32-bit forms (see emit_run)
    uint32_t act_bytes, wgt_bytes;   // operand extents (the vector paths read through bounds-checked buffer loads)
    int act_load, wgt_load;      // LOAD_*
    // gemm: element (row,k) at row*rs + k*ks
    long long act_rs, act_ks, wgt_rs, wgt_ks;
    // conv geometry
    int n, h, w, c, k, r, s, stride, pad, p, q;
    FastDiv div_c, div_s, div_q, div_p, div_k, div_w, div_h, div_stride;
    // stride-2 data gradient: an input pixel sees only the filter taps of its row / column parity.
    // Rows are visited in parity-class order (class = 2*(h%2) + w%2, each n*(h/2)*(w/2) rows), so a tile
    // lies in one class and skips the stages of the other taps, which hold nothing but zeros.
    int dg_classes;              // 0: off, 4: on
    int dg_rows;                 // rows per class
    FastDiv dg_div_w2, dg_div_h2;
    uint32_t dg_mask[5];         // active taps (bit r*s_dim + s) of class 0..3; [4]: all taps, for tiles across classes
    int uniform_tap;             // 64 consecutive, 64-aligned k always lie in one filter tap
    int xcd_remap;               // contiguous ranges of blocks per XCD (see the kernel)
    int k_per_split;             // multiple of the kernel's stage depth
    int k_bound;                 // reduction length that decides the accumulator type (0: K); smaller than K when
                                 // zero channels were appended
    int force_finish;            // always go through slabs and finish_kernel
    int pad_c, pad_to;           // finish_kernel: the slabs hold pad_to channels per filter tap, the output pad_c (0: same)
    long long slab_bytes;        // split-K: split y writes its exact partial sums to out + y*slab_bytes
    long long ldc;               // output row stride in elements
    int out_mode;
    int shift, wl_o, relu, rmode;
    uint64_t seed, stream;
    // Exact output modes, optional (the fitting requantization that follows needs the tensor's largest magnitude):
    // block b of the launch that writes the final output stores the largest magnitude of its outputs at amax_part[b]
    // (b < amax_cap), and its first block clears *amax_zero (the sum the fitting pass adds to) when that is not null.
    unsigned long long *amax_part;
    unsigned long long *amax_zero;
    unsigned amax_cap;
};

// stride-2 data gradient in class order: visited row v -> row of dx (v < M)
__device__ __forceinline__ uint32_t dgrad_class_of(const ContractArgs &a, uint32_t v)
{
    return (uint32_t)(v >= (uint32_t)a.dg_rows) + (uint32_t)(v >= 2u * (uint32_t)a.dg_rows) + (uint32_t)(v >= 3u * (uint32_t)a.dg_rows);
}
__device__ __forceinline__ uint32_t dgrad_real_row(const ContractArgs &a, uint32_t v)
{
    const uint32_t cls = dgrad_class_of(a, v), local = v - cls * (uint32_t)a.dg_rows;
    const uint32_t nh = fdiv(local, a.dg_div_w2), w2 = local - nh * (uint32_t)(a.w >> 1);
    const uint32_t n = fdiv(nh, a.dg_div_h2), h2 = nh - n * (uint32_t)(a.h >> 1);
    return (n * (uint32_t)a.h + 2u * h2 + (cls >> 1)) * (uint32_t)a.w + 2u * w2 + (cls & 1u);
}
// position of the i-th set bit of mask (i < popcount)
__device__ __forceinline__ int nth_set_bit(uint32_t mask, int i)
{
    for (; i > 0; --i) mask &= mask - 1u;
    return __builtin_ctz(mask);
}

// ---------------------------------------------------------------------------------------------
// address functions: element offset of ACT[row][k] / WGT[row][k], or -1 for a zero
// ---------------------------------------------------------------------------------------------
template <int OP>
__device__ __forceinline__ long long act_offset(const ContractArgs &a, int row, int k)
{
    if (row >= a.M || k >= a.K) return -1;
    if (OP == OP_GEMM) return (long long)row * a.act_rs + (long long)k * a.act_ks;
    if (OP == OP_FWD) {
        const uint32_t pq = fdiv(row, a.div_q), q = row - pq * a.q;
        const uint32_t n = fdiv(pq, a.div_p), p = pq - n * a.p;
        const uint32_t tap = fdiv(k, a.div_c), c = k - tap * a.c;
        const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
        const int hh = (int)p * a.stride + (int)r - a.pad, ww = (int)q * a.stride + (int)s - a.pad;
        if ((unsigned)hh >= (unsigned)a.h || (unsigned)ww >= (unsigned)a.w) return -1;
        return (((long long)n * a.h + hh) * a.w + ww) * a.c + c;
    }
    if (is_dgrad(OP)) {
        const uint32_t nh = fdiv(row, a.div_w), w = row - nh * a.w;
        const uint32_t n = fdiv(nh, a.div_h), h = nh - n * a.h;
        const uint32_t tap = fdiv(k, a.div_k), ko = k - tap * a.k;
        const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
        const int hp = (int)h + a.pad - (int)r, wp = (int)w + a.pad - (int)s;
        if (hp < 0 || wp < 0) return -1;
        const uint32_t p = fdiv(hp, a.div_stride), q = fdiv(wp, a.div_stride);
        if ((int)(p * a.stride) != hp || (int)(q * a.stride) != wp || (int)p >= a.p || (int)q >= a.q) return -1;
        return (((long long)n * a.p + p) * a.q + q) * a.k + ko;
    }
    // OP_WGRAD: row = kout, k = (n,p,q)
    return (long long)k * a.k + row;
}

template <int OP>
__device__ __forceinline__ long long wgt_offset(const ContractArgs &a, int row, int k)
{
    if (row >= a.N || k >= a.K) return -1;
    if (OP == OP_GEMM) return (long long)row * a.wgt_rs + (long long)k * a.wgt_ks;
    if (OP == OP_FWD) return (long long)row * a.K + k;
    if (is_dgrad(OP)) {                                         // row = c, k = (r,s,kout): w[kout][r][s][c]
        const uint32_t tap = fdiv(k, a.div_k), ko = k - tap * a.k;
        return ((long long)ko * (a.r * a.s) + tap) * a.c + row;
    }
    // OP_WGRAD: row = (r,s,c), k = (n,p,q)
    const uint32_t tap = fdiv(row, a.div_c), c = row - tap * a.c;
    const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
    const uint32_t np = fdiv(k, a.div_q), q = k - np * a.q;
    const uint32_t n = fdiv(np, a.div_p), p = np - n * a.p;
    const int hh = (int)p * a.stride + (int)r - a.pad, ww = (int)q * a.stride + (int)s - a.pad;
    if ((unsigned)hh >= (unsigned)a.h || (unsigned)ww >= (unsigned)a.w) return -1;
    return (((long long)n * a.h + hh) * a.w + ww) * a.c + c;
}

template <int OP, bool ACT>
__device__ __forceinline__ long long operand_offset(const ContractArgs &a, int row, int k)
{
    return ACT ? act_offset<OP>(a, row, k) : wgt_offset<OP>(a, row, k);
}

// ---------------------------------------------------------------------------------------------
// limb splitting
// ---------------------------------------------------------------------------------------------
constexpr int es_of(int limb_mode) { return limb_mode == 1 ? 1 : 2; }          // bytes per stored code
constexpr int limbs_of(int limb_mode) { return limb_mode == 1 ? 1 : 2; }
constexpr bool bal_of(int limb_mode) { return limb_mode == 3; }

typedef short v2s __attribute__((ext_vector_type(2)));
// four int16 in (d0 = e1:e0, d1 = e3:e2) -> the limbs of e0..e3 (see the header of this file)
template <bool BAL>
__device__ __forceinline__ void split16(uint32_t d0, uint32_t d1, uint32_t &hi, uint32_t &lo)
{
    if (BAL) {
        const v2s half = {128, 128};
        const uint32_t t0 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(v2s, d0) + half);      // one packed 16-bit add
        const uint32_t t1 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(v2s, d1) + half);
        hi = __builtin_amdgcn_perm(t1, t0, 0x07050301u);
        lo = __builtin_amdgcn_perm(d1, d0, 0x06040200u);
    } else {
        hi = __builtin_amdgcn_perm(d1, d0, 0x07050301u);
        lo = __builtin_amdgcn_perm(d1, d0, 0x06040200u) ^ 0x80808080u;
    }
}
// ---------------------------------------------------------------------------------------------
// tile staging: global -> registers (prefetch) -> LDS
//
// A stage holds BKT reduction indices of both operands.  Two LDS layouts:
//   K-major  [row][BKT + 16 bytes]: k contiguous; fragments are read with one 16-byte LDS load.
//            Used when k is the contiguous direction in memory (LOAD_VEC, 16-byte global loads)
//            and by the element-wise fallback (LOAD_SCALAR).
//   R-major  [k][ROWS + 16 bytes]: rows contiguous, the operand's natural layout when the
//            reduction index is the slow direction in memory (weight gradient, transposed GEMM
//            operands).  Global 16-byte loads go to LDS untouched and fragments are read with
//            ds_read_b64_tr_b8, which hands each lane the 8 k-values of its row out of an
//            8 (k) x 16 (rows) byte block: no shuffling in registers.
// Zero elements are stored as code 0, i.e. limbs (hi = 0, lo = 0x80) after the offset split, (0, 0) after the balanced one.
// Everything that depends only on the thread's rows is computed once (init); per stage only
// the k-dependent part of the address remains, and when 64 consecutive k share one filter tap
// (a.uniform_tap) that part is the same for the whole block and lives in scalar registers.
// ---------------------------------------------------------------------------------------------

// A unit is 16 codes.  load_unit fetches one (ES = 1: one 16-byte load, ES = 2: two) at element offset `off` into
// staging registers as it lies in memory; split_unit turns a staged unit into limb words, which happens only when the
// unit is written to LDS, a stage later: a wavefront never waits on a load it has just issued.  Branch-free: the
// operand is read through a raw buffer descriptor whose range check returns zeros for out-of-range offsets, so an
// invalid unit just uses an offset beyond the tensor; zeros split into the limbs of code 0.
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    // dword 3 of the descriptor: 32-bit data format, raw (unstrided) addressing
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

template <int ES>
__device__ __forceinline__ void load_unit(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, bool ok, uint32_t (&r0)[4], uint32_t (&r1)[4])
{
    const uint32_t byte_off = ok ? off * ES : 0xfffffff0u;
    const v4u v0 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) r0[i] = v0[i];
    if (ES == 2) {
        const v4u v1 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 16, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) r1[i] = v1[i];
    }
}

template <int ES, bool BAL>
__device__ __forceinline__ void split_unit(const uint32_t (&r0)[4], const uint32_t (&r1)[4], uint32_t (&hi)[4], uint32_t (&lo)[4])
{
    if (ES == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) hi[i] = r0[i];
    } else {
        split16<BAL>(r0[0], r0[1], hi[0], lo[0]);
        split16<BAL>(r0[2], r0[3], hi[1], lo[1]);
        split16<BAL>(r1[0], r1[1], hi[2], lo[2]);
        split16<BAL>(r1[2], r1[3], hi[3], lo[3]);
    }
}

// ---- K-major operand: thread t owns rows (t/4) + 64*i and the 16-byte column (t%4) of every
//      64-k sub-chunk of the stage.  Element offsets are 32-bit (operands below 2^32 elements,
//      checked by the host); intermediate values may wrap, valid results do not.
template <int OP, bool ACT, int MODE, int ROWS, int LIMBS, int BKT, int ES, bool BAL>
struct LoaderK {
    static constexpr int RPT = ROWS / 64, SUB = BKT / 64, UNITS = RPT * SUB;
    static constexpr int ROW_BYTES = BKT + 16;
    static constexpr int TILE_BYTES = ROWS * ROW_BYTES;
    // one stage in flight: the units as loaded (hi = first, lo = second 16 bytes of a unit of int16 codes); the
    // element-wise gather stages limb words instead
    struct Regs { uint32_t hi[UNITS][4], lo[UNITS][4]; };
    uint32_t base[RPT];       // row part of the element offset, plus the thread's 16-element column
    // convolution activations (forward x, data-gradient dy): bit t = filter tap t reads inside the tensor for this row
    // (0 for rows beyond M); at most 32 taps on this path.  Other operands: all ones / zero by row validity.
    uint32_t tapmask[RPT];
    bool valid[RPT];
    __amdgpu_buffer_rsrc_t rsrc;

    __device__ __forceinline__ void init(const ContractArgs &a, int row0)
    {
        rsrc = make_rsrc(ACT ? a.act : a.wgt, ACT ? a.act_bytes : a.wgt_bytes);
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int row = row0 + (threadIdx.x >> 2) + 64 * i;
            valid[i] = row < (ACT ? a.M : a.N);
            base[i] = 0;
            tapmask[i] = valid[i] ? 0xffffffffu : 0u;
            if (MODE == LOAD_SCALAR) continue;
            if (OP == OP_GEMM) {
                base[i] = (uint32_t)row * (uint32_t)(ACT ? a.act_rs : a.wgt_rs);
            } else if (ACT && OP == OP_FWD) {
                const uint32_t pq = fdiv(row, a.div_q), q = row - pq * a.q;
                const uint32_t n = fdiv(pq, a.div_p), p = pq - n * a.p;
                const int ra = (int)p * a.stride - a.pad, rb = (int)q * a.stride - a.pad;
                base[i] = ((n * (uint32_t)a.h + (uint32_t)ra) * (uint32_t)a.w + (uint32_t)rb) * (uint32_t)a.c;
                // tap (r, s) reads x[ra + r][rb + s]
                uint32_t vs = 0, m = 0;
                for (int ss = 0; ss < a.s; ++ss) vs |= (uint32_t)((unsigned)(rb + ss) < (unsigned)a.w) << ss;
                for (int rr = 0; rr < a.r; ++rr)
                    if ((unsigned)(ra + rr) < (unsigned)a.h) m |= vs << (rr * a.s);
                tapmask[i] = valid[i] ? m : 0u;
            } else if (ACT && is_dgrad(OP)) {
                const uint32_t rr = (OP == OP_DGRAD_S2 && valid[i]) ? dgrad_real_row(a, row) : (uint32_t)row;
                const uint32_t nh = fdiv(rr, a.div_w), w = rr - nh * a.w;
                const uint32_t n = fdiv(nh, a.div_h), h = nh - n * a.h;
                const int ra = (int)h + a.pad, rb = (int)w + a.pad;
                // tap (r, s) reads dy[(ra - r) / stride][(rb - s) / stride] when both divide and lie inside; then
                // (ra - r) / stride = floor(ra / stride) - floor(r / stride) (equal remainders cancel), so the offset
                // splits into a row part (here) and a tap part (uniform, see load_sub)
                const uint32_t pa = fdiv((uint32_t)ra, a.div_stride), qa = fdiv((uint32_t)rb, a.div_stride);
                base[i] = (n * (uint32_t)(a.p * a.q) + pa * (uint32_t)a.q + qa) * (uint32_t)a.k;
                uint32_t vs = 0, m = 0;
                for (int ss = 0; ss < a.s; ++ss) {
                    const int wp = rb - ss;
                    const uint32_t qq = fdiv((uint32_t)max(wp, 0), a.div_stride);
                    vs |= (uint32_t)(wp >= 0 && (int)(qq * a.stride) == wp && (int)qq < a.q) << ss;
                }
                for (int r2 = 0; r2 < a.r; ++r2) {
                    const int hp = ra - r2;
                    const uint32_t pp = fdiv((uint32_t)max(hp, 0), a.div_stride);
                    if (hp >= 0 && (int)(pp * a.stride) == hp && (int)pp < a.p) m |= vs << (r2 * a.s);
                }
                tapmask[i] = valid[i] ? m : 0u;
            } else {
                base[i] = (uint32_t)row * (uint32_t)a.K;      // filters: [row][k]
            }
            base[i] += (threadIdx.x & 3) * 16;
        }
    }

    // One 64-k sub-chunk of all the thread's rows.  kq decides the filter tap: the sub-chunk's first k
    // when 64 aligned k share a tap (a uniform value: the tap arithmetic runs on the scalar unit),
    // else the thread's own k.
    // rows [i0, i1) of the thread's RPT rows
    template <typename KQ>
    __device__ __forceinline__ void load_sub(const ContractArgs &a, int sc, int k, int k64, KQ kq, Regs &rg, int i0 = 0, int i1 = RPT) const
    {
        const __amdgpu_buffer_rsrc_t ptr = rsrc;
        const bool kin = k < a.K;
        if (ACT && OP == OP_FWD) {
            const uint32_t tap = fdiv(kq, a.div_c);
            const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
            const uint32_t koff = (r * a.w + s) * a.c + ((uint32_t)k64 - tap * a.c);
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                if (i < i0 || i >= i1) continue;
                const bool ok = kin && ((tapmask[i] >> (tap & 31u)) & 1u);
                load_unit<ES>(ptr, base[i] + koff, ok, rg.hi[sc * RPT + i], rg.lo[sc * RPT + i]);
            }
        } else if (ACT && is_dgrad(OP)) {
            const uint32_t tap = fdiv(kq, a.div_k), ko = (uint32_t)k64 - tap * a.k;
            const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
            const uint32_t koff = ko - (fdiv(r, a.div_stride) * (uint32_t)a.q + fdiv(s, a.div_stride)) * (uint32_t)a.k;
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                if (i < i0 || i >= i1) continue;
                const bool ok = kin && ((tapmask[i] >> (tap & 31u)) & 1u);
                load_unit<ES>(ptr, base[i] + koff, ok, rg.hi[sc * RPT + i], rg.lo[sc * RPT + i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < RPT; ++i)
                if (i >= i0 && i < i1) load_unit<ES>(ptr, base[i] + (uint32_t)k64, valid[i] && kin, rg.hi[sc * RPT + i], rg.lo[sc * RPT + i]);
        }
    }

    __device__ __forceinline__ void load(const ContractArgs &a, int row0, int k0, Regs &rg) const
    {
        if (MODE == LOAD_VEC) {
#pragma unroll
            for (int sc = 0; sc < SUB; ++sc) {
                const int k64 = k0 + sc * 64, k = k64 + (threadIdx.x & 3) * 16;
                if (a.uniform_tap) load_sub(a, sc, k, k64, (uint32_t)__builtin_amdgcn_readfirstlane(k64), rg);
                else load_sub(a, sc, k, k64, (uint32_t)k, rg);
            }
        } else {
            // element-wise gather: any shape, any alignment
            const void *ptr = ACT ? a.act : a.wgt;
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const int row = row0 + (threadIdx.x >> 2) + 64 * i;
                const int k = k0 + (threadIdx.x & 3) * 16;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t h = 0, l = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const long long off = operand_offset<OP, ACT>(a, row, k + 4 * w + b);
                        int v = 0;
                        if (off >= 0)
                            v = ES == 1 ? (int)static_cast<const int8_t *>(ptr)[off] : (int)static_cast<const int16_t *>(ptr)[off];
                        if (LIMBS == 1) {
                            h |= (uint32_t)(v & 0xff) << (8 * b);
                        } else if (BAL) {
                            h |= (uint32_t)(((v + 128) >> 8) & 0xff) << (8 * b);
                            l |= (uint32_t)(v & 0xff) << (8 * b);
                        } else {
                            h |= (uint32_t)((v >> 8) & 0xff) << (8 * b);
                            l |= (uint32_t)((v & 0xff) ^ 0x80) << (8 * b);
                        }
                    }
                    rg.hi[i][w] = h;
                    rg.lo[i][w] = l;
                }
            }
        }
    }

    // unit u = sc * RPT + i alone (vector path): the pipelined main loop spreads a stage's loads over its MFMAs
    __device__ __forceinline__ void load_one(const ContractArgs &a, int k0, int u, Regs &rg) const
    {
        static_assert(MODE == LOAD_VEC, "per-unit loads exist for the vector path");
        const int sc = u / RPT, i = u % RPT;
        const int k64 = k0 + sc * 64, k = k64 + (threadIdx.x & 3) * 16;
        if (a.uniform_tap) load_sub(a, sc, k, k64, (uint32_t)__builtin_amdgcn_readfirstlane(k64), rg, i, i + 1);
        else load_sub(a, sc, k, k64, (uint32_t)k, rg, i, i + 1);
    }

    __device__ __forceinline__ static void store_one(const Regs &rg, int u, char *tile_hi, char *tile_lo)
    {
        const int sc = u / RPT, i = u % RPT;
        const int o = ((threadIdx.x >> 2) + 64 * i) * ROW_BYTES + sc * 64 + (threadIdx.x & 3) * 16;
        uint32_t hi[4], lo[4];
        if (MODE == LOAD_SCALAR) {
#pragma unroll
            for (int w = 0; w < 4; ++w) { hi[w] = rg.hi[u][w]; lo[w] = rg.lo[u][w]; }
        } else {
            split_unit<ES, BAL>(rg.hi[u], rg.lo[u], hi, lo);
        }
        *reinterpret_cast<uint4 *>(tile_hi + o) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        if (LIMBS == 2) *reinterpret_cast<uint4 *>(tile_lo + o) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }

    __device__ __forceinline__ static void store(const Regs &rg, char *tile_hi, char *tile_lo)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) store_one(rg, u, tile_hi, tile_lo);
    }

    // MFMA fragment: the 16 k-values [32*ks + 16*g, +16) of tile row `row`
    __device__ __forceinline__ static v4i frag(const char *tile, int row, int ks, int g)
    {
        return *reinterpret_cast<const v4i *>(tile + row * ROW_BYTES + ks * 32 + g * 16);
    }
};

// ---- R-major operand: a unit is 16 consecutive rows of one k
template <int OP, bool ACT, int ROWS, int LIMBS, int BKT, int ES, bool BAL>
struct LoaderR {
    static constexpr int CPL = ROWS / 16;                 // 16-row chunks per k line
    static constexpr int UNITS = BKT * CPL / kThreads;
    static constexpr int ROW_BYTES = ROWS + 16;           // bytes per k line
    static constexpr int TILE_BYTES = BKT * ROW_BYTES;
    struct Regs { uint32_t hi[UNITS][4], lo[UNITS][4]; };   // one stage in flight
    uint32_t coff[UNITS];
    int ra[UNITS], rb[UNITS];
    bool valid[UNITS];
    __amdgpu_buffer_rsrc_t rsrc;

    __device__ __forceinline__ void init(const ContractArgs &a, int row0)
    {
        rsrc = make_rsrc(ACT ? a.act : a.wgt, ACT ? a.act_bytes : a.wgt_bytes);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id = threadIdx.x + u * kThreads;
            const int row = row0 + (id % CPL) * 16;
            valid[u] = row < (ACT ? a.M : a.N);
            ra[u] = 0; rb[u] = 0; coff[u] = row;
            if (!ACT && OP == OP_WGRAD) {
                const uint32_t tap = fdiv(valid[u] ? row : 0, a.div_c), c = row - tap * a.c;
                const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
                ra[u] = (int)r - a.pad;
                rb[u] = (int)s - a.pad;
                coff[u] = c;
            }
        }
    }

    __device__ __forceinline__ void load(const ContractArgs &a, int row0, int k0, Regs &rg) const
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) load_one(a, k0, u, rg);
    }

    __device__ __forceinline__ void load_one(const ContractArgs &a, int k0, int u0, Regs &rg) const
    {
        const __amdgpu_buffer_rsrc_t ptr = rsrc;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            if (u != u0) continue;
            const int id = threadIdx.x + u * kThreads;
            const int kk = k0 + id / CPL;
            bool ok = valid[u] && kk < a.K;
            uint32_t off;
            if (OP == OP_GEMM) {
                off = coff[u] + (uint32_t)kk * (uint32_t)(ACT ? a.act_ks : a.wgt_ks);
            } else if (ACT) {                      // wgrad: dy[(n,p,q)][kout]
                off = coff[u] + (uint32_t)kk * (uint32_t)a.k;
            } else if (is_dgrad(OP)) {             // filters w[kout][r][s][c], k line = (r,s,kout)
                const uint32_t tap = fdiv(ok ? kk : 0, a.div_k), ko = kk - tap * a.k;
                off = (ko * (uint32_t)(a.r * a.s) + tap) * (uint32_t)a.c + coff[u];
            } else {                               // wgrad: x[n, p*st+r-pad, q*st+s-pad, c]
                const uint32_t np = fdiv(ok ? kk : 0, a.div_q), q = kk - np * a.q;
                const uint32_t n = fdiv(np, a.div_p), p = np - n * a.p;
                const int hh = (int)p * a.stride + ra[u], ww = (int)q * a.stride + rb[u];
                ok = ok && (unsigned)hh < (unsigned)a.h && (unsigned)ww < (unsigned)a.w;
                off = ((n * (uint32_t)a.h + (uint32_t)hh) * (uint32_t)a.w + (uint32_t)ww) * (uint32_t)a.c + coff[u];
            }
            load_unit<ES>(ptr, off, ok, rg.hi[u], rg.lo[u]);
        }
    }

    __device__ __forceinline__ static void store_one(const Regs &rg, int u, char *tile_hi, char *tile_lo)
    {
        const int id = threadIdx.x + u * kThreads;
        const int o = (id / CPL) * ROW_BYTES + (id % CPL) * 16;
        uint32_t hi[4], lo[4];
        split_unit<ES, BAL>(rg.hi[u], rg.lo[u], hi, lo);
        *reinterpret_cast<uint4 *>(tile_hi + o) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        if (LIMBS == 2) *reinterpret_cast<uint4 *>(tile_lo + o) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }

    __device__ __forceinline__ static void store(const Regs &rg, char *tile_hi, char *tile_lo)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) store_one(rg, u, tile_hi, tile_lo);
    }

    // MFMA fragment for the 32 rows starting at row32: lane l gets row row32 + l%32, k-values
    // [32*ks + 16*(l/32), +16).  Within a group of 16 lanes, ds_read_b64_tr_b8 gives lane i byte j
    // = byte (i%8) of the 8 bytes addressed by lane 2j + i/8; so lane 2j + h of the group points at
    // rows [8h, 8h+8) of k line j.
    __device__ __forceinline__ static v4i frag(const char *tile, int row32, int ks, int lane)
    {
        const int grp = lane >> 4, a = lane & 15;
        const int k = ks * 32 + 16 * (grp >> 1) + (a >> 1);
        const char *p = tile + k * ROW_BYTES + row32 + 16 * (grp & 1) + 8 * (a & 1);
        typedef v2i __attribute__((address_space(3))) * lds_v2i;
        const v2i x = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p));
        const v2i y = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p + 8 * ROW_BYTES));
        v4i f;
        f[0] = x[0]; f[1] = x[1]; f[2] = y[0]; f[3] = y[1];
        return f;
    }
};

// LM: the operand's limb mode; LIMBS: of the kernel (a one-limb kernel has both operands in mode 1)
template <int OP, bool ACT, int MODE, int ROWS, int LM, int BKT>
struct LoaderSelect { typedef LoaderK<OP, ACT, MODE, ROWS, limbs_of(LM), BKT, es_of(LM), bal_of(LM)> type; };
template <int OP, bool ACT, int ROWS, int LM, int BKT>
struct LoaderSelect<OP, ACT, LOAD_ROWS, ROWS, LM, BKT> { typedef LoaderR<OP, ACT, ROWS, limbs_of(LM), BKT, es_of(LM), bal_of(LM)> type; };

// ---------------------------------------------------------------------------------------------
// accumulator -> output format (the SR rule applied to the accumulator's low bits)
// ---------------------------------------------------------------------------------------------
// one-limb accumulators fit 32 bits with room for the rounding bits (|acc| <= 2^30).  `w` holds the
// rounding bits of two neighbouring outputs (low / high half); shift >= 1.
__device__ __forceinline__ int requantize_i32(int acc, int shift, int qlo, int qhi, uint32_t w, int half)
{
    int q;
    if (shift <= 16) q = (acc + (int)__builtin_amdgcn_ubfe(w, 16 * half + 16 - shift, shift)) >> shift;
    else q = ((acc >> (shift - 16)) + (int)__builtin_amdgcn_ubfe(w, 16 * half, 16)) >> 16;
    return min(max(q, qlo), qhi);      // one v_med3_i32
}

__device__ __forceinline__ uint32_t pack4_i8(int q0, int q1, int q2, int q3)
{
    // byte selectors: 0-3 second operand, 4-7 first operand, 0x0c constant zero
    return __builtin_amdgcn_perm((uint32_t)q1, (uint32_t)q0, 0x0c0c0400u) | __builtin_amdgcn_perm((uint32_t)q3, (uint32_t)q2, 0x04000c0cu);
}

// Writes 16 consecutive outputs (m, n0 .. n0+15) held by one lane.  FORM says what v holds:
//   FORM_I64   the exact value
//   FORM_I32   the exact value, known to fit 32 bits with room for the rounding bits (one-limb accumulators; mixed
//              two-limb sums whose bound allows it)
//   FORM_PAIR  (u, lo8) in the high and low halves of v, the exact value being 256 u + lo8 with 0 <= lo8 < 256 and u
//              in 32 bits: the two-limb sum with its lowest byte split off, for 1 <= shift <= 16.  With r the top
//              `shift` rounding bits, floor((256 u + lo8 + r) / 2^shift) = (u + ((lo8 + r) >> 8)) >> (shift - 8):
//              everything stays in 32-bit arithmetic.  Only requantized outputs take this form.
enum { FORM_I64 = 0, FORM_I32 = 1, FORM_PAIR = 2 };
template <int RUN, int FORM, bool AMAX = false>
__device__ __forceinline__ void emit_run(const ContractArgs &a, void *out, int m, int n0, const long long (&v)[RUN],
                                         unsigned long long &vmax)
{
    constexpr bool FITS32 = FORM == FORM_I32;
    static_assert(RUN == 16, "a lane holds runs of 16 outputs");
    if (m >= a.M || n0 >= a.N) return;
    const int cnt = min(RUN, a.N - n0);
    const long long row = (long long)m * a.ldc + n0;
    if constexpr (AMAX) {
        // the exact modes hold the true sums in v (the 32-bit forms belong to the requantizing epilogue)
        if (a.out_mode == OUT_RAW32 || a.out_mode == OUT_RAW64) {
#pragma unroll
            for (int i = 0; i < RUN; ++i)
                if (i < cnt) {
                    const unsigned long long mag = v[i] < 0 ? 0ull - (unsigned long long)v[i] : (unsigned long long)v[i];
                    vmax = mag > vmax ? mag : vmax;
                }
        }
    }
    if (a.out_mode == OUT_RAW32) {
        int32_t *o = static_cast<int32_t *>(out) + row;
        if (cnt == RUN && ((a.ldc | n0) & 3) == 0) {
#pragma unroll
            for (int i = 0; i < RUN / 4; ++i)
                reinterpret_cast<int4 *>(o)[i] = make_int4((int)v[4 * i], (int)v[4 * i + 1], (int)v[4 * i + 2], (int)v[4 * i + 3]);
        } else {
#pragma unroll
            for (int i = 0; i < RUN; ++i)
                if (i < cnt) o[i] = (int32_t)v[i];
        }
        return;
    }
    if (a.out_mode == OUT_RAW64) {
        long long *o = static_cast<long long *>(out) + row;
        if (cnt == RUN && ((a.ldc | n0) & 1) == 0) {
#pragma unroll
            for (int i = 0; i < RUN / 2; ++i) reinterpret_cast<longlong2 *>(o)[i] = make_longlong2(v[2 * i], v[2 * i + 1]);
        } else {
#pragma unroll
            for (int i = 0; i < RUN; ++i)
                if (i < cnt) o[i] = v[i];
        }
        return;
    }
    // requantize: output element index = m * N + n (row-major over the logical tensor); rw[i/2] holds
    // the rounding bits of outputs i (low half) and i+1 (high half)
    const uint64_t idx0 = (uint64_t)m * (uint64_t)a.N + (uint64_t)n0;
    uint32_t rw[RUN / 2];
    if (a.rmode != ADAPT_SR) {
#pragma unroll
        for (int i = 0; i < RUN / 2; ++i) rw[i] = 0x80008000u;
    } else if ((a.N & 7) == 0) {
        // rows are whole groups of 8 outputs (n0 is a multiple of 16): two Philox blocks cover the run
#pragma unroll
        for (int h = 0; h < RUN / 8; ++h) {
            const u32x4 b = rounding_block(a.seed, a.stream, (idx0 >> 3) + h);
            rw[4 * h] = b.x; rw[4 * h + 1] = b.y; rw[4 * h + 2] = b.z; rw[4 * h + 3] = b.w;
        }
    } else {
        // Any row length: the run starts at 16-bit lane idx0 % 8 of block idx0 / 8 and touches at most three blocks.
        // Their 24 lanes are drawn and shifted down by the lane's own offset (a select by word, then by half word).
        uint32_t w[13];
#pragma unroll
        for (int h = 0; h < 3; ++h) {
            const u32x4 b = rounding_block(a.seed, a.stream, (idx0 >> 3) + h);
            w[4 * h] = b.x; w[4 * h + 1] = b.y; w[4 * h + 2] = b.z; w[4 * h + 3] = b.w;
        }
        w[12] = 0;
        const uint32_t first = (uint32_t)idx0 & 7u, wo = first >> 1;
        uint32_t t[RUN / 2 + 1];
#pragma unroll
        for (int k = 0; k <= RUN / 2; ++k) t[k] = wo == 0 ? w[k] : wo == 1 ? w[k + 1] : wo == 2 ? w[k + 2] : w[k + 3];
#pragma unroll
        for (int k = 0; k < RUN / 2; ++k) rw[k] = (first & 1u) ? __builtin_amdgcn_alignbit(t[k + 1], t[k], 16) : t[k];
    }
    int q[RUN];
    if (FORM == FORM_PAIR) {
        const int qhi = (1 << (a.wl_o - 1)) - 1, qlo = a.relu ? 0 : -(1 << (a.wl_o - 1));
        if (a.shift >= 8) {
            const int sh8 = a.shift - 8;
#pragma unroll
            for (int i = 0; i < RUN; ++i) {
                const int u = (int)(v[i] >> 32), lo8 = (int)(uint32_t)v[i];
                const int r = (int)__builtin_amdgcn_ubfe(rw[i >> 1], 16 * (i & 1) + 16 - a.shift, a.shift);
                q[i] = min(max((u + ((lo8 + r) >> 8)) >> sh8, qlo), qhi);
            }
        } else {
            // shift below 8: (256 u + lo8 + r) >> shift = (u << (8 - shift)) + ((lo8 + r) >> shift); |u| >= 2^16 saturates
            // whatever the rest, so u is clamped to +-2^20 first and the left shift stays in 32 bits
            const int up = 8 - a.shift;
#pragma unroll
            for (int i = 0; i < RUN; ++i) {
                const int u = min(max((int)(v[i] >> 32), -(1 << 20)), 1 << 20), lo8 = (int)(uint32_t)v[i];
                const int r = (int)__builtin_amdgcn_ubfe(rw[i >> 1], 16 * (i & 1) + 16 - a.shift, a.shift);
                q[i] = min(max((u << up) + ((lo8 + r) >> a.shift), qlo), qhi);
            }
        }
    } else if (FITS32 && a.shift >= 1) {
        const int qhi = (1 << (a.wl_o - 1)) - 1, qlo = a.relu ? 0 : -(1 << (a.wl_o - 1));
#pragma unroll
        for (int i = 0; i < RUN; ++i) q[i] = requantize_i32((int)v[i], a.shift, qlo, qhi, rw[i >> 1], i & 1);
    } else {
#pragma unroll
        for (int i = 0; i < RUN; ++i)
            q[i] = requantize_one(v[i], a.shift, a.wl_o, a.relu, (rw[i >> 1] >> (16 * (i & 1))) & 0xffffu);
    }
    if (a.out_mode == OUT_Q8) {
        int8_t *o = static_cast<int8_t *>(out) + row;
        if (cnt == RUN && ((a.ldc | n0) & 15) == 0) {
            *reinterpret_cast<uint4 *>(o) = make_uint4(pack4_i8(q[0], q[1], q[2], q[3]), pack4_i8(q[4], q[5], q[6], q[7]),
                                                       pack4_i8(q[8], q[9], q[10], q[11]), pack4_i8(q[12], q[13], q[14], q[15]));
        } else {
#pragma unroll
            for (int i = 0; i < RUN; ++i)
                if (i < cnt) o[i] = (int8_t)q[i];
        }
    } else {
        int16_t *o = static_cast<int16_t *>(out) + row;
        if (cnt == RUN && ((a.ldc | n0) & 7) == 0) {
            uint32_t w[RUN / 2];
#pragma unroll
            for (int i = 0; i < RUN / 2; ++i) w[i] = (uint32_t)(q[2 * i] & 0xffff) | ((uint32_t)q[2 * i + 1] << 16);
            reinterpret_cast<uint4 *>(o)[0] = make_uint4(w[0], w[1], w[2], w[3]);
            reinterpret_cast<uint4 *>(o)[1] = make_uint4(w[4], w[5], w[6], w[7]);
        } else {
#pragma unroll
            for (int i = 0; i < RUN; ++i)
                if (i < cnt) o[i] = (int16_t)q[i];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// the kernel: block tile BM x BN, 4 wavefronts in a WGM x WGN grid, wave tile (BM/WGM) x (BN/WGN)
// built from 32x32 MFMA blocks; BKT reduction indices per stage.  One LDS stage: the global
// loads of the next stage are in flight (in registers) while the MFMAs of the current one
// run; several blocks per CU cover the rest of the load latency and each other's epilogues.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int dot4_ones(uint32_t v) { return __builtin_amdgcn_sdot4((int)v, 0x01010101, 0, false); }

// `lin` of `nwg` blocks, `ntiles` output tiles (the rest of the factor nwg / ntiles are K splits);
// `smem` is the block's dynamic LDS.
//
// PIPE = 1 is the pipeline of the large tiles (one wavefront per SIMD, so nothing else on the CU covers a
// wavefront's waits; PIPE = 2: the same with one staging set, for tiles that run two blocks per CU so that one
// block's epilogue overlaps the other's MFMAs): two LDS stages and one barrier per stage.  While stage kt is multiplied out of one
// buffer, the tile of stage kt+1 (loaded from memory during stage kt-1) is written to the other and the
// loads of stage kt+2 are issued; MFMA fragments are read one 32-deep sub-step ahead into a second set of
// registers, and the barrier sits before the last sub-step, so that the fragment reads of the next stage's
// first sub-step are in flight behind the MFMAs of this stage's last one.
// AMAX: an instance that also stores the largest magnitude of each block's outputs (ContractArgs::amax_part); the
// plain instances carry none of that code
template <int OP, int LIMBS, int AMODE, int WMODE, int AES, int WES, int BM, int BN, int WGM, int WGN, int BKT, int PIPE = 0, bool AMAX = false>
__device__ __forceinline__ void contract_body(const ContractArgs &a, const unsigned lin, const unsigned nwg,
                                              const unsigned ntiles, char *const smem)
{
    static_assert(WGM * WGN == 4, "four wavefronts per block");
    // Limbs per operand: in a two-limb kernel an operand stored as int8 (WL <= 8) stays one limb, so a mixed
    // layer issues two MFMA products per step instead of four:
    //   a one limb, b = 256 b_hi + b_lo' + 128:   a b = 256 (a b_hi) + (a b_lo') + 128 a
    //   a = 256 a_hi + a_lo' + 128, b one limb:   a b = 256 (a_hi b) + (a_lo' b) + 128 b
    // AES / WES are the operands' limb modes
    static_assert(LIMBS == 2 || (AES == 1 && WES == 1), "a one-limb kernel takes int8 operands");
    static_assert(AES == 1 || WES == 1 || AES == WES, "two int16 operands share their split");
    constexpr int LAL = limbs_of(AES), LBL = limbs_of(WES);
    constexpr bool BOTH2 = LAL == 2 && LBL == 2;
    constexpr bool OFFS = AES == 2 || WES == 2;      // offset split: the "+128" terms need the operands' row sums
    typedef typename LoaderSelect<OP, true, AMODE, BM, AES, BKT>::type LA;
    typedef typename LoaderSelect<OP, false, WMODE, BN, WES, BKT>::type LB;
    constexpr bool A_R = AMODE == LOAD_ROWS, W_R = WMODE == LOAD_ROWS;
    constexpr int WM = BM / WGM, WN = BN / WGN;     // wave tile
    constexpr int MB = WM / 32, NB = WN / 32;       // 32x32 blocks per wave
    // one LDS stage: [ACT hi | ACT lo | WGT hi | WGT lo]
    constexpr int A_LO = LA::TILE_BYTES, B_HI = LA::TILE_BYTES * LAL, B_LO = B_HI + LB::TILE_BYTES;
    constexpr int STAGE_BYTES = B_HI + LB::TILE_BYTES * LBL;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, g = lane >> 5;
    // K-major WGT operand: MFMA row i carries n_local = nperm(i), so that accumulator register r
    // of a lane is n_local = 16*g + r (16 consecutive outputs per lane).  R-major WGT operand:
    // rows arrive in order, register r is n_local = 8*(r/4) + 4*g + r%4 (runs of 4).
    const int nperm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    const int wrow = W_R ? l32 : nperm;

    // Workgroups go to the 8 XCDs round-robin in launch order and each XCD has its own L2: give
    // every XCD one contiguous range of the (split, tile_m, tile_n) order, so that blocks which
    // share operand rows (neighbouring tiles, all tiles of one split) fetch them from HBM once.
    const unsigned per_xcd = nwg / kXcds, extra = nwg % kXcds, xcd = lin % kXcds;
    const unsigned vid = a.xcd_remap ? xcd * per_xcd + min(xcd, extra) + lin / kXcds : lin;
    const int split = vid / ntiles, tile = vid % ntiles;
    const int tiles_n = (a.N + BN - 1) / BN;
    const int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int kbeg = split * a.k_per_split;
    const int kend = min(a.K, kbeg + a.k_per_split);
    int ksteps = (kend - kbeg + BKT - 1) / BKT;
    // stride-2 data gradient: only the stages of the taps this tile's parity class can see
    uint32_t dg_mask = 0;
    int dg_spt = 1;                 // stages per tap
    constexpr bool dg = OP == OP_DGRAD_S2;
    if (dg) {
        const uint32_t c0 = dgrad_class_of(a, (uint32_t)m0), c1 = dgrad_class_of(a, (uint32_t)min(m0 + BM, a.M) - 1u);
        dg_mask = a.dg_mask[c0 == c1 ? c0 : 4u];
        dg_spt = a.k / BKT;
        ksteps = __builtin_popcount(dg_mask) * dg_spt;
    }
    // the rows of dx this lane writes, mapped before the main loop (one register each; in the epilogue the
    // temporaries of the mapping would come on top of the peak register use)
    int dg_row[dg ? MB : 1];
    if (dg) {
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            const int m = m0 + wm * WM + j * 32 + l32;
            dg_row[j] = m < a.M ? (int)dgrad_real_row(a, (uint32_t)m) : m;
        }
    }
    auto stage_k = [&](int j) -> int {
        if (!dg) return kbeg + j * BKT;
        const int t = j / dg_spt;
        return nth_set_bit(dg_mask, t) * a.k + (j - t * dg_spt) * BKT;
    };

    v16i acc_hh[NB][MB], acc_x[NB][MB], acc_ll[NB][MB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc_hh[i][j][r] = 0; acc_x[i][j][r] = 0; acc_ll[i][j][r] = 0; }
    int sum_m[MB], sum_n[NB];       // two-limb: per-lane partial sums of a' = 256 hi + lo'
#pragma unroll
    for (int j = 0; j < MB; ++j) sum_m[j] = 0;
#pragma unroll
    for (int i = 0; i < NB; ++i) sum_n[i] = 0;

    LA la;
    LB lb;
    la.init(a, m0);
    lb.init(a, n0);
    // Register staging: the global loads of stage kt+1 are in flight while stage kt is multiplied out
    // of LDS.  (Two and three stages in flight were measured no faster at any tile shape: a stage is
    // bound by the rate at which the CU's vector-memory and LDS pipes move the operand bytes, not by
    // the latency of the loads, and the extra staging registers cost the large tiles a resident block.)
    typename LA::Regs ra;
    typename LB::Regs rb;
    if (ksteps > 0) {
        const int k0 = stage_k(0);
        la.load(a, m0, k0, ra);
        lb.load(a, n0, k0, rb);
    }

    struct Frags { v4i fa_h[MB], fa_l[MB], fb_h[NB], fb_l[NB]; };
    // MFMA fragments of the 32-deep sub-step ks of the stage at `st`
    auto read_frags = [&](const char *st, int ks, Frags &f) {
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            if constexpr (A_R) {
                f.fa_h[j] = LA::frag(st, wm * WM + j * 32, ks, lane);
                if (LAL == 2) f.fa_l[j] = LA::frag(st + A_LO, wm * WM + j * 32, ks, lane);
            } else {
                f.fa_h[j] = LA::frag(st, wm * WM + j * 32 + l32, ks, g);
                if (LAL == 2) f.fa_l[j] = LA::frag(st + A_LO, wm * WM + j * 32 + l32, ks, g);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if constexpr (W_R) {
                f.fb_h[i] = LB::frag(st + B_HI, wn * WN + i * 32, ks, lane);
                if (LBL == 2) f.fb_l[i] = LB::frag(st + B_LO, wn * WN + i * 32, ks, lane);
            } else {
                f.fb_h[i] = LB::frag(st + B_HI, wn * WN + i * 32 + nperm, ks, g);
                if (LBL == 2) f.fb_l[i] = LB::frag(st + B_LO, wn * WN + i * 32 + nperm, ks, g);
            }
        }
    };
    // the MFMAs of one 32 x 32 output block (i, j) for one sub-step, with that block's share of the row sums
    auto mfma_block = [&](const Frags &f, int i, int j) {
        acc_hh[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb_h[i], f.fa_h[j], acc_hh[i][j], 0, 0, 0);
        if (LAL == 2) acc_x[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb_h[i], f.fa_l[j], acc_x[i][j], 0, 0, 0);
        if (LBL == 2) acc_x[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb_l[i], f.fa_h[j], acc_x[i][j], 0, 0, 0);
        if (BOTH2) acc_ll[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.fb_l[i], f.fa_l[j], acc_ll[i][j], 0, 0, 0);
        // sums of the other side's k-values for the "+128" terms: of a' = 256 a_hi + a_lo' when a has two
        // limbs, of the plain codes when it has one (needed only when b has two limbs); likewise for b
        if (OFFS && LBL == 2 && i == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                sum_m[j] += LAL == 2 ? 256 * dot4_ones((uint32_t)f.fa_h[j][e]) + dot4_ones((uint32_t)f.fa_l[j][e])
                                     : dot4_ones((uint32_t)f.fa_h[j][e]);
        }
        if (OFFS && LAL == 2 && j == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                sum_n[i] += LBL == 2 ? 256 * dot4_ones((uint32_t)f.fb_h[i][e]) + dot4_ones((uint32_t)f.fb_l[i][e])
                                     : dot4_ones((uint32_t)f.fb_h[i][e]);
        }
    };
    auto mfma_step = [&](const Frags &f) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j < MB; ++j) mfma_block(f, i, j);
    };

    if constexpr (PIPE == 0) {
        for (int kt = 0; kt < ksteps; ++kt) {
            __syncthreads();                 // every wavefront is done with the previous stage
            LA::store(ra, smem, smem + A_LO);
            LB::store(rb, smem + B_HI, smem + B_LO);
            __syncthreads();
            if (kt + 1 < ksteps) {
                const int k0 = stage_k(kt + 1);
                la.load(a, m0, k0, ra);
                lb.load(a, n0, k0, rb);
            }
#pragma unroll
            for (int ks = 0; ks < BKT / 32; ++ks) {
                Frags f;
                read_frags(smem, ks, f);
                mfma_step(f);
            }
        }
    } else {
        // Everything a stage does besides its MFMAs is cut into NC pieces per sub-step, one after each output block's
        // MFMAs, with a scheduling fence between the pieces: the wavefront is alone on its SIMD, so LDS stores, global
        // loads and fragment reads overlap with the matrix unit only if they are issued between its instructions.
        //   sub-steps 0 .. KS-2 (before the barrier): the tile of stage kt+1 goes from staging set (kt+1)&1 to the other
        //     LDS buffer; fragments of the next sub-step
        //   sub-step KS-1 (after the barrier): loads of stage kt+3 into the staging set just freed; fragments of the
        //     next stage's first sub-step
        // The loop has no branches: beyond the last stage the loads are out of range (they read zeros without
        // memory traffic) and the stores and fragment reads touch LDS that nobody uses any more.
        constexpr int KS = BKT / 32, NC = NB * MB;
        static_assert(KS % 2 == 0, "the two fragment register sets alternate per sub-step");
        constexpr int UA = LA::UNITS, UT = LA::UNITS + LB::UNITS;      // staged units of a stage
        constexpr int FI = MB + NB;                                   // fragment items of a sub-step (one 32-row block each)
        Frags f[2];
        typename LA::Regs ra2;
        typename LB::Regs rb2;
        auto frag_item = [&](const char *st, int ks, int item, Frags &fr) {
            if (item < MB) {
                const int j = item;
                if constexpr (A_R) {
                    fr.fa_h[j] = LA::frag(st, wm * WM + j * 32, ks, lane);
                    if (LAL == 2) fr.fa_l[j] = LA::frag(st + A_LO, wm * WM + j * 32, ks, lane);
                } else {
                    fr.fa_h[j] = LA::frag(st, wm * WM + j * 32 + l32, ks, g);
                    if (LAL == 2) fr.fa_l[j] = LA::frag(st + A_LO, wm * WM + j * 32 + l32, ks, g);
                }
            } else {
                const int i = item - MB;
                if constexpr (W_R) {
                    fr.fb_h[i] = LB::frag(st + B_HI, wn * WN + i * 32, ks, lane);
                    if (LBL == 2) fr.fb_l[i] = LB::frag(st + B_LO, wn * WN + i * 32, ks, lane);
                } else {
                    fr.fb_h[i] = LB::frag(st + B_HI, wn * WN + i * 32 + nperm, ks, g);
                    if (LBL == 2) fr.fb_l[i] = LB::frag(st + B_LO, wn * WN + i * 32 + nperm, ks, g);
                }
            }
        };
        // reduction offset of stage j; beyond the last stage an offset past the reduction, whose loads return zeros
        auto stage_of = [&](int j) { return j < ksteps ? stage_k(j) : (a.K + 63) / 64 * 64; };
        // one stage; SET: the parity of kt (LDS buffer of the stage; the other staging set holds stage kt+1)
        auto run_stage = [&](auto setc, int kt) {
            constexpr int SET = decltype(setc)::value;
            char *const cur = smem + SET * STAGE_BYTES, *const nxt = smem + (SET ^ 1) * STAGE_BYTES;
            // staging set of this stage: with two sets, set (kt+1)&1 (set 0 = (ra, rb), set 1 = (ra2, rb2)), which holds
            // stage kt+1 and then takes stage kt+3; with one set (PIPE = 2) it holds stage kt+1 and takes stage kt+2
            typename LA::Regs &sa = (PIPE == 2 || SET) ? ra : ra2;
            typename LB::Regs &sb = (PIPE == 2 || SET) ? rb : rb2;
            const int k3 = stage_of(kt + (PIPE == 2 ? 2 : 3));
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == KS - 1) __syncthreads();      // the next stage's tile is written, this stage's fragments are read
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if (ks < KS - 1) {
                        constexpr int R1 = (KS - 1) * NC;                 // pieces before the barrier
                        const int piece = ks * NC + c;
#pragma unroll
                        for (int u = 0; u < UT; ++u)
                            if (u * R1 / UT == piece) {
                                if (u < UA) LA::store_one(sa, u, nxt, nxt + A_LO);
                                else LB::store_one(sb, u - UA, nxt + B_HI, nxt + B_LO);
                            }
#pragma unroll
                        for (int it = 0; it < FI; ++it)
                            if (it * NC / FI == c) frag_item(cur, ks + 1, it, f[(ks + 1) & 1]);
                    } else {
#pragma unroll
                        for (int it = 0; it < FI; ++it)
                            if (it * NC / FI == c) frag_item(nxt, 0, it, f[0]);
#pragma unroll
                        for (int u = 0; u < UT; ++u)
                            if (u * NC / UT == c) {
                                if (u < UA) la.load_one(a, k3, u, sa);
                                else lb.load_one(a, k3, u - UA, sb);
                            }
                    }
                    mfma_block(f[ks & 1], c / MB, c % MB);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        // No path around the loop: with nothing to reduce (K = 0, or a parity class that sees no filter tap) one stage of
        // zeros is multiplied.  (A second path from the zeroed accumulators to the epilogue made the register allocator
        // hold a copy of every accumulator in VGPRs across the loop.)
        const int nsteps = max(ksteps, 1);
        {
            // stage 0 is in set 0: write it, then stage 1 into set 1 and stage 2 into set 0
            if (ksteps <= 0) {
                la.load(a, m0, stage_of(0), ra);
                lb.load(a, n0, stage_of(0), rb);
            }
            LA::store(ra, smem, smem + A_LO);
            LB::store(rb, smem + B_HI, smem + B_LO);
            if constexpr (PIPE == 2) {
                la.load(a, m0, stage_of(1), ra);
                lb.load(a, n0, stage_of(1), rb);
            } else {
                la.load(a, m0, stage_of(1), ra2);
                lb.load(a, n0, stage_of(1), rb2);
                la.load(a, m0, stage_of(2), ra);
                lb.load(a, n0, stage_of(2), rb);
            }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < FI; ++it) frag_item(smem, 0, it, f[0]);
        }
        // Stage 0 always runs; then pairs of stages, then a last odd one.  (Written this way every path into a stage
        // has the same order of outstanding loads, older staging set first, so that the stores of a stage wait for their
        // own set only; with a conditional second stage inside the loop body the compiler had to drain all loads.)
        run_stage(std::integral_constant<int, 0>{}, 0);
        int kt = 1;
        for (; kt + 1 < nsteps; kt += 2) {
            run_stage(std::integral_constant<int, 1>{}, kt);
            run_stage(std::integral_constant<int, 0>{}, kt + 1);
        }
        if (kt < nsteps) run_stage(std::integral_constant<int, 1>{}, kt);
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // lane holds, for block (i,j): m = m0 + wm*WM + j*32 + l32 and 16 values of n (see above)
    long long corr_m[MB];
    int *sn = reinterpret_cast<int *>(smem);          // [4 waves][NB][32] n-side sums
    if (OFFS) {
        __syncthreads();                              // the tiles are no longer read
#pragma unroll
        for (int j = 0; j < MB; ++j) corr_m[j] = (long long)(sum_m[j] + __shfl_xor(sum_m[j], 32, 64));
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int t = sum_n[i] + __shfl_xor(sum_n[i], 32, 64);
            if (g == 0) sn[(wave * NB + i) * 32 + wrow] = t;
        }
        __syncthreads();
    }
    const long long kpad = (long long)ksteps * BKT;
    void *out = static_cast<char *>(a.out) + (long long)split * a.slab_bytes;
    unsigned long long vmax = 0;                      // largest magnitude of this lane's outputs (exact modes, when asked for)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            int m_of = 0, nb_of = 0;
            long long v[16];
            // a.fast: the host has checked the bound that lets a two-limb sum take one of the 32-bit forms
            const bool pair_form = BOTH2 && !OFFS && a.fast, i32_form = LIMBS == 2 && !BOTH2 && !OFFS && a.fast;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (LIMBS == 1) {
                    v[r] = acc_hh[i][j][r];
                } else if (pair_form) {
                    const int u = (acc_hh[i][j][r] << 8) + acc_x[i][j][r] + (acc_ll[i][j][r] >> 8);
                    v[r] = ((long long)u << 32) | (uint32_t)(acc_ll[i][j][r] & 255);
                } else if (i32_form) {
                    v[r] = (long long)((acc_hh[i][j][r] << 8) + acc_x[i][j][r]);
                } else {
                    if (BOTH2) v[r] = ((long long)acc_hh[i][j][r] << 16) + ((long long)acc_x[i][j][r] << 8) + (long long)acc_ll[i][j][r];
                    else v[r] = ((long long)acc_hh[i][j][r] << 8) + (long long)acc_x[i][j][r];
                    if (OFFS) {
                        const int nl = W_R ? 8 * (r >> 2) + 4 * g + (r & 3) : 16 * g + r;
                        const long long s_n = sn[(wave * NB + i) * 32 + nl];
                        // one side with one limb: the other side's sums are zero and never enter
                        v[r] += BOTH2 ? 128 * (corr_m[j] + s_n) + 16384 * kpad : 128 * (LBL == 2 ? corr_m[j] : s_n);
                    }
                }
            }
            auto emit = [&](const long long (&vals)[16]) {
                if (LIMBS == 1) emit_run<16, FORM_I32, AMAX>(a, out, m_of, nb_of + 16 * g, vals, vmax);
                else if (pair_form) emit_run<16, FORM_PAIR, AMAX>(a, out, m_of, nb_of + 16 * g, vals, vmax);
                else if (i32_form) emit_run<16, FORM_I32, AMAX>(a, out, m_of, nb_of + 16 * g, vals, vmax);
                else emit_run<16, FORM_I64, AMAX>(a, out, m_of, nb_of + 16 * g, vals, vmax);
            };
            int m = m0 + wm * WM + j * 32 + l32;
            const int nb0 = n0 + wn * WN + i * 32;
            if (dg) m = dg_row[dg ? j : 0];                                  // class order -> row of dx
            m_of = m; nb_of = nb0;
            if constexpr (W_R) {
                // lanes l and l^32 hold interleaved runs of 4 of the same output row: swap halves
                // so that each ends up with 16 consecutive n (lane/32 = 0: n 0..15, 1: n 16..31)
                long long recv[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const long long send = g == 0 ? v[8 + t] : v[t];
                    const int lo = __shfl_xor((int)(uint32_t)send, 32, 64);
                    const int hi = LIMBS == 1 ? (lo >> 31) : __shfl_xor((int)(send >> 32), 32, 64);
                    recv[t] = ((long long)hi << 32) | (uint32_t)lo;
                }
                long long w[16];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    w[t] = g == 0 ? v[t] : recv[t];
                    w[4 + t] = g == 0 ? recv[t] : v[8 + t];
                    w[8 + t] = g == 0 ? v[4 + t] : recv[4 + t];
                    w[12 + t] = g == 0 ? recv[4 + t] : v[12 + t];
                }
                emit(w);
            } else {
                emit(v);
            }
        }
    if constexpr (AMAX) {
        unsigned long long *sm = reinterpret_cast<unsigned long long *>(smem);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(vmax, off, 64);
            vmax = o > vmax ? o : vmax;
        }
        __syncthreads();                              // every wavefront has left the main loop: the tiles are free
        if (lane == 0) sm[wave] = vmax;
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long m = sm[0];
#pragma unroll
            for (int i = 1; i < 4; ++i) m = sm[i] > m ? sm[i] : m;
            if (a.amax_part != nullptr && lin < a.amax_cap) a.amax_part[lin] = m;
            if (lin == 0 && a.amax_zero != nullptr) *a.amax_zero = 0;
        }
    }
}

// Two-limb 64x64 tiles: three accumulator sets and the staging registers land a few registers above what three
// resident wavefronts per SIMD allow; asking for three makes the register allocator fit them without spills
// (forward 64->64 3x3 at 32x32, batch 256, <14,11>: 118 -> 86 us).  The weight gradient on its own gains nothing from it.
constexpr int min_waves_per_simd(int op, int limbs, int amode, int wmode, int aes, int wes, int bm, int bn, int pipe)
{
    if (pipe == 1) return 1;                                         // the large tiles: one wavefront per SIMD
    if (pipe == 2) return 2;                                         // two blocks per CU
    if (amode == LOAD_SCALAR || wmode == LOAD_SCALAR) return 1;      // the element-wise gather needs its registers
    // one limb: the same request moves the 128x128 tile from two to three resident wavefronts per SIMD
    // and the 128x64 tile from three to four
    // (only where the allocator manages without spills and it was measured to help: 256 x 32 x 32 x 256 -> 256 forward
    // 209 -> 200 us; the 64x128 tile spills, the 64x192 tile gains nothing)
    if (limbs == 1 && bm == 128 && bn == 128) return 3;
    if (limbs == 1 && bm == 128 && bn == 64) return 4;
    return (op != OP_WGRAD && limbs == 2 && aes >= 2 && wes >= 2 && bm == 64 && bn == 64) ? 3 : 1;
}

template <int OP, int LIMBS, int AMODE, int WMODE, int AES, int WES, int BM, int BN, int WGM, int WGN, int BKT, int PIPE = 0, bool AMAX = false>
__global__ void __launch_bounds__(kThreads, min_waves_per_simd(OP, LIMBS, AMODE, WMODE, AES, WES, BM, BN, PIPE))
contract_kernel(const ContractArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    contract_body<OP, LIMBS, AMODE, WMODE, AES, WES, BM, BN, WGM, WGN, BKT, PIPE, AMAX>(a, blockIdx.y * gridDim.x + blockIdx.x,
                                                                                     gridDim.x * gridDim.y, gridDim.x, smem);
}

// Two independent contractions in one launch (the two gradients of a layer): blocks [0, n_first)
// run the first, the rest the second, so that each fills the CUs the other leaves idle and one
// launch floor is paid instead of two.  Both have the same limb mode and stage depth.
// LM: the limb mode of all four operands (1, or 2 / 3 for int16 operands).
template <int LM, int BKT, int OPA, int AMA, int WMA, int BMA, int BNA, int OPB, int AMB, int WMB, int BMB, int BNB, bool AMAX = false>
__global__ void __launch_bounds__(kThreads, (LM >= 2 && BMA == 64 && BNA == 64 && BMB == 64 && BNB == 64) ? 3 : 1)      // as above; measured faster for the pair
contract_pair_kernel(const ContractArgs a, const ContractArgs b, const unsigned n_first, const unsigned tiles_a,
                     const unsigned tiles_b)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    if (blockIdx.x < n_first)
        contract_body<OPA, limbs_of(LM), AMA, WMA, LM, LM, BMA, BNA, 2, 2, BKT, 0, AMAX>(a, blockIdx.x, n_first, tiles_a, smem);
    else
        contract_body<OPB, limbs_of(LM), AMB, WMB, LM, LM, BMB, BNB, 2, 2, BKT, 0, AMAX>(b, blockIdx.x - n_first, gridDim.x - n_first,
                                                                                          tiles_b, smem);
}

// ---- helper: split-K finish ---------------------------------------------------------------------------
// split-K: sums the `splits` slabs of exact partial sums (dense M x N each) and converts
template <typename AccT>
__global__ void __launch_bounds__(256)
finish_kernel(const AccT *__restrict__ ws, int splits, ContractArgs a)
{
    const size_t total = (size_t)a.M * a.N;
    const size_t slab = (size_t)a.slab_bytes / sizeof(AccT);        // elements per slab (more than total with appended channels)
    unsigned long long vmax = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t m = i / a.N, n = i % a.N;
        size_t j = i;                                               // position inside a slab
        if (a.pad_c) {
            const size_t tap = n / a.pad_c, c = n - tap * a.pad_c;
            j = m * ((size_t)a.N / a.pad_c * a.pad_to) + tap * a.pad_to + c;
        }
        long long v = 0;
        int y = 0;
        for (; y + 8 <= splits; y += 8) {      // eight independent loads in flight
            AccT t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = ws[(size_t)(y + u) * slab + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) v += (long long)t[u];
        }
        for (; y < splits; ++y) v += (long long)ws[(size_t)y * slab + j];
        const size_t o = m * (size_t)a.ldc + n;
        if (a.out_mode == OUT_RAW32 || a.out_mode == OUT_RAW64) {
            const unsigned long long mag = v < 0 ? 0ull - (unsigned long long)v : (unsigned long long)v;
            vmax = mag > vmax ? mag : vmax;
        }
        switch (a.out_mode) {
            case OUT_RAW32: static_cast<int32_t *>(a.out)[o] = (int32_t)v; break;
            case OUT_RAW64: static_cast<long long *>(a.out)[o] = v; break;
            default: {
                const int q = requantize_one(v, a.shift, a.wl_o, a.relu, rounding_bits_of(a.seed, a.stream, i, a.rmode));
                if (a.out_mode == OUT_Q8) static_cast<int8_t *>(a.out)[o] = (int8_t)q;
                else static_cast<int16_t *>(a.out)[o] = (int16_t)q;
            }
        }
    }
    if (a.amax_part != nullptr) {                     // uniform over the launch
        __shared__ unsigned long long sm[4];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(vmax, off, 64);
            vmax = o > vmax ? o : vmax;
        }
        if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = vmax;
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long m = sm[0];
#pragma unroll
            for (int i = 1; i < 4; ++i) m = sm[i] > m ? sm[i] : m;
            if (blockIdx.x < a.amax_cap) a.amax_part[blockIdx.x] = m;
            if (blockIdx.x == 0 && a.amax_zero != nullptr) *a.amax_zero = 0;
        }
    }
}

// ---- host side ---------------------------------------------------------------------------------
struct TileShape { int bm, bn, bkt, pipe; };      // pipe: the double-buffered pipeline of the large tiles

// A launch that stores per-block maxima (ContractArgs::amax_part) tells the sink it fills how many there are
static inline void note_amax_blocks(adapt_ctx *ctx, const ContractArgs &a, long long blocks)
{
    if (a.amax_part == nullptr) return;
    for (adapt_amax_sink &s : ctx->amax)
        if (s.part == a.amax_part) s.count = blocks <= (long long)s.capacity ? (int)blocks : -1;
}

template <int OP, int LIMBS, int AMODE, int WMODE, int AES, int WES, int BM, int BN, int WGM, int WGN, int BKT, int PIPE = 0>
static hipError_t launch_es(adapt_ctx *ctx, const ContractArgs &a, int splits)
{
    constexpr int LAL = limbs_of(AES), LBL = limbs_of(WES);      // limbs per operand, as in the kernel
    typedef typename LoaderSelect<OP, true, AMODE, BM, AES, BKT>::type LA;
    typedef typename LoaderSelect<OP, false, WMODE, BN, WES, BKT>::type LB;
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    const size_t lds = std::max<size_t>(((size_t)LA::TILE_BYTES * LAL + (size_t)LB::TILE_BYTES * LBL) * (PIPE ? 2 : 1), 4 * 4 * 32 * sizeof(int) * 4);
    void (*kern)(const ContractArgs) = contract_kernel<OP, LIMBS, AMODE, WMODE, AES, WES, BM, BN, WGM, WGN, BKT, PIPE>;
    if constexpr (is_dgrad(OP) || OP == OP_WGRAD)      // the gradient contractions of a chained step (see plan_contraction)
        if (a.amax_part != nullptr) kern = contract_kernel<OP, LIMBS, AMODE, WMODE, AES, WES, BM, BN, WGM, WGN, BKT, PIPE, true>;
    if (hipError_t e = allow_big_lds(ctx, reinterpret_cast<const void *>(kern), lds); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(tiles, splits), dim3(kThreads), lds, ctx->stream, a);
    note_amax_blocks(ctx, a, (long long)tiles * splits);
    return hipGetLastError();
}

// storage types of the two operands: one limb means both int8
template <int OP, int LIMBS, int AMODE, int WMODE, int BM, int BN, int WGM, int WGN, int BKT>
static hipError_t launch_variant(adapt_ctx *ctx, const ContractArgs &a, int splits)
{
    if constexpr (LIMBS == 1) {
        return launch_es<OP, 1, AMODE, WMODE, 1, 1, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
    } else {
        // limb modes: balanced split when no int16 operand is wider than 15 bits, else the offset split
        if (a.act_es == 2 && a.wgt_es == 2) {
            if (a.balanced) return launch_es<OP, 2, AMODE, WMODE, 3, 3, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
            return launch_es<OP, 2, AMODE, WMODE, 2, 2, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
        }
        if (a.act_es == 2) {
            if (a.balanced) return launch_es<OP, 2, AMODE, WMODE, 3, 1, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
            return launch_es<OP, 2, AMODE, WMODE, 2, 1, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
        }
        if (a.balanced) return launch_es<OP, 2, AMODE, WMODE, 1, 3, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
        return launch_es<OP, 2, AMODE, WMODE, 1, 2, BM, BN, WGM, WGN, BKT>(ctx, a, splits);
    }
}

// Tile shapes: BM in {64, 128}, BN in {64, 128} and (one-limb convolutions only) 192; stage depth
// 64, or 192 for the vector paths of the convolutions.
template <int OP, int LIMBS, int AMODE, int WMODE, int BM, int BKT>
static hipError_t launch_bn(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    if (t.bn == 64) return launch_variant<OP, LIMBS, AMODE, WMODE, BM, 64, 2, 2, BKT>(ctx, a, splits);
    if constexpr (LIMBS == 1 && OP != OP_GEMM)
        if (t.bn == 192) return launch_variant<OP, LIMBS, AMODE, WMODE, BM, 192, 2, 2, BKT>(ctx, a, splits);
    return launch_variant<OP, LIMBS, AMODE, WMODE, BM, 128, 2, 2, BKT>(ctx, a, splits);
}

// The tiles of the double-buffered pipeline: two limbs (both operands int16, one split for both).
template <int OP, int AMODE, int WMODE, int LM>
static hipError_t launch_pipe2(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    if (t.pipe == 2) {
        if (t.bm == 128) return launch_es<OP, 2, AMODE, WMODE, LM, LM, 128, 64, 2, 2, 64, 2>(ctx, a, splits);
        return launch_es<OP, 2, AMODE, WMODE, LM, LM, 64, 128, 2, 2, 64, 2>(ctx, a, splits);
    }
    return launch_es<OP, 2, AMODE, WMODE, LM, LM, 128, 128, 2, 2, 64, 1>(ctx, a, splits);
}

template <int OP, int LIMBS, int AMODE, int WMODE>
static hipError_t launch_tile(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    if constexpr (LIMBS == 2 && AMODE != LOAD_SCALAR && WMODE != LOAD_SCALAR && OP != OP_GEMM && OP != OP_WGRAD)
        if (t.pipe) return a.balanced ? launch_pipe2<OP, AMODE, WMODE, 3>(ctx, a, splits, t) : launch_pipe2<OP, AMODE, WMODE, 2>(ctx, a, splits, t);
    if constexpr (AMODE == LOAD_SCALAR) {
        return launch_variant<OP, LIMBS, AMODE, WMODE, 128, 64, 2, 2, 64>(ctx, a, splits);
    } else if constexpr (OP == OP_GEMM) {
        if (t.bm == 64) return launch_bn<OP, LIMBS, AMODE, WMODE, 64, 64>(ctx, a, splits, t);
        return launch_bn<OP, LIMBS, AMODE, WMODE, 128, 64>(ctx, a, splits, t);
    } else {
        if constexpr (LIMBS == 1)
            if (t.bkt == 192) {
                if (t.bm == 64) return launch_bn<OP, LIMBS, AMODE, WMODE, 64, 192>(ctx, a, splits, t);
                return launch_bn<OP, LIMBS, AMODE, WMODE, 128, 192>(ctx, a, splits, t);
            }
        if (t.bm == 64) return launch_bn<OP, LIMBS, AMODE, WMODE, 64, 64>(ctx, a, splits, t);
        return launch_bn<OP, LIMBS, AMODE, WMODE, 128, 64>(ctx, a, splits, t);
    }
}

// Instantiated load-mode pairs: the vector paths that each op can use, and one element-wise
// fallback per op for shapes that are not multiples of the vector width.
template <int OP, int LIMBS>
static hipError_t launch_modes(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    const bool scalar = a.act_load == LOAD_SCALAR || a.wgt_load == LOAD_SCALAR;
    if constexpr (is_dgrad(OP))        // few input channels (first layer): the gradient tile still takes the vector path
        if (a.act_load == LOAD_VEC && a.wgt_load == LOAD_SCALAR)
            return launch_variant<OP, LIMBS, LOAD_VEC, LOAD_SCALAR, 128, 64, 2, 2, 64>(ctx, a, splits);
    if constexpr (OP == OP_DGRAD_S2) {
        if (scalar) return hipErrorInvalidValue;      // the class order is only planned for the vector path of dy
    } else {
        if (scalar) return launch_tile<OP, LIMBS, LOAD_SCALAR, LOAD_SCALAR>(ctx, a, splits, t);
    }
    if constexpr (OP == OP_WGRAD) {
        return launch_tile<OP, LIMBS, LOAD_ROWS, LOAD_ROWS>(ctx, a, splits, t);
    } else if constexpr (OP == OP_GEMM) {
        if (a.act_load == LOAD_VEC && a.wgt_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_VEC>(ctx, a, splits, t);
        if (a.act_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_ROWS>(ctx, a, splits, t);
        if (a.wgt_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_ROWS, LOAD_VEC>(ctx, a, splits, t);
        return launch_tile<OP, LIMBS, LOAD_ROWS, LOAD_ROWS>(ctx, a, splits, t);
    } else if constexpr (is_dgrad(OP)) {
        return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_ROWS>(ctx, a, splits, t);
    } else {
        return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_VEC>(ctx, a, splits, t);
    }
}

template <int OP>
static TileShape pick_tile(const ContractArgs &a, int limbs, int num_cu)
{
    TileShape t;
    t.pipe = 0;
    const bool scalar = a.act_load == LOAD_SCALAR || a.wgt_load == LOAD_SCALAR;
    if (a.N <= 64 || scalar) t.bn = 64;
    else if (OP != OP_GEMM && limbs == 1 && (a.N % 192 == 0 || (a.N > 128 && a.N <= 192))) t.bn = 192;   // 3 x 96 accumulators do not fit
                                                                                                           // the register file
    else if ((a.N + 127) / 128 * 128 - a.N >= 64) t.bn = 64;
    else t.bn = 128;
    // deeper stages cut the number of exposed load latencies; zero padding of the last stage must stay small
    // (two limbs: four times the MFMA work per stage already, and the staging registers are needed for accumulators)
    t.bkt = (OP != OP_GEMM && !scalar && limbs == 1 && (a.K % 192 == 0 || a.K >= 3072)) ? 192 : 64;
    // Small problems: several resident blocks per CU hide each other's load latency and epilogue,
    // so halve the tile when 128-row tiles would leave fewer than two blocks per CU.  (Split-K
    // contractions get their parallelism from the splits instead.)
    const long long tiles128 = (long long)((a.M + 127) / 128) * ((a.N + t.bn - 1) / t.bn);
    t.bm = (!scalar && OP != OP_WGRAD && tiles128 < 2 * num_cu && a.M > 64) ? 64 : 128;
    if (limbs == 1 && !scalar && OP != OP_WGRAD) {
        // One limb, forward / data gradient / GEMM: the largest of the 128x128, 128x64, 64x128 and 64x64 tiles that
        // still gives every CU two blocks (three when the reduction is short and a block's fixed costs weigh more)
        // without much padding; 64x64 when none does.  Measured (batch 128..256, 3x3): 64->192 at 16x16 forward
        // 12.0 us with 64x192 tiles, 10.6 with 128x64; 192->384 at 8x8 17.8 -> 14.0 (forward) and 35.9 -> 21.6
        // (data gradient, which had been split over K); 512->512 at 4x4 28.0 -> 23.3.
        const long long want = (long long)(a.K >= 1024 ? 2 : 3) * num_cu;
        auto fits = [&](int bm, int bn, double &waste) {
            const long long tm = (a.M + bm - 1) / bm, tn = (a.N + bn - 1) / bn;
            waste = (double)(tm * bm) * (double)(tn * bn) / ((double)a.M * (double)a.N);
            return tm * tn >= want && waste <= 1.25;
        };
        double w0, w1, w2;
        t.bm = t.bn = 64;
        if (fits(128, 128, w0)) {
            t.bm = t.bn = 128;
        } else {
            const bool tall = fits(128, 64, w1), wide = fits(64, 128, w2);
            if (tall && (!wide || w1 <= w2)) { t.bm = 128; t.bn = 64; }
            else if (wide) { t.bm = 64; t.bn = 128; }
        }
    }
    if (limbs == 2 && !scalar && OP != OP_WGRAD) {
        // Two limbs: the 64x64 tile runs four resident wavefronts per SIMD (three accumulator sets fit one unified
        // register file, see min_waves_per_simd), the 128x128 tile one; 64x64 was measured faster at every size
        // (conv 128->128 at 16x16, batch 256: 67 against 82 us; at 32x32: 250 against 325 us).
        t.bm = t.bn = 64;
        // Both operands int16, long rows of tiles: the double-buffered pipeline.  A stage of a 64 x 64 tile stores as many
        // bytes to LDS per MFMA clock as the LDS can take (about 64 B/clk per CU).  128 x 128 tiles store half of that and
        // run one block per CU, which leaves the epilogue (Philox, 64-bit recombination) uncovered: they pay when the
        // reduction is long.  128 x 64 / 64 x 128 tiles (three quarters) run two blocks per CU, one block's epilogue
        // behind the other's MFMAs.
        if (OP != OP_GEMM && a.act_es == 2 && a.wgt_es == 2 && a.K % 64 == 0) {
            auto tiles_of = [&](int bm, int bn) { return (long long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
            auto waste_of = [&](int bm, int bn) { return (double)tiles_of(bm, bn) * bm * bn / ((double)a.M * (double)a.N); };
            if (a.K >= 1536 && tiles_of(128, 128) >= num_cu && waste_of(128, 128) <= 1.15) {
                t.bm = t.bn = 128; t.bkt = 64; t.pipe = 1;
            } else if (tiles_of(128, 64) >= 2 * num_cu && waste_of(128, 64) <= 1.15) {
                t.bm = 128; t.bn = 64; t.bkt = 64; t.pipe = 2;
            } else if (tiles_of(64, 128) >= 2 * num_cu && waste_of(64, 128) <= 1.15) {
                t.bm = 64; t.bn = 128; t.bkt = 64; t.pipe = 2;
            }
        }
    }
    return t;
}

// Weight gradients have a small output and a very long reduction, so they are always split
// across blocks.  The tile and the number of splits are chosen together from a model fitted to
// measurements on MI355X: operand bytes pulled through L2 (at about 10.7 TB/s), slab bytes written
// and read back by the finish kernel (about 3.1 TB/s), a fixed cost for the second launch, and
// the rounding up to whole rounds of two blocks per CU.  Returns the number of splits.
static int pick_split_tile(const ContractArgs &a, int limbs, int acc_bits, int num_cu, TileShape &t)
{
    static const int cand[5][2] = {{64, 64}, {128, 64}, {64, 128}, {128, 128}, {128, 192}};
    const int bkt = t.bkt;
    double best = 1e30;
    int best_splits = 1;
    for (int i = 0; i < 5; ++i) {
        const int bm = cand[i][0], bn = cand[i][1];
        // two limbs: only the 64x64 tile (two resident blocks per CU) and the 128x128 tile (one block
        // per CU, whose exposed latencies cost about 1.6x) are worth considering
        if (limbs == 2 && bm != bn) continue;
        const bool single = limbs == 2 && bm == 128;
        const long long per_cu = single ? 1 : 2;
        const long long tm = (a.M + bm - 1) / bm, tn = (a.N + bn - 1) / bn, tiles = tm * tn;
        long long sp = tiles >= num_cu ? 1 : std::max(1ll, per_cu * num_cu / tiles);
        sp = std::max(1ll, std::min(sp, (long long)a.K / (2 * bkt)));
        const double slots = (double)(per_cu * num_cu), wgs = (double)tiles * sp;
        if (single && wgs < 0.9 * num_cu) continue;       // measured far slower than the model when CUs stay idle
        const double rounds = std::ceil(wgs / slots) / (wgs / slots);
        const double operand = (double)a.K * (double)(tm * bm) * (double)(tn * bn) * (1.0 / bm + 1.0 / bn) * limbs *
                               (single ? 1.6 : 1.0);
        const double slab = sp > 1 ? 2.0 * (double)a.M * a.N * (acc_bits / 8) * sp : 0.0;
        // unsplit two-limb kernels with a large output and a short reduction (fully connected layers) are bound
        // by their epilogue: about 0.5 T outputs/s with two resident blocks per CU, 0.28 T/s with one
        const double epilogue = (limbs == 2 && sp == 1) ? (double)a.M * a.N / (single ? 0.28e12 : 0.5e12) : 0.0;
        const double cost = operand * rounds / 10.7e12 + slab / 3.1e12 + (sp > 1 ? 5e-6 : 0.0) + epilogue;
        if (cost < best) { best = cost; best_splits = (int)sp; t.bm = bm; t.bn = bn; }
    }
    return best_splits;
}

// A contraction planned on the host: what the kernel gets, and what finish_kernel gets when K is
// split across blocks (exact partial sums in workspace slabs) because a single block could overflow
// its int32 accumulators or because the output has too few tiles to fill the GPU.
struct ContractPlan {
    ContractArgs kern;      // arguments of the contraction kernel (final output, or slabs)
    ContractArgs fin;       // arguments of finish_kernel (splits > 1)
    TileShape tile;
    int limbs, bits, splits;
    const char *acc;        // slabs
    bool empty;             // nothing to do (M or N is 0)
    size_t ws_end;          // bytes of scratch in use after this contraction's slabs
};

template <int OP>
static int plan_contraction(adapt_ctx *ctx, ContractArgs a, adapt_fmt fa, adapt_fmt fb, adapt_epilogue ep,
                            size_t ws_offset /* bytes of scratch already in use */, ContractPlan &p,
                            size_t ws_limit = (size_t)-1 /* bytes of scratch there are; default: the context's */)
{
    if (ws_limit == (size_t)-1) ws_limit = scratch_bytes(ctx);
    const int limbs = (fa.wl > 8 || fb.wl > 8) ? 2 : 1;
    const int bits = adapt_acc_bits(a.k_bound ? a.k_bound : a.K, fa, fb);
    int final_mode;
    if (ep.raw) {
        final_mode = bits == 32 ? OUT_RAW32 : OUT_RAW64;
    } else {
        if (!fmt_ok(ep.fmt) || (ep.rng.mode != ADAPT_SR && ep.rng.mode != ADAPT_RN_HALF_UP)) return ADAPT_EINVAL;
        final_mode = ep.fmt.wl <= 8 ? OUT_Q8 : OUT_Q16;
        a.shift = fa.fl + fb.fl - ep.fmt.fl;
        a.wl_o = ep.fmt.wl;
        a.relu = ep.relu != 0;
        a.rmode = ep.rng.mode;
        a.seed = ep.rng.seed;
        a.stream = ep.rng.stream;
    }
    a.balanced = fa.wl <= 15 && fb.wl <= 15;
    a.fast = 0;
    if (!ep.raw && limbs == 2 && a.balanced) {
        // bound of |sum|: K 2^(wl_a-1) 2^(wl_b-1)
        const long long kb = a.k_bound ? a.k_bound : a.K;
        const int mag = fa.wl + fb.wl - 2;
        int kbits = 0;
        while ((1ll << kbits) < kb) ++kbits;
        if (fa.wl > 8 && fb.wl > 8) a.fast = a.shift >= 1 && a.shift <= 16 && kbits + mag <= 38;      // (u, low byte) form
        else a.fast = a.shift >= 1 && kbits + mag <= 30;                                                // fits 32 bits
    }
    p.limbs = limbs;
    p.bits = bits;
    p.empty = a.M == 0 || a.N == 0;
    p.splits = 1;
    p.acc = nullptr;
    p.ws_end = ws_offset;
    if (p.empty) return ADAPT_OK;

    TileShape t = pick_tile<OP>(a, limbs, ctx->num_cu);
    int model_splits = 0;
    if (OP == OP_WGRAD && a.act_load != LOAD_SCALAR && a.wgt_load != LOAD_SCALAR) model_splits = pick_split_tile(a, limbs, bits, ctx->num_cu, t);
    a.xcd_remap = 1;
    // stride-2 data gradient: three of four stages hold only zeros for any one parity class (see ContractArgs);
    // skipping them needs stages that do not straddle taps
    const bool want_dg = OP == OP_DGRAD && a.stride == 2 && a.h % 2 == 0 && a.w % 2 == 0 && a.act_load == LOAD_VEC &&
                         a.k % 64 == 0 && a.r * a.s <= 32;
    if (want_dg && a.k % t.bkt != 0) t.bkt = 64;
    const long long tiles = (long long)((a.M + t.bm - 1) / t.bm) * ((a.N + t.bn - 1) / t.bn);
    // int32 accumulators: |product| <= 2^14 per limb pair, the cross accumulator holds two per k
    const int k_cap = limbs == 1 ? 65536 : 32768;
    int splits = (a.K + k_cap - 1) / k_cap;
    if (model_splits > 0) {
        splits = std::max(splits, model_splits);
    } else if (tiles < ctx->num_cu && a.K >= 8 * t.bkt) {
        // few tiles and a long reduction (fully connected layers at training batch sizes): two blocks per
        // CU hide each other's stage latencies (fc 128 x 4096 x 4096: 44 -> 34 us two-limb, 21 -> 19 one-limb)
        const long long want = (2 * ctx->num_cu + tiles - 1) / tiles;
        const long long max_by_k = a.K / (4 * t.bkt);
        splits = (int)std::max<long long>(splits, std::min(want, std::max(1ll, max_by_k)));
    }
    if (splits < 1) splits = 1;
    int k_per = ((a.K + splits - 1) / splits + t.bkt - 1) / t.bkt * t.bkt;
    if (k_per == 0) k_per = t.bkt;
    splits = a.K == 0 ? 1 : (a.K + k_per - 1) / k_per;
    a.k_per_split = k_per;
    a.slab_bytes = 0;
    a.dg_classes = 0;
    if (want_dg && splits == 1 && a.k % t.bkt == 0) {
        a.dg_classes = 4;
        a.dg_rows = a.n * (a.h / 2) * (a.w / 2);
        a.dg_div_w2 = make_fastdiv(a.w / 2);
        a.dg_div_h2 = make_fastdiv(a.h / 2);
        for (int cls = 0; cls < 4; ++cls) {
            uint32_t mask = 0;
            for (int r = 0; r < a.r; ++r)
                for (int sx = 0; sx < a.s; ++sx)
                    if ((((cls >> 1) + a.pad - r) & 1) == 0 && (((cls & 1) + a.pad - sx) & 1) == 0) mask |= 1u << (r * a.s + sx);
            a.dg_mask[cls] = mask;
        }
        a.dg_mask[4] = a.r * a.s == 32 ? 0xffffffffu : (1u << (a.r * a.s)) - 1u;
    }
    p.tile = t;
    p.splits = splits;
    p.ws_end = ws_offset;
    // exact output with a sink armed: the launch that writes the final output also stores its blocks' largest magnitudes
    const adapt_amax_sink &sink = ctx->amax[OP == OP_WGRAD ? 1 : 0];
    auto arm = [&](ContractArgs &dst) {
        if (!(OP == OP_DGRAD || OP == OP_WGRAD) || !ep.raw || sink.part == nullptr) return;
        dst.amax_part = sink.part;
        dst.amax_zero = sink.zero;
        dst.amax_cap = (unsigned)sink.capacity;
    };
    if (splits == 1 && !a.force_finish) {
        a.out_mode = final_mode;
        arm(a);
        p.kern = a;
        return ADAPT_OK;
    }
    // a partial sum is bounded like the total, so the slabs use the total's accumulator type
    const size_t acc_bytes = bits == 32 ? 4 : 8;
    const size_t slab = (size_t)a.M * a.N * acc_bytes;
    const size_t off = (ws_offset + 255) & ~(size_t)255;
    const size_t room = ws_limit > off ? ws_limit - off : 0;
    if (slab * (size_t)splits > room) {
        // Not enough workspace for the preferred number of splits: take as many as fit.  Splits that only
        // serve parallelism may go down to none (the result is the same, only slower); the splits that
        // keep a block's int32 accumulators inside their bound may not.
        const int must = std::max(1, (a.K + k_cap - 1) / k_cap);
        int take = (int)std::min<size_t>(room / slab, (size_t)splits);
        if (take < must) {
            if (must > 1) return ADAPT_EBOUND;
            if (a.force_finish) return ADAPT_EWORKSPACE;
            take = 1;                                  // unsplit, straight to the output: no workspace needed
        }
        k_per = ((a.K + take - 1) / take + t.bkt - 1) / t.bkt * t.bkt;
        if (k_per == 0) k_per = t.bkt;
        splits = a.K == 0 ? 1 : (a.K + k_per - 1) / k_per;
        a.k_per_split = k_per;
        p.splits = splits;
        if (splits == 1 && !a.force_finish) {
            a.out_mode = final_mode;
            arm(a);
            p.kern = a;
            return ADAPT_OK;
        }
    }
    p.ws_end = off + slab * (size_t)splits;
    char *acc = ctx->ws ? scratch(ctx) + off : nullptr;      // no workspace: a sizing query, nothing is launched
    p.acc = acc;
    p.kern = a;
    p.kern.out = acc;
    p.kern.ldc = a.N;
    p.kern.slab_bytes = (long long)slab;
    p.kern.out_mode = bits == 32 ? OUT_RAW32 : OUT_RAW64;
    p.kern.fast = 0;                                  // exact partial sums go to the slabs
    p.fin = a;
    p.fin.out_mode = final_mode;
    p.fin.slab_bytes = (long long)slab;
    arm(p.fin);
    return ADAPT_OK;
}

// the stride-2 data gradient in class order: its kernel instances are compiled in a file of their own (contract_dgrad_s2.hip)
hipError_t launch_planned_dgrad_s2(adapt_ctx *ctx, const ContractPlan &p);

template <int OP>
static hipError_t launch_planned(adapt_ctx *ctx, const ContractPlan &p)
{
    if (p.empty) return hipSuccess;
    if constexpr (OP == OP_DGRAD)
        if (p.kern.dg_classes) return launch_planned_dgrad_s2(ctx, p);
    return p.limbs == 1 ? launch_modes<OP, 1>(ctx, p.kern, p.splits, p.tile) : launch_modes<OP, 2>(ctx, p.kern, p.splits, p.tile);
}

// The planned gradient contractions as plain functions (contract_dgrad.hip, contract_wgrad.hip), so that the combined
// backward call does not compile a second copy of every kernel instance
hipError_t launch_planned_dgrad(adapt_ctx *ctx, const ContractPlan &p);
hipError_t launch_planned_wgrad(adapt_ctx *ctx, const ContractPlan &p);

// the slab sum + epilogue of a split contraction
static hipError_t finish_planned(adapt_ctx *ctx, const ContractPlan &p)
{
    if (p.empty || p.acc == nullptr) return hipSuccess;
    const unsigned fgrid = (unsigned)std::min<size_t>(((size_t)p.fin.M * p.fin.N + 255) / 256, (size_t)ctx->num_cu * 8);
    if (p.bits == 32)
        hipLaunchKernelGGL(finish_kernel<int32_t>, dim3(fgrid), dim3(256), 0, ctx->stream, reinterpret_cast<const int32_t *>(p.acc), p.splits, p.fin);
    else
        hipLaunchKernelGGL(finish_kernel<long long>, dim3(fgrid), dim3(256), 0, ctx->stream, reinterpret_cast<const long long *>(p.acc), p.splits, p.fin);
    note_amax_blocks(ctx, p.fin, fgrid);
    return hipGetLastError();
}

template <int OP>
static int run_contraction(adapt_ctx *ctx, const ContractArgs &a, adapt_fmt fa, adapt_fmt fb, adapt_epilogue ep, size_t ws_offset)
{
    ContractPlan p;
    if (int s = plan_contraction<OP>(ctx, a, fa, fb, ep, ws_offset, p)) return s;
    hipError_t e = launch_planned<OP>(ctx, p);
    if (e == hipSuccess) e = finish_planned(ctx, p);
    return hip_status(ctx, e);
}

// ---- layers with few input channels ------------------------------------------------------------
// The first layer of an image network has 3 input channels: too few for 16-byte operand loads, so
// the contraction would gather element by element.  Such layers run on copies of x and w with
// zero channels appended up to 16 (in the context's workspace): the zeros add nothing to any sum, the
// outputs keep their logical shape and index (and with it their rounding bits), and the vector
// paths apply.  Measured on 256 x 32 x 32 x 3 -> 64, <12,9>: fwd 90 -> 60 us, dgrad 277 -> 95, wgrad 104 -> 51.
constexpr int kPadC = 16;

template <typename T>
__global__ void __launch_bounds__(256) pad_channels_kernel(const T *__restrict__ src, T *__restrict__ dst, const uint32_t rows, const int c)
{
    for (uint32_t r = blockIdx.x * 256 + threadIdx.x; r < rows; r += gridDim.x * 256) {
        constexpr int PER = 4 / (int)sizeof(T);                      // codes per 32-bit word
        uint32_t wds[kPadC / PER];
#pragma unroll
        for (int q = 0; q < kPadC / PER; ++q) wds[q] = 0;
#pragma unroll
        for (int e = 0; e < kPadC; ++e) {
            const uint32_t v = e < c ? (uint32_t)src[(size_t)r * c + e] & (sizeof(T) == 1 ? 0xffu : 0xffffu) : 0u;
            wds[e / PER] |= v << (8 * (int)sizeof(T) * (e % PER));
        }
        uint4 *o = reinterpret_cast<uint4 *>(dst + (size_t)r * kPadC);
#pragma unroll
        for (int q = 0; q < kPadC / PER / 4; ++q) o[q] = make_uint4(wds[4 * q], wds[4 * q + 1], wds[4 * q + 2], wds[4 * q + 3]);
    }
}

// Appends zero channels to a [rows][c] tensor of es-byte codes; the copy lives at scratch + off, which is advanced.
static int pad_channels(adapt_ctx *ctx, const void *src, int es, size_t rows, int c, size_t &off, const void **out)
{
    const size_t bytes = rows * kPadC * (size_t)es;
    off = (off + 255) & ~(size_t)255;
    if (rows >= ((size_t)1 << 31) || off + bytes > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    char *dst = scratch(ctx) + off;
    const unsigned grid = (unsigned)std::min<size_t>(std::max<size_t>((rows + 255) / 256, 1), (size_t)ctx->num_cu * 8);
    if (es == 1)
        hipLaunchKernelGGL(pad_channels_kernel<int8_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int8_t *>(src),
                           reinterpret_cast<int8_t *>(dst), (uint32_t)rows, c);
    else
        hipLaunchKernelGGL(pad_channels_kernel<int16_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int16_t *>(src),
                           reinterpret_cast<int16_t *>(dst), (uint32_t)rows, c);
    if (hipGetLastError() != hipSuccess) return ADAPT_EHIP;
    *out = dst;
    off += bytes;
    return ADAPT_OK;
}

// A classifier has 10 or 100 output channels: the rows of dy are then not a multiple of 16 codes, and both gradient
// contractions would gather dy element by element.  They run on a copy of dy with zero channels appended up to the
// next multiple of 16 instead (in the context's workspace): zeros add nothing to the data gradient (the filter rows
// that would meet them lie beyond the filter tensor and read as zero as well), and the weight gradient keeps its
// d.k real rows.  Measured on 256 x 512 -> 100, one limb: dgrad 25 -> 9 us, wgrad 30 -> 12 us.
template <typename T>
__global__ void __launch_bounds__(256)
pad_rows_kernel(const T *__restrict__ src, T *__restrict__ dst, const uint64_t chunks, const int c, const int c_to)
{
    constexpr int PER = 16 / (int)sizeof(T);                       // codes per 16-byte chunk
    const int cpr = c_to / PER;                                      // chunks per row
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < chunks; i += (uint64_t)gridDim.x * 256) {
        const uint64_t r = i / (uint64_t)cpr;
        const int e0 = (int)(i - r * cpr) * PER;
        T v[PER];
#pragma unroll
        for (int e = 0; e < PER; ++e) v[e] = e0 + e < c ? src[r * (uint64_t)c + e0 + e] : (T)0;
        reinterpret_cast<uint4 *>(dst)[i] = *reinterpret_cast<const uint4 *>(v);
    }
}

static inline int round_up16(int k) { return (k + 15) & ~15; }

// Copy of dy [rows][k] with rows of round_up16(k) codes at scratch + off, which is advanced.
static int pad_cout(adapt_ctx *ctx, const void *dy, int es, size_t rows, int k, size_t &off, const void **out)
{
    const int k_to = round_up16(k);
    const size_t bytes = rows * (size_t)k_to * (size_t)es;
    off = (off + 255) & ~(size_t)255;
    if (bytes >= ((size_t)1 << 32) || off + bytes > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    char *dst = scratch(ctx) + off;
    const uint64_t chunks = bytes / 16;
    const unsigned grid = (unsigned)std::min<uint64_t>(std::max<uint64_t>((chunks + 255) / 256, 1), (uint64_t)ctx->num_cu * 8);
    if (es == 1)
        hipLaunchKernelGGL(pad_rows_kernel<int8_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int8_t *>(dy),
                           reinterpret_cast<int8_t *>(dst), chunks, k, k_to);
    else
        hipLaunchKernelGGL(pad_rows_kernel<int16_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int16_t *>(dy),
                           reinterpret_cast<int16_t *>(dst), chunks, k, k_to);
    if (hipGetLastError() != hipSuccess) return ADAPT_EHIP;
    *out = dst;
    off += bytes;
    return ADAPT_OK;
}

// true when the gradient contractions of this layer take the padded copy of dy
static inline bool wants_cout_pad(const adapt_conv_desc &d) { return d.n > 0 && d.k % 16 != 0 && d.c >= 16 && d.c % 16 == 0; }

static bool epilogue_ok(const adapt_epilogue &ep)
{
    return ep.raw || (fmt_ok(ep.fmt) && (ep.rng.mode == ADAPT_SR || ep.rng.mode == ADAPT_RN_HALF_UP));
}

static bool conv_ok(const adapt_conv_desc &d)
{
    if (d.n < 0 || d.h < 1 || d.w < 1 || d.c < 1 || d.k < 1 || d.r < 1 || d.s < 1 || d.stride < 1 || d.pad < 0) return false;
    if (d.h + 2 * d.pad < d.r || d.w + 2 * d.pad < d.s) return false;
    return true;
}

static int fill_conv(ContractArgs &a, const adapt_conv_desc &d)
{
    a.n = d.n; a.h = d.h; a.w = d.w; a.c = d.c; a.k = d.k; a.r = d.r; a.s = d.s; a.stride = d.stride; a.pad = d.pad;
    a.p = (d.h + 2 * d.pad - d.r) / d.stride + 1;
    a.q = (d.w + 2 * d.pad - d.s) / d.stride + 1;
    const long long lim = (1ll << 31) - 1;
    if ((long long)d.n * d.h * d.w >= lim || (long long)d.n * a.p * a.q >= lim || (long long)d.r * d.s * d.c >= lim ||
        (long long)d.r * d.s * d.k >= lim)
        return ADAPT_EUNSUPPORTED;
    // the kernels index every tensor with 32-bit byte offsets (int16 storage assumed)
    const long long lim32 = 1ll << 32;
    if ((long long)d.n * d.h * d.w * d.c * 2 >= lim32 || (long long)d.n * a.p * a.q * d.k * 2 >= lim32 ||
        (long long)d.k * d.r * d.s * d.c * 2 >= lim32)
        return ADAPT_EUNSUPPORTED;
    a.div_c = make_fastdiv(d.c); a.div_s = make_fastdiv(d.s); a.div_q = make_fastdiv(a.q); a.div_p = make_fastdiv(a.p);
    a.div_k = make_fastdiv(d.k); a.div_w = make_fastdiv(d.w); a.div_h = make_fastdiv(d.h);
    a.div_stride = make_fastdiv(d.stride);
    return ADAPT_OK;
}

static int fill_dgrad(ContractArgs &a, const adapt_conv_desc &d, const void *dy, adapt_fmt fdy, const void *w, adapt_fmt fw, void *dx)
{
    if (int s = fill_conv(a, d)) return s;
    a.act = dy; a.wgt = w; a.out = dx;
    a.M = d.n * d.h * d.w; a.N = d.c; a.K = d.r * d.s * d.k;
    a.act_es = storage_bytes(fdy); a.wgt_es = storage_bytes(fw);
    a.act_bytes = (uint32_t)((long long)d.n * a.p * a.q * d.k * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);
    // the vector path of dy keeps one validity bit per filter tap and row: at most 32 taps
    a.act_load = (d.k % 16 == 0 && d.r * d.s <= 32) ? LOAD_VEC : LOAD_SCALAR;
    a.wgt_load = (d.c % 16 == 0 && d.r * d.s <= 32) ? LOAD_ROWS : LOAD_SCALAR;     // rows (c) are contiguous in w[kout][r][s][c]
    a.ldc = d.c;
    a.uniform_tap = d.k % 64 == 0;
    return ADAPT_OK;
}

static int fill_wgrad(ContractArgs &a, const adapt_conv_desc &d, const void *dy, adapt_fmt fdy, const void *x, adapt_fmt fx, void *dw)
{
    if (int s = fill_conv(a, d)) return s;
    a.act = dy; a.wgt = x; a.out = dw;
    a.M = d.k; a.N = d.r * d.s * d.c; a.K = d.n * a.p * a.q;
    a.act_es = storage_bytes(fdy); a.wgt_es = storage_bytes(fx);
    a.act_bytes = (uint32_t)((long long)d.n * a.p * a.q * d.k * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.n * d.h * d.w * d.c * a.wgt_es);
    // rows (kout / c) are the contiguous direction of both operands
    a.act_load = (d.k % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR;
    a.wgt_load = (d.c % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR;
    a.ldc = a.N;
    return ADAPT_OK;
}

static int fill_fwd(ContractArgs &a, const adapt_conv_desc &d, const void *x, adapt_fmt fx, const void *w, adapt_fmt fw, void *y)
{
    if (int s = fill_conv(a, d)) return s;
    a.act = x; a.wgt = w; a.out = y;
    a.M = d.n * a.p * a.q; a.N = d.k; a.K = d.r * d.s * d.c;
    a.act_es = storage_bytes(fx); a.wgt_es = storage_bytes(fw);
    a.act_bytes = (uint32_t)((long long)d.n * d.h * d.w * d.c * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);
    // the vector path of x keeps one validity bit per filter tap and row: at most 32 taps
    a.act_load = (d.c % 16 == 0 && d.r * d.s <= 32) ? LOAD_VEC : LOAD_SCALAR;
    a.wgt_load = a.K % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.ldc = d.k;
    a.uniform_tap = d.c % 64 == 0;
    return ADAPT_OK;
}

// The same contractions on operands with zero channels appended (see pad_channels): `wp` / `xp` hold kPadC channels.
static int fill_fwd_padded(ContractArgs &a, const adapt_conv_desc &d, const void *xp, adapt_fmt fx, const void *wp, adapt_fmt fw, void *y)
{
    adapt_conv_desc d2 = d;
    d2.c = kPadC;
    if (int s = fill_fwd(a, d2, xp, fx, wp, fw, y)) return s;
    a.k_bound = d.r * d.s * d.c;       // the caller's accumulator type follows the logical reduction length
    return ADAPT_OK;
}

static int fill_dgrad_padded(ContractArgs &a, const adapt_conv_desc &d, const void *dy, adapt_fmt fdy, const void *wp, adapt_fmt fw, void *dx)
{
    if (int s = fill_dgrad(a, d, dy, fdy, wp, fw, dx)) return s;
    a.c = kPadC;                       // stride of the filter rows; the output keeps d.c columns
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * kPadC * a.wgt_es);
    a.wgt_load = LOAD_ROWS;
    return ADAPT_OK;
}

// Weight gradient on a padded x: the kernel fills slabs of r*s*kPadC columns, finish_kernel picks the d.c real ones.
static int fill_wgrad_padded(ContractArgs &a, const adapt_conv_desc &d, const void *dy, adapt_fmt fdy, const void *xp, adapt_fmt fx, void *dw)
{
    adapt_conv_desc d2 = d;
    d2.c = kPadC;
    if (int s = fill_wgrad(a, d2, dy, fdy, xp, fx, dw)) return s;
    a.force_finish = 1;
    return ADAPT_OK;
}

static void unpad_wgrad_finish(ContractPlan &p, const adapt_conv_desc &d)
{
    if (p.empty) return;
    p.fin.N = d.r * d.s * d.c;
    p.fin.ldc = p.fin.N;
    p.fin.pad_c = d.c;
    p.fin.pad_to = kPadC;
}

// The gradient contractions on dy with zero channels appended (see pad_cout): dyp has rows of round_up16(d.k) codes.
static int fill_dgrad_kpad(ContractArgs &a, const adapt_conv_desc &d, const void *dyp, adapt_fmt fdy, const void *w, adapt_fmt fw, void *dx)
{
    adapt_conv_desc d2 = d;
    d2.k = round_up16(d.k);
    if (int s = fill_dgrad(a, d2, dyp, fdy, w, fw, dx)) return s;
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);      // the filter rows of the appended channels read as zero
    a.k_bound = d.r * d.s * d.k;       // the caller's accumulator type follows the logical reduction length
    return ADAPT_OK;
}

static int fill_wgrad_kpad(ContractArgs &a, const adapt_conv_desc &d, const void *dyp, adapt_fmt fdy, const void *x, adapt_fmt fx, void *dw)
{
    adapt_conv_desc d2 = d;
    d2.k = round_up16(d.k);
    if (int s = fill_wgrad(a, d2, dyp, fdy, x, fx, dw)) return s;
    a.M = d.k;                         // dw keeps its real rows; the appended ones are never written
    return ADAPT_OK;
}

static void fill_gemm(ContractArgs &a, int transA, int transB, int M, int N, int K, const void *A, adapt_fmt fa, int lda,
                      const void *B, adapt_fmt fb, int ldb, void *C, int ldc)
{
    a.act = A; a.wgt = B; a.out = C;
    a.M = M; a.N = N; a.K = K;
    a.act_es = storage_bytes(fa); a.wgt_es = storage_bytes(fb);
    // extents: the last row may be shorter than the leading dimension
    a.act_bytes = (uint32_t)((((long long)(transA ? K : M) - 1) * lda + (transA ? M : K)) * a.act_es);
    a.wgt_bytes = (uint32_t)((((long long)(transB ? N : K) - 1) * ldb + (transB ? K : N)) * a.wgt_es);
    a.act_rs = transA ? 1 : lda; a.act_ks = transA ? lda : 1;
    a.wgt_rs = transB ? ldb : 1; a.wgt_ks = transB ? 1 : ldb;
    // vector paths need whole 16-element groups (along k, or along rows) inside the matrix and aligned starts
    a.act_load = !transA ? ((K % 16 == 0 && lda % 16 == 0) ? LOAD_VEC : LOAD_SCALAR)
                         : ((M % 16 == 0 && lda % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR);
    a.wgt_load = transB ? ((K % 16 == 0 && ldb % 16 == 0) ? LOAD_VEC : LOAD_SCALAR)
                        : ((N % 16 == 0 && ldb % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR);
    a.ldc = ldc;
}

static bool check_ptrs(const void *x, const void *y, const void *z) { return x && y && z && aligned16(x) && aligned16(y) && aligned16(z); }

}  // namespace adapt

