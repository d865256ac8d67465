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
//   dgrad   (n,h,w)      c          (r,s,kout)   dy[n,(h+pad-r)/st,(w+pad-s)/st,kout]   wt[c,r,s,kout]
//   wgrad   kout         (r,s,c)    (n,p,q)      dy[n,p,q,kout]                 x[n,p*st+r-pad,q*st+s-pad,c]
//
// Tiles of ACT and WGT are staged in LDS with k contiguous, and fed to
// v_mfma_i32_32x32x32_i8 with WGT as the row operand, so that a lane ends up holding 16
// consecutive n for one m: the requantizing epilogue then needs one Philox block per 8
// outputs and issues 16-byte stores.
//
// 9..16-bit operands are split on load into two int8 limbs, a = 256*hi + (lo - 128) + 128
// with hi = a >> 8 and lo - 128 = (a & 255) ^ 0x80, both in [-128,127] for every int16 a.
// The four limb products accumulate in three int32 accumulators (hi*hi, cross, lo*lo); the
// "+128" offsets are undone in the epilogue from the row sums of both operands:
//   sum a*b = sum a'b' + 128 (sum a' + sum b') + 16384 * K,   a' = a - 128.
#pragma once
#include <algorithm>

#include "common.hpp"
#include "context.hpp"

namespace adapt {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

enum { OP_GEMM = 0, OP_FWD = 1, OP_DGRAD = 2, OP_WGRAD = 3 };
enum { LOAD_SCALAR = 0, LOAD_VEC = 1, LOAD_TRANS = 2 };
enum { OUT_RAW32 = 0, OUT_RAW64 = 1, OUT_Q8 = 2, OUT_Q16 = 3 };

constexpr int BK = 64;           // k bytes per LDS tile row
constexpr int LDS_ROW = BK + 16; // padded row: 80 B keeps 16-byte fragment reads conflict-free
constexpr int kThreads = 256;

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
    int act_load, wgt_load;      // LOAD_*
    // gemm: element (row,k) at row*rs + k*ks
    long long act_rs, act_ks, wgt_rs, wgt_ks;
    // conv geometry
    int n, h, w, c, k, r, s, stride, pad, p, q;
    FastDiv div_c, div_s, div_q, div_p, div_k, div_w, div_h, div_stride;
    int k_per_split;             // multiple of BK
    long long slab_bytes;        // split-K: split y writes its exact partial sums to out + y*slab_bytes
    long long ldc;               // output row stride in elements
    int out_mode;
    int shift, wl_o, relu, rmode;
    uint64_t seed, stream;
};

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
    if (OP == OP_DGRAD) {
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
    if (OP == OP_DGRAD) return (long long)row * a.K + k;       // filters re-laid-out as [c][r][s][kout]
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
// four int16 in (d0 = e1:e0, d1 = e3:e2) -> high bytes / offset low bytes of e0..e3
__device__ __forceinline__ void split16(uint32_t d0, uint32_t d1, uint32_t &hi, uint32_t &lo)
{
    hi = __builtin_amdgcn_perm(d1, d0, 0x07050301u);
    lo = __builtin_amdgcn_perm(d1, d0, 0x06040200u) ^ 0x80808080u;
}
// four int8 treated as 16-bit codes: high limb is the sign, low limb the offset byte
__device__ __forceinline__ void split8(uint32_t d, uint32_t &hi, uint32_t &lo)
{
    hi = ((d >> 7) & 0x01010101u) * 0xffu;
    lo = d ^ 0x80808080u;
}
// 4x4 byte transpose: in d[k] = bytes of rows 0..3 at k; out o[row] = bytes of k 0..3
__device__ __forceinline__ void transpose4x4(const uint32_t (&d)[4], uint32_t (&o)[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u);
    const uint32_t t1 = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u);
    const uint32_t t2 = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

// ---------------------------------------------------------------------------------------------
// tile staging: global -> registers (prefetch) -> LDS
// A tile is ROWS x BK codes per limb plane, row stride LDS_ROW bytes.  Zero elements are stored
// as code 0, i.e. limbs (hi = 0, lo = 0x80) in two-limb mode.
//
// Work is dealt in units of 16 elements.  LOAD_VEC / LOAD_SCALAR: unit = one row x 16 consecutive
// k.  LOAD_TRANS: unit = 4 consecutive rows x 4 consecutive k (rows contiguous in memory), byte-
// transposed in registers.  Everything that depends only on the unit's row is computed once
// (Loader::init); per k step only the k-dependent part of the address remains.
// ---------------------------------------------------------------------------------------------
template <int ROWS, int LIMBS>
struct Staged {
    static constexpr int UNITS = ROWS * (BK / 16) / kThreads;   // 16-element units per thread
    uint32_t hi[UNITS][4];   // one-limb: the codes themselves
    uint32_t lo[UNITS][4];   // two-limb only
};

__device__ __forceinline__ void zero_unit(uint32_t (&hi)[4], uint32_t (&lo)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) { hi[i] = 0; lo[i] = 0x80808080u; }
}

template <int OP, bool ACT, int MODE, int ROWS, int LIMBS>
struct Loader {
    static constexpr int UNITS = Staged<ROWS, LIMBS>::UNITS;
    long long base[UNITS];   // row part of the element offset
    int a0[UNITS], a1[UNITS];
    bool valid[UNITS];

    __device__ __forceinline__ static int unit_row(int id)
    {
        return MODE == LOAD_TRANS ? ((id >> 2) % (ROWS / 4)) * 4 : (id >> 2);
    }
    __device__ __forceinline__ static int unit_k(int id)
    {
        return MODE == LOAD_TRANS ? ((id & 3) + 4 * (id / ROWS)) * 4 : (id & 3) * 16;
    }

    __device__ __forceinline__ void init(const ContractArgs &a, int row0)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int row = row0 + unit_row(threadIdx.x + u * kThreads);
            valid[u] = row < (ACT ? a.M : a.N);
            a0[u] = 0; a1[u] = 0; base[u] = 0;
            if (MODE == LOAD_SCALAR || !valid[u]) continue;
            if (OP == OP_GEMM) {
                base[u] = (long long)row * (ACT ? a.act_rs : a.wgt_rs);
            } else if (ACT && OP == OP_FWD) {
                const uint32_t pq = fdiv(row, a.div_q), q = row - pq * a.q;
                const uint32_t n = fdiv(pq, a.div_p), p = pq - n * a.p;
                a0[u] = (int)p * a.stride - a.pad;
                a1[u] = (int)q * a.stride - a.pad;
                base[u] = (((long long)n * a.h + a0[u]) * a.w + a1[u]) * a.c;
            } else if (ACT && OP == OP_DGRAD) {
                const uint32_t nh = fdiv(row, a.div_w), w = row - nh * a.w;
                const uint32_t n = fdiv(nh, a.div_h), h = nh - n * a.h;
                a0[u] = (int)h + a.pad;
                a1[u] = (int)w + a.pad;
                base[u] = (long long)n * a.p * a.q * a.k;
            } else if (ACT && OP == OP_WGRAD) {
                base[u] = row;
            } else if (!ACT && OP == OP_WGRAD) {
                const uint32_t tap = fdiv(row, a.div_c), c = row - tap * a.c;
                const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
                a0[u] = (int)r - a.pad;
                a1[u] = (int)s - a.pad;
                base[u] = c;
            } else {
                base[u] = (long long)row * a.K;      // filters: [row][k]
            }
        }
    }

    // element offset of (unit row, k) for the K-contiguous operands, -1 for zeros
    __device__ __forceinline__ long long vec_offset(const ContractArgs &a, int u, int k) const
    {
        if (!valid[u] || k >= a.K) return -1;
        if (ACT && OP == OP_FWD) {
            const uint32_t tap = fdiv(k, a.div_c), c = k - tap * a.c;
            const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
            if ((unsigned)(a0[u] + (int)r) >= (unsigned)a.h || (unsigned)(a1[u] + (int)s) >= (unsigned)a.w) return -1;
            return base[u] + ((long long)r * a.w + s) * a.c + c;
        }
        if (ACT && OP == OP_DGRAD) {
            const uint32_t tap = fdiv(k, a.div_k), ko = k - tap * a.k;
            const uint32_t r = fdiv(tap, a.div_s), s = tap - r * a.s;
            const int hp = a0[u] - (int)r, wp = a1[u] - (int)s;
            if (hp < 0 || wp < 0) return -1;
            uint32_t p = hp, q = wp;
            if (a.stride != 1) {
                p = fdiv(hp, a.div_stride); q = fdiv(wp, a.div_stride);
                if ((int)(p * a.stride) != hp || (int)(q * a.stride) != wp) return -1;
            }
            if ((int)p >= a.p || (int)q >= a.q) return -1;
            return base[u] + ((long long)p * a.q + q) * a.k + ko;
        }
        return base[u] + k;
    }

    __device__ __forceinline__ void load(const ContractArgs &a, int row0, int k0, Staged<ROWS, LIMBS> &st) const
    {
        const void *ptr = ACT ? a.act : a.wgt;
        const int es = ACT ? a.act_es : a.wgt_es;
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id = threadIdx.x + u * kThreads;
            const int k = k0 + unit_k(id);
            if (MODE == LOAD_VEC) {
                const long long off = vec_offset(a, u, k);
                if (off < 0) {
                    zero_unit(st.hi[u], st.lo[u]);
                } else if (es == 1) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const int8_t *>(ptr) + off);
                    const uint32_t raw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (LIMBS == 1) st.hi[u][i] = raw[i]; else split8(raw[i], st.hi[u][i], st.lo[u][i]);
                    }
                } else {
                    const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const int16_t *>(ptr) + off);
                    const uint4 v0 = p[0], v1 = p[1];
                    split16(v0.x, v0.y, st.hi[u][0], st.lo[u][0]);
                    split16(v0.z, v0.w, st.hi[u][1], st.lo[u][1]);
                    split16(v1.x, v1.y, st.hi[u][2], st.lo[u][2]);
                    split16(v1.z, v1.w, st.hi[u][3], st.lo[u][3]);
                }
            } else if (MODE == LOAD_TRANS) {
                uint32_t dh[4], dl[4];
                uint32_t n = 0, p = 0, q = 0;
                if (!ACT && OP == OP_WGRAD) {
                    const uint32_t np = fdiv(k, a.div_q);
                    q = k - np * a.q;
                    n = fdiv(np, a.div_p);
                    p = np - n * a.p;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    long long off = -1;
                    if (valid[u] && k + j < a.K) {
                        if (OP == OP_GEMM) {
                            off = base[u] + (long long)(k + j) * (ACT ? a.act_ks : a.wgt_ks);
                        } else if (ACT) {                  // wgrad: dy[(n,p,q)][kout]
                            off = base[u] + (long long)(k + j) * a.k;
                        } else {                           // wgrad: x[n, p*st+r-pad, q*st+s-pad, c]
                            const int hh = (int)p * a.stride + a0[u], ww = (int)q * a.stride + a1[u];
                            if ((unsigned)hh < (unsigned)a.h && (unsigned)ww < (unsigned)a.w)
                                off = (((long long)n * a.h + hh) * a.w + ww) * a.c + base[u];
                        }
                    }
                    if (!ACT && OP == OP_WGRAD) {
                        if (++q == (uint32_t)a.q) { q = 0; if (++p == (uint32_t)a.p) { p = 0; ++n; } }
                    }
                    if (off < 0) {
                        dh[j] = 0; dl[j] = 0x80808080u;
                    } else if (es == 1) {
                        const uint32_t v = *reinterpret_cast<const uint32_t *>(static_cast<const int8_t *>(ptr) + off);
                        if (LIMBS == 1) dh[j] = v; else split8(v, dh[j], dl[j]);
                    } else {
                        const uint2 v = *reinterpret_cast<const uint2 *>(static_cast<const int16_t *>(ptr) + off);
                        split16(v.x, v.y, dh[j], dl[j]);
                    }
                }
                transpose4x4(dh, st.hi[u]);
                if (LIMBS == 2) transpose4x4(dl, st.lo[u]);
            } else {
                // element-wise gather: any shape, any alignment
                const int row = row0 + unit_row(id);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t h = 0, l = 0;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const long long off = operand_offset<OP, ACT>(a, row, k + 4 * i + b);
                        int v = 0;
                        if (off >= 0)
                            v = es == 1 ? (int)static_cast<const int8_t *>(ptr)[off] : (int)static_cast<const int16_t *>(ptr)[off];
                        if (LIMBS == 1) {
                            h |= (uint32_t)(v & 0xff) << (8 * b);
                        } else {
                            h |= (uint32_t)((v >> 8) & 0xff) << (8 * b);
                            l |= (uint32_t)((v & 0xff) ^ 0x80) << (8 * b);
                        }
                    }
                    st.hi[u][i] = h;
                    st.lo[u][i] = l;
                }
            }
        }
    }

    __device__ __forceinline__ static void store(const Staged<ROWS, LIMBS> &st, char *tile_hi, char *tile_lo)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id = threadIdx.x + u * kThreads;
            if (MODE == LOAD_TRANS) {
                const int o0 = unit_row(id) * LDS_ROW + unit_k(id);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *reinterpret_cast<uint32_t *>(tile_hi + o0 + i * LDS_ROW) = st.hi[u][i];
                    if (LIMBS == 2) *reinterpret_cast<uint32_t *>(tile_lo + o0 + i * LDS_ROW) = st.lo[u][i];
                }
            } else {
                const int o = unit_row(id) * LDS_ROW + unit_k(id);
                *reinterpret_cast<uint4 *>(tile_hi + o) = make_uint4(st.hi[u][0], st.hi[u][1], st.hi[u][2], st.hi[u][3]);
                if (LIMBS == 2)
                    *reinterpret_cast<uint4 *>(tile_lo + o) = make_uint4(st.lo[u][0], st.lo[u][1], st.lo[u][2], st.lo[u][3]);
            }
        }
    }
};

// ---------------------------------------------------------------------------------------------
// accumulator -> output format (the SR rule applied to the accumulator's low bits)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int requantize_one(long long acc, int shift, int wl, int relu, uint32_t r16)
{
    long long q;
    if (shift <= 0) {
        const long long lim = 1ll << 20;               // beyond any 16-bit range: saturates below
        const long long c = acc > lim ? lim : acc < -lim ? -lim : acc;
        q = (-shift >= 40) ? (c > 0 ? (1ll << 60) : c < 0 ? -(1ll << 60) : 0) : (long long)((unsigned long long)c << -shift);
    } else if (shift <= 16) {
        q = (acc + (long long)(r16 >> (16 - shift))) >> shift;
    } else {
        q = ((acc >> (shift - 16)) + (long long)r16) >> 16;
    }
    if (relu && q < 0) q = 0;
    const long long qmax = (1ll << (wl - 1)) - 1, qmin = -(1ll << (wl - 1));
    return (int)(q > qmax ? qmax : q < qmin ? qmin : q);
}

// Writes 16 consecutive outputs (m, n0..n0+15) held by one lane.
__device__ __forceinline__ void emit16(const ContractArgs &a, void *out, int m, int n0, const long long (&v)[16])
{
    if (m >= a.M || n0 >= a.N) return;
    const int cnt = min(16, a.N - n0);
    const long long row = (long long)m * a.ldc + n0;
    switch (a.out_mode) {
        case OUT_RAW32: {
            int32_t *o = static_cast<int32_t *>(out) + row;
            if (cnt == 16 && ((a.ldc | n0) & 3) == 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    reinterpret_cast<int4 *>(o)[i] = make_int4((int)v[4 * i], (int)v[4 * i + 1], (int)v[4 * i + 2], (int)v[4 * i + 3]);
            } else {
                for (int i = 0; i < cnt; ++i) o[i] = (int32_t)v[i];
            }
            break;
        }
        case OUT_RAW64: {
            long long *o = static_cast<long long *>(out) + row;
            for (int i = 0; i < cnt; ++i) o[i] = v[i];
            break;
        }
        default: {
            // requantize: output element index = m * N + n (row-major over the logical tensor)
            const uint64_t idx0 = (uint64_t)m * (uint64_t)a.N + (uint64_t)n0;
            uint32_t r[16];
            if (a.rmode != ADAPT_SR) {
#pragma unroll
                for (int i = 0; i < 16; ++i) r[i] = 0x8000u;
            } else if ((idx0 & 7) == 0) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const u32x4 b = rounding_block(a.seed, a.stream, (idx0 >> 3) + h);
                    r[8 * h + 0] = b.x & 0xffffu; r[8 * h + 1] = b.x >> 16; r[8 * h + 2] = b.y & 0xffffu; r[8 * h + 3] = b.y >> 16;
                    r[8 * h + 4] = b.z & 0xffffu; r[8 * h + 5] = b.z >> 16; r[8 * h + 6] = b.w & 0xffffu; r[8 * h + 7] = b.w >> 16;
                }
            } else {
                for (int i = 0; i < 16; ++i) r[i] = rounding_bits_of(a.seed, a.stream, idx0 + i, ADAPT_SR);
            }
            int q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = requantize_one(v[i], a.shift, a.wl_o, a.relu, r[i]);
            if (a.out_mode == OUT_Q8) {
                int8_t *o = static_cast<int8_t *>(out) + row;
                if (cnt == 16 && ((a.ldc | n0) & 15) == 0) {
                    uint32_t w[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        w[i] = (uint32_t)(q[4 * i] & 0xff) | ((uint32_t)(q[4 * i + 1] & 0xff) << 8) |
                               ((uint32_t)(q[4 * i + 2] & 0xff) << 16) | ((uint32_t)(q[4 * i + 3] & 0xff) << 24);
                    *reinterpret_cast<uint4 *>(o) = make_uint4(w[0], w[1], w[2], w[3]);
                } else {
                    for (int i = 0; i < cnt; ++i) o[i] = (int8_t)q[i];
                }
            } else {
                int16_t *o = static_cast<int16_t *>(out) + row;
                if (cnt == 16 && ((a.ldc | n0) & 7) == 0) {
                    uint32_t w[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) w[i] = (uint32_t)(q[2 * i] & 0xffff) | ((uint32_t)q[2 * i + 1] << 16);
                    reinterpret_cast<uint4 *>(o)[0] = make_uint4(w[0], w[1], w[2], w[3]);
                    reinterpret_cast<uint4 *>(o)[1] = make_uint4(w[4], w[5], w[6], w[7]);
                } else {
                    for (int i = 0; i < cnt; ++i) o[i] = (int16_t)q[i];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// the kernel: block tile BM x BN, 4 wavefronts in a WGM x WGN grid, wave tile (BM/WGM) x (BN/WGN)
// built from 32x32 MFMA blocks.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int dot4_ones(uint32_t v) { return __builtin_amdgcn_sdot4((int)v, 0x01010101, 0, false); }

template <int OP, int LIMBS, int AMODE, int WMODE, int BM, int BN, int WGM, int WGN>
__global__ void __launch_bounds__(kThreads)
contract_kernel(const ContractArgs a)
{
    static_assert(WGM * WGN == 4, "four wavefronts per block");
    constexpr int WM = BM / WGM, WN = BN / WGN;     // wave tile
    constexpr int MB = WM / 32, NB = WN / 32;       // 32x32 blocks per wave
    constexpr int TILE_A = BM * LDS_ROW, TILE_B = BN * LDS_ROW;
    constexpr int STAGE = (TILE_A + TILE_B) * LIMBS;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, g = lane >> 5;
    // MFMA row i of the WGT operand carries n_local = perm(i), so that accumulator register r of
    // a lane is n_local = 16*g + r
    const int nperm = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);

    const int tiles_n = (a.N + BN - 1) / BN;
    const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int kbeg = blockIdx.y * a.k_per_split;
    const int kend = min(a.K, kbeg + a.k_per_split);
    const int ksteps = (kend - kbeg + BK - 1) / BK;

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

    Staged<BM, LIMBS> sa;
    Staged<BN, LIMBS> sb;
    Loader<OP, true, AMODE, BM, LIMBS> la;
    Loader<OP, false, WMODE, BN, LIMBS> lb;
    ADAPT_STAMP(0);
    la.init(a, m0);
    lb.init(a, n0);
    ADAPT_STAMP(1);
    auto tiles = [&](int buf, char *&a_hi, char *&a_lo, char *&b_hi, char *&b_lo) {
        char *base = smem + buf * STAGE;
        a_hi = base; a_lo = base + TILE_A;
        b_hi = base + TILE_A * LIMBS; b_lo = b_hi + TILE_B;
    };

    if (ksteps > 0) {
        la.load(a, m0, kbeg, sa);
        lb.load(a, n0, kbeg, sb);
        char *ah, *al, *bh, *bl;
        tiles(0, ah, al, bh, bl);
        la.store(sa, ah, al);
        lb.store(sb, bh, bl);
    }
    __syncthreads();
    ADAPT_STAMP(2);

    for (int kt = 0; kt < ksteps; ++kt) {
        const bool more = kt + 1 < ksteps;
        if (more) {
            la.load(a, m0, kbeg + (kt + 1) * BK, sa);
            lb.load(a, n0, kbeg + (kt + 1) * BK, sb);
        }
        char *ah, *al, *bh, *bl;
        tiles(kt & 1, ah, al, bh, bl);
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            const int koff = ks * 32 + g * 16;
            v4i fa_h[MB], fa_l[MB], fb_h[NB], fb_l[NB];
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                const int o = (wm * WM + j * 32 + l32) * LDS_ROW + koff;
                fa_h[j] = *reinterpret_cast<const v4i *>(ah + o);
                if (LIMBS == 2) fa_l[j] = *reinterpret_cast<const v4i *>(al + o);
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int o = (wn * WN + i * 32 + nperm) * LDS_ROW + koff;
                fb_h[i] = *reinterpret_cast<const v4i *>(bh + o);
                if (LIMBS == 2) fb_l[i] = *reinterpret_cast<const v4i *>(bl + o);
            }
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int j = 0; j < MB; ++j) {
                    acc_hh[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb_h[i], fa_h[j], acc_hh[i][j], 0, 0, 0);
                    if (LIMBS == 2) {
                        acc_x[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb_h[i], fa_l[j], acc_x[i][j], 0, 0, 0);
                        acc_x[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb_l[i], fa_h[j], acc_x[i][j], 0, 0, 0);
                        acc_ll[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb_l[i], fa_l[j], acc_ll[i][j], 0, 0, 0);
                    }
                }
            if (LIMBS == 2) {
#pragma unroll
                for (int j = 0; j < MB; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        sum_m[j] += 256 * dot4_ones((uint32_t)fa_h[j][e]) + dot4_ones((uint32_t)fa_l[j][e]);
#pragma unroll
                for (int i = 0; i < NB; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        sum_n[i] += 256 * dot4_ones((uint32_t)fb_h[i][e]) + dot4_ones((uint32_t)fb_l[i][e]);
            }
        }
        if (more) {
            tiles((kt + 1) & 1, ah, al, bh, bl);
            la.store(sa, ah, al);
            lb.store(sb, bh, bl);
        }
        __syncthreads();
    }

    ADAPT_STAMP(3);
    // ---- epilogue -----------------------------------------------------------------------------
    // lane holds, for block (i,j): m = m0 + wm*WM + j*32 + l32, n = n0 + wn*WN + i*32 + 16*g + r
    long long corr_m[MB];
    int *sn = reinterpret_cast<int *>(smem);          // [4 waves][NB][32] n-side sums
    if (LIMBS == 2) {
#pragma unroll
        for (int j = 0; j < MB; ++j) corr_m[j] = (long long)(sum_m[j] + __shfl_xor(sum_m[j], 32, 64));
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int t = sum_n[i] + __shfl_xor(sum_n[i], 32, 64);
            if (g == 0) sn[(wave * NB + i) * 32 + nperm] = t;
        }
        __syncthreads();
    }
    const long long kpad = (long long)ksteps * BK;
    void *out = static_cast<char *>(a.out) + (long long)blockIdx.y * a.slab_bytes;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            long long v[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (LIMBS == 1) {
                    v[r] = acc_hh[i][j][r];
                } else {
                    const long long s_n = sn[(wave * NB + i) * 32 + 16 * g + r];
                    v[r] = ((long long)acc_hh[i][j][r] << 16) + ((long long)acc_x[i][j][r] << 8) + (long long)acc_ll[i][j][r] +
                           128 * (corr_m[j] + s_n) + 16384 * kpad;
                }
            }
            emit16(a, out, m0 + wm * WM + j * 32 + l32, n0 + wn * WN + i * 32 + 16 * g, v);
        }
    ADAPT_STAMP(4);
}

// ---- helpers: filter re-layout for dgrad, split-K finish --------------------------------------------
// w[k][rs][c] -> wt[c][rs][k]
template <typename T>
__global__ void relayout_filter_kernel(const T *__restrict__ w, T *__restrict__ wt, int K, int RS, int C)
{
    const size_t total = (size_t)K * RS * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int k = (int)(i % K);
        const size_t t = i / K;
        const int rs = (int)(t % RS), c = (int)(t / RS);
        wt[i] = w[((size_t)k * RS + rs) * C + c];
    }
}

// split-K: sums the `splits` slabs of exact partial sums (dense M x N each) and converts
template <typename AccT>
__global__ void __launch_bounds__(256)
finish_kernel(const AccT *__restrict__ ws, int splits, ContractArgs a)
{
    const size_t total = (size_t)a.M * a.N;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        long long v = 0;
        for (int y = 0; y < splits; ++y) v += (long long)ws[(size_t)y * total + i];
        const size_t m = i / a.N, n = i % a.N;
        const size_t o = m * (size_t)a.ldc + n;
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
}

// ---- host side ---------------------------------------------------------------------------------
struct TileShape { int bm, bn; };

template <int OP, int LIMBS, int AMODE, int WMODE, int BM, int BN, int WGM, int WGN>
static hipError_t launch_variant(adapt_ctx *ctx, const ContractArgs &a, int splits)
{
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    const size_t lds = (size_t)2 * (BM + BN) * LDS_ROW * LIMBS;
    auto kern = contract_kernel<OP, LIMBS, AMODE, WMODE, BM, BN, WGM, WGN>;
    static bool attr_done = false;
    if (!attr_done && lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles, splits), dim3(kThreads), lds, ctx->stream, a);
    return hipGetLastError();
}

template <int OP, int LIMBS, int AMODE, int WMODE>
static hipError_t launch_tile(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    if (AMODE == LOAD_SCALAR) return launch_variant<OP, LIMBS, AMODE, WMODE, 128, 64, 2, 2>(ctx, a, splits);
    if (t.bn == 64) return launch_variant<OP, LIMBS, AMODE, WMODE, 128, 64, 2, 2>(ctx, a, splits);
    if (t.bn == 192) return launch_variant<OP, LIMBS, AMODE, WMODE, 128, 192, 2, 2>(ctx, a, splits);
    return launch_variant<OP, LIMBS, AMODE, WMODE, 128, 128, 2, 2>(ctx, a, splits);
}

// Instantiated load-mode pairs: the vector paths that each op can use, and one element-wise
// fallback per op for shapes that are not multiples of the vector width.
template <int OP, int LIMBS>
static hipError_t launch_modes(adapt_ctx *ctx, const ContractArgs &a, int splits, TileShape t)
{
    const bool scalar = a.act_load == LOAD_SCALAR || a.wgt_load == LOAD_SCALAR;
    if (scalar) return launch_tile<OP, LIMBS, LOAD_SCALAR, LOAD_SCALAR>(ctx, a, splits, t);
    if (OP == OP_WGRAD) return launch_tile<OP, LIMBS, LOAD_TRANS, LOAD_TRANS>(ctx, a, splits, t);
    if (OP == OP_GEMM) {
        if (a.act_load == LOAD_VEC && a.wgt_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_VEC>(ctx, a, splits, t);
        if (a.act_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_TRANS>(ctx, a, splits, t);
        if (a.wgt_load == LOAD_VEC) return launch_tile<OP, LIMBS, LOAD_TRANS, LOAD_VEC>(ctx, a, splits, t);
        return launch_tile<OP, LIMBS, LOAD_TRANS, LOAD_TRANS>(ctx, a, splits, t);
    }
    return launch_tile<OP, LIMBS, LOAD_VEC, LOAD_VEC>(ctx, a, splits, t);
}

static TileShape pick_tile(const ContractArgs &a)
{
    TileShape t;
    t.bm = 128;
    if (a.N <= 64) t.bn = 64;
    else if (a.N % 192 == 0 || (a.N > 128 && a.N <= 192)) t.bn = 192;
    else if ((a.N + 127) / 128 * 128 - a.N >= 64) t.bn = 64;
    else t.bn = 128;
    return t;
}

// Fills the parts of ContractArgs common to all ops and runs the kernel.  K is split across
// blocks (exact partial sums in workspace slabs, summed by finish_kernel) when a single block
// could overflow its int32 accumulators or when the output has too few tiles to fill the GPU.
template <int OP>
static int run_contraction(adapt_ctx *ctx, ContractArgs a, adapt_fmt fa, adapt_fmt fb, adapt_epilogue ep,
                           size_t ws_offset /* bytes of scratch already in use */)
{
    const int limbs = (fa.wl > 8 || fb.wl > 8) ? 2 : 1;
    const int bits = adapt_acc_bits(a.K, fa, fb);
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
    if (a.M == 0 || a.N == 0) return ADAPT_OK;

    const TileShape t = pick_tile(a);
    const long long tiles = (long long)((a.M + t.bm - 1) / t.bm) * ((a.N + t.bn - 1) / t.bn);
    // int32 accumulators: |product| <= 2^14 per limb pair, the cross accumulator holds two per k
    const int k_cap = limbs == 1 ? 65536 : 32768;
    int splits = (a.K + k_cap - 1) / k_cap;
    if (tiles < ctx->num_cu && a.K >= 8 * BK) {
        const long long want = (ctx->num_cu + tiles - 1) / tiles;
        const long long max_by_k = a.K / (4 * BK);
        splits = (int)std::max<long long>(splits, std::min(want, std::max(1ll, max_by_k)));
    }
    if (splits < 1) splits = 1;
    int k_per = ((a.K + splits - 1) / splits + BK - 1) / BK * BK;
    if (k_per == 0) k_per = BK;
    splits = a.K == 0 ? 1 : (a.K + k_per - 1) / k_per;
    a.k_per_split = k_per;
    a.slab_bytes = 0;

    hipError_t e;
    if (splits == 1) {
        a.out_mode = final_mode;
        e = limbs == 1 ? launch_modes<OP, 1>(ctx, a, 1, t) : launch_modes<OP, 2>(ctx, a, 1, t);
        return hip_status(ctx, e);
    }
    // a partial sum is bounded like the total, so the slabs use the total's accumulator type
    const size_t acc_bytes = bits == 32 ? 4 : 8;
    const size_t slab = (size_t)a.M * a.N * acc_bytes;
    const size_t off = (ws_offset + 255) & ~(size_t)255;
    if (off + slab * splits > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    char *acc = scratch(ctx) + off;
    ContractArgs part = a;
    part.out = acc;
    part.ldc = a.N;
    part.slab_bytes = (long long)slab;
    part.out_mode = bits == 32 ? OUT_RAW32 : OUT_RAW64;
    e = limbs == 1 ? launch_modes<OP, 1>(ctx, part, splits, t) : launch_modes<OP, 2>(ctx, part, splits, t);
    if (e != hipSuccess) return hip_status(ctx, e);
    ContractArgs fin = a;
    fin.out_mode = final_mode;
    const unsigned fgrid = (unsigned)std::min<size_t>(((size_t)a.M * a.N + 255) / 256, (size_t)ctx->num_cu * 8);
    if (bits == 32)
        hipLaunchKernelGGL(finish_kernel<int32_t>, dim3(fgrid), dim3(256), 0, ctx->stream, reinterpret_cast<const int32_t *>(acc), splits, fin);
    else
        hipLaunchKernelGGL(finish_kernel<long long>, dim3(fgrid), dim3(256), 0, ctx->stream, reinterpret_cast<const long long *>(acc), splits, fin);
    return hip_status(ctx, hipGetLastError());
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
    a.div_c = make_fastdiv(d.c); a.div_s = make_fastdiv(d.s); a.div_q = make_fastdiv(a.q); a.div_p = make_fastdiv(a.p);
    a.div_k = make_fastdiv(d.k); a.div_w = make_fastdiv(d.w); a.div_h = make_fastdiv(d.h);
    a.div_stride = make_fastdiv(d.stride);
    return ADAPT_OK;
}

static bool check_ptrs(const void *x, const void *y, const void *z) { return x && y && z && aligned16(x) && aligned16(y) && aligned16(z); }

}  // namespace adapt

