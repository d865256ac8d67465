// C entry point of the fwd contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

ADAPT_PROF_GETTER(adapt_debug_prof_fwd)

extern "C" int adapt_conv_fwd(adapt_ctx *ctx, adapt_conv_desc d, const void *x, adapt_fmt fx, const void *w, adapt_fmt fw,
                              void *y, adapt_epilogue ep)
{
    if (!ctx || !fmt_ok(fx) || !fmt_ok(fw) || !conv_ok(d)) return ADAPT_EINVAL;
    if (d.n == 0) return ADAPT_OK;
    if (!check_ptrs(x, w, y)) return ADAPT_EINVAL;
    ContractArgs a = {};
    if (int s = fill_conv(a, d)) return s;
    a.act = x; a.wgt = w; a.out = y;
    a.M = d.n * a.p * a.q; a.N = d.k; a.K = d.r * d.s * d.c;
    a.act_es = storage_bytes(fx); a.wgt_es = storage_bytes(fw);
    a.act_bytes = (uint32_t)((long long)d.n * d.h * d.w * d.c * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);
    a.act_load = d.c % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.wgt_load = a.K % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.ldc = d.k;
    a.uniform_tap = d.c % 64 == 0;
    return run_contraction<OP_FWD>(ctx, a, fx, fw, ep, 0);
}

