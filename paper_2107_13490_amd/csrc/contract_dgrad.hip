// C entry point of the dgrad contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

ADAPT_PROF_GETTER(adapt_debug_prof_dgrad)

extern "C" int adapt_conv_dgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy, const void *w,
                                adapt_fmt fw, void *dx, adapt_epilogue ep)
{
    if (!ctx || !fmt_ok(fdy) || !fmt_ok(fw) || !conv_ok(d)) return ADAPT_EINVAL;
    if (d.n == 0) return ADAPT_OK;
    if (!check_ptrs(dy, w, dx)) return ADAPT_EINVAL;
    ContractArgs a = {};
    if (int s = fill_conv(a, d)) return s;
    a.act = dy; a.wgt = w; a.out = dx;
    a.M = d.n * d.h * d.w; a.N = d.c; a.K = d.r * d.s * d.k;
    a.act_es = storage_bytes(fdy); a.wgt_es = storage_bytes(fw);
    a.act_bytes = (uint32_t)((long long)d.n * a.p * a.q * d.k * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);
    a.act_load = d.k % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.wgt_load = d.c % 16 == 0 ? LOAD_ROWS : LOAD_SCALAR;     // rows (c) are contiguous in w[kout][r][s][c]
    a.ldc = d.c;
    a.uniform_tap = d.k % 64 == 0;
    return run_contraction<OP_DGRAD>(ctx, a, fdy, fw, ep, 0);
}

