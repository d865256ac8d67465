// C entry point of the wgrad contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

ADAPT_PROF_GETTER(adapt_debug_prof_wgrad)

extern "C" int adapt_conv_wgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy, const void *x,
                                adapt_fmt fx, void *dw, adapt_epilogue ep)
{
    if (!ctx || !fmt_ok(fdy) || !fmt_ok(fx) || !conv_ok(d)) return ADAPT_EINVAL;
    if (!dw || !aligned16(dw)) return ADAPT_EINVAL;
    if (d.n > 0 && !check_ptrs(dy, x, dw)) return ADAPT_EINVAL;
    ContractArgs a = {};
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
    return run_contraction<OP_WGRAD>(ctx, a, fdy, fx, ep, 0);
}
