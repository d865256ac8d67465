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
    if (int s = fill_wgrad(a, d, dy, fdy, x, fx, dw)) return s;
    return run_contraction<OP_WGRAD>(ctx, a, fdy, fx, ep, 0);
}
