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
    // filters re-laid-out as [c][r][s][kout] so that the reduction index is contiguous
    const size_t wbytes = (size_t)d.k * d.r * d.s * d.c * storage_bytes(fw);
    if (wbytes > scratch_bytes(ctx)) return ADAPT_EWORKSPACE;
    void *wt = scratch(ctx);
    const unsigned grid = (unsigned)std::min<size_t>(((size_t)d.k * d.r * d.s * d.c + 255) / 256, (size_t)ctx->num_cu * 8);
    if (storage_bytes(fw) == 1)
        hipLaunchKernelGGL(relayout_filter_kernel<int8_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int8_t *>(w),
                           static_cast<int8_t *>(wt), d.k, d.r * d.s, d.c);
    else
        hipLaunchKernelGGL(relayout_filter_kernel<int16_t>, dim3(grid), dim3(256), 0, ctx->stream, static_cast<const int16_t *>(w),
                           static_cast<int16_t *>(wt), d.k, d.r * d.s, d.c);
    a.act = dy; a.wgt = wt; a.out = dx;
    a.M = d.n * d.h * d.w; a.N = d.c; a.K = d.r * d.s * d.k;
    a.act_es = storage_bytes(fdy); a.wgt_es = storage_bytes(fw);
    a.act_bytes = (uint32_t)((long long)d.n * a.p * a.q * d.k * a.act_es);
    a.wgt_bytes = (uint32_t)((long long)d.k * d.r * d.s * d.c * a.wgt_es);
    a.act_load = d.k % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.wgt_load = a.K % 16 == 0 ? LOAD_VEC : LOAD_SCALAR;
    a.ldc = d.c;
    a.uniform_tap = d.k % 64 == 0;
    return run_contraction<OP_DGRAD>(ctx, a, fdy, fw, ep, wbytes);
}

