// C entry point of the dgrad contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

namespace adapt {
hipError_t launch_planned_dgrad(adapt_ctx *ctx, const ContractPlan &p) { return launch_planned<OP_DGRAD>(ctx, p); }
}  // namespace adapt

extern "C" int adapt_conv_dgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy, const void *w,
                                adapt_fmt fw, void *dx, adapt_epilogue ep)
{
    if (ctx && wants_wide(fdy, fw, ep)) {
        if (!conv_ok(d)) return ADAPT_EINVAL;
        if (d.n == 0) return ADAPT_OK;
        if (!check_ptrs(dy, w, dx)) return ADAPT_EINVAL;
        const int p = (d.h + 2 * d.pad - d.r) / d.stride + 1, q = (d.w + 2 * d.pad - d.s) / d.stride + 1;
        const SubContraction sub = [&](const void *pa, adapt_fmt fpa, const void *pb, adapt_fmt fpb, void *c, adapt_epilogue ex) {
            return adapt_conv_dgrad(ctx, d, pa, fpa, pb, fpb, c, ex);
        };
        return wide_contraction(ctx, dy, fdy, (uint64_t)d.n * p * q * d.k, w, fw, (uint64_t)d.k * d.r * d.s * d.c, (uint64_t)d.n * d.h * d.w * d.c,
                                (int64_t)d.r * d.s * d.k, dx, ep, sub);
    }
    if (!ctx || !fmt_ok(fdy) || !fmt_ok(fw) || !conv_ok(d)) return ADAPT_EINVAL;
    if (d.n == 0) return ADAPT_OK;
    if (!check_ptrs(dy, w, dx)) return ADAPT_EINVAL;
    if (!epilogue_ok(ep)) return ADAPT_EINVAL;
    ContractArgs a = {};
    if (d.c < kPadC) {           // few input channels: the filters get zero channels appended (vector loads of their rows)
        size_t off = 0;
        const void *wp;
        if (pad_channels(ctx, w, storage_bytes(fw), (size_t)d.k * d.r * d.s, d.c, off, &wp) == ADAPT_OK &&
            fill_dgrad_padded(a, d, dy, fdy, wp, fw, dx) == ADAPT_OK) {
            const int s = run_contraction<OP_DGRAD>(ctx, a, fdy, fw, ep, off);
            if (s != ADAPT_EWORKSPACE) return s;
        }
        a = ContractArgs{};
    }
    if (wants_cout_pad(d) && d.r * d.s <= 32) {      // output channels not a multiple of 16: dy with zero channels appended
        size_t off = 0;
        const void *dyp;
        if (pad_cout(ctx, dy, storage_bytes(fdy), (size_t)d.n * ((d.h + 2 * d.pad - d.r) / d.stride + 1) * ((d.w + 2 * d.pad - d.s) / d.stride + 1),
                     d.k, off, &dyp) == ADAPT_OK &&
            fill_dgrad_kpad(a, d, dyp, fdy, w, fw, dx) == ADAPT_OK) {
            const int s = run_contraction<OP_DGRAD>(ctx, a, fdy, fw, ep, off);
            if (s != ADAPT_EWORKSPACE) return s;
        }
        a = ContractArgs{};
    }
    if (int s = fill_dgrad(a, d, dy, fdy, w, fw, dx)) return s;
    return run_contraction<OP_DGRAD>(ctx, a, fdy, fw, ep, 0);
}

