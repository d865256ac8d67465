// C entry point of the wgrad contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

namespace adapt {
hipError_t launch_planned_wgrad(adapt_ctx *ctx, const ContractPlan &p) { return launch_planned<OP_WGRAD>(ctx, p); }
}  // namespace adapt


extern "C" int adapt_conv_wgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy, const void *x,
                                adapt_fmt fx, void *dw, adapt_epilogue ep)
{
    if (ctx && wants_wide(fdy, fx, ep)) {
        if (!conv_ok(d)) return ADAPT_EINVAL;
        if (!dw || !aligned16(dw) || (d.n > 0 && !check_ptrs(dy, x, dw))) return ADAPT_EINVAL;
        if (d.n == 0) return ADAPT_EUNSUPPORTED;             // (an empty batch would only clear dw)
        const int p = (d.h + 2 * d.pad - d.r) / d.stride + 1, q = (d.w + 2 * d.pad - d.s) / d.stride + 1;
        const SubContraction sub = [&](const void *pa, adapt_fmt fpa, const void *pb, adapt_fmt fpb, void *c, adapt_epilogue ex) {
            return adapt_conv_wgrad(ctx, d, pa, fpa, pb, fpb, c, ex);
        };
        return wide_contraction(ctx, dy, fdy, (uint64_t)d.n * p * q * d.k, x, fx, (uint64_t)d.n * d.h * d.w * d.c, (uint64_t)d.k * d.r * d.s * d.c,
                                (int64_t)d.n * p * q, dw, ep, sub);
    }
    if (!ctx || !fmt_ok(fdy) || !fmt_ok(fx) || !conv_ok(d)) return ADAPT_EINVAL;
    if (!dw || !aligned16(dw)) return ADAPT_EINVAL;
    if (d.n > 0 && !check_ptrs(dy, x, dw)) return ADAPT_EINVAL;
    if (!epilogue_ok(ep)) return ADAPT_EINVAL;
    ContractArgs a = {};
    if (d.c < kPadC && d.n > 0) {      // few input channels: x gets zero channels appended, the finish kernel drops them again
        size_t off = 0;
        const void *xp;
        ContractPlan p;
        if (pad_channels(ctx, x, storage_bytes(fx), (size_t)d.n * d.h * d.w, d.c, off, &xp) == ADAPT_OK &&
            fill_wgrad_padded(a, d, dy, fdy, xp, fx, dw) == ADAPT_OK) {
            const int s = plan_contraction<OP_WGRAD>(ctx, a, fdy, fx, ep, off, p);
            if (s == ADAPT_OK) {
                unpad_wgrad_finish(p, d);
                hipError_t e = launch_planned<OP_WGRAD>(ctx, p);
                if (e == hipSuccess) e = finish_planned(ctx, p);
                return hip_status(ctx, e);
            }
            if (s != ADAPT_EWORKSPACE) return s;
        }
        a = ContractArgs{};
    }
    if (wants_cout_pad(d)) {           // output channels not a multiple of 16: dy with zero channels appended
        size_t off = 0;
        const void *dyp;
        if (pad_cout(ctx, dy, storage_bytes(fdy), (size_t)d.n * ((d.h + 2 * d.pad - d.r) / d.stride + 1) * ((d.w + 2 * d.pad - d.s) / d.stride + 1),
                     d.k, off, &dyp) == ADAPT_OK &&
            fill_wgrad_kpad(a, d, dyp, fdy, x, fx, dw) == ADAPT_OK) {
            const int s = run_contraction<OP_WGRAD>(ctx, a, fdy, fx, ep, off);
            if (s != ADAPT_EWORKSPACE) return s;
        }
        a = ContractArgs{};
    }
    if (int s = fill_wgrad(a, d, dy, fdy, x, fx, dw)) return s;
    return run_contraction<OP_WGRAD>(ctx, a, fdy, fx, ep, 0);
}
