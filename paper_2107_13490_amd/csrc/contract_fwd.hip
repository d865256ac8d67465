// C entry point of the fwd contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;


extern "C" int adapt_conv_fwd(adapt_ctx *ctx, adapt_conv_desc d, const void *x, adapt_fmt fx, const void *w, adapt_fmt fw,
                              void *y, adapt_epilogue ep)
{
    if (ctx && wants_wide(fx, fw, ep)) {
        if (!conv_ok(d)) return ADAPT_EINVAL;
        if (d.n == 0) return ADAPT_OK;
        if (!check_ptrs(x, w, y)) return ADAPT_EINVAL;
        const int p = (d.h + 2 * d.pad - d.r) / d.stride + 1, q = (d.w + 2 * d.pad - d.s) / d.stride + 1;
        const SubContraction sub = [&](const void *pa, adapt_fmt fpa, const void *pb, adapt_fmt fpb, void *c, adapt_epilogue ex) {
            return adapt_conv_fwd(ctx, d, pa, fpa, pb, fpb, c, ex);
        };
        return wide_contraction(ctx, x, fx, (uint64_t)d.n * d.h * d.w * d.c, w, fw, (uint64_t)d.k * d.r * d.s * d.c, (uint64_t)d.n * p * q * d.k,
                                (int64_t)d.r * d.s * d.c, y, ep, sub);
    }
    if (!ctx || !fmt_ok(fx) || !fmt_ok(fw) || !conv_ok(d)) return ADAPT_EINVAL;
    if (d.n == 0) return ADAPT_OK;
    if (!check_ptrs(x, w, y)) return ADAPT_EINVAL;
    if (!epilogue_ok(ep)) return ADAPT_EINVAL;
    ContractArgs a = {};
    if (d.c < kPadC) {           // few input channels: run on zero-padded copies when the workspace holds them
        size_t off = 0;
        const void *xp, *wp;
        if (pad_channels(ctx, x, storage_bytes(fx), (size_t)d.n * d.h * d.w, d.c, off, &xp) == ADAPT_OK &&
            pad_channels(ctx, w, storage_bytes(fw), (size_t)d.k * d.r * d.s, d.c, off, &wp) == ADAPT_OK &&
            fill_fwd_padded(a, d, xp, fx, wp, fw, y) == ADAPT_OK) {
            const int s = run_contraction<OP_FWD>(ctx, a, fx, fw, ep, off);
            if (s != ADAPT_EWORKSPACE) return s;
        }
        a = ContractArgs{};
    }
    if (int s = fill_fwd(a, d, x, fx, w, fw, y)) return s;
    return run_contraction<OP_FWD>(ctx, a, fx, fw, ep, 0);
}
