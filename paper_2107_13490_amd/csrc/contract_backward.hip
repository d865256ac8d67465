// C entry point of a layer's backward pass: data gradient and weight gradient of one convolution
// (Alg. 1, the backward-pass line, per layer).  Results are exactly those of adapt_conv_dgrad and
// adapt_conv_wgrad; when both contractions take a vector path with matching tiles (one limb:
// 192-deep stages; two limbs: int16 operands, equal square tiles) they run as one launch.
#include "contract_pair.hpp"

using namespace adapt;

static bool pairable(const ContractPlan &p, bool is_dgrad)
{
    if (p.empty || p.tile.pipe || p.tile.bkt != (p.limbs == 1 ? 192 : 64)) return false;
    if (p.limbs == 2 && (p.kern.act_es != 2 || p.kern.wgt_es != 2)) return false;      // mixed storage: not paired
    if (is_dgrad) {
        if (p.kern.dg_classes) return false;      // stride 2 in class order: its own kernel, worth more than the shared launch
        if (p.splits != 1 || p.kern.act_load != LOAD_VEC || p.kern.wgt_load != LOAD_ROWS) return false;
    } else {
        if (p.kern.act_load != LOAD_ROWS || p.kern.wgt_load != LOAD_ROWS) return false;
    }
    return (p.tile.bm == 64 || p.tile.bm == 128) && (p.tile.bn == 64 || p.tile.bn == 128);
}

extern "C" int adapt_conv_backward(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy, const void *w,
                                   adapt_fmt fw, const void *x, adapt_fmt fx, void *dx, adapt_epilogue ep_dx, void *dw,
                                   adapt_epilogue ep_dw)
{
    if (ctx && (wants_wide(fdy, fw, ep_dx) || wants_wide(fdy, fx, ep_dw))) {
        // word lengths above 16: the two contractions one after the other, each composed of its parts
        if (d.n > 0)
            if (int s = adapt_conv_dgrad(ctx, d, dy, fdy, w, fw, dx, ep_dx)) return s;
        return adapt_conv_wgrad(ctx, d, dy, fdy, x, fx, dw, ep_dw);
    }
    if (!ctx || !fmt_ok(fdy) || !fmt_ok(fw) || !fmt_ok(fx) || !conv_ok(d)) return ADAPT_EINVAL;
    if (!dw || !aligned16(dw)) return ADAPT_EINVAL;
    if (d.n > 0 && (!check_ptrs(dy, w, dx) || !check_ptrs(dy, x, dw))) return ADAPT_EINVAL;
    if (!epilogue_ok(ep_dx) || !epilogue_ok(ep_dw)) return ADAPT_EINVAL;
    ContractArgs aw = {}, ad = {};
    ContractPlan pd, pw;
    bool planned = false;
    if (d.c < kPadC && d.n > 0) {      // few input channels: zero-padded copies of x and w (see pad_channels)
        size_t off = 0;
        const void *xp, *wp;
        if (pad_channels(ctx, x, storage_bytes(fx), (size_t)d.n * d.h * d.w, d.c, off, &xp) == ADAPT_OK &&
            pad_channels(ctx, w, storage_bytes(fw), (size_t)d.k * d.r * d.s, d.c, off, &wp) == ADAPT_OK &&
            fill_wgrad_padded(aw, d, dy, fdy, xp, fx, dw) == ADAPT_OK && fill_dgrad_padded(ad, d, dy, fdy, wp, fw, dx) == ADAPT_OK) {
            int s = plan_contraction<OP_DGRAD>(ctx, ad, fdy, fw, ep_dx, off, pd);
            if (s == ADAPT_OK) s = plan_contraction<OP_WGRAD>(ctx, aw, fdy, fx, ep_dw, off, pw);
            if (s == ADAPT_OK) {
                unpad_wgrad_finish(pw, d);
                planned = true;
            } else if (s != ADAPT_EWORKSPACE) {
                return s;
            }
        }
    }
    if (!planned && wants_cout_pad(d) && d.r * d.s <= 32) {      // output channels not a multiple of 16 (see pad_cout)
        size_t off = 0;
        const void *dyp;
        const size_t rows = (size_t)d.n * ((d.h + 2 * d.pad - d.r) / d.stride + 1) * ((d.w + 2 * d.pad - d.s) / d.stride + 1);
        aw = ContractArgs{};
        ad = ContractArgs{};
        if (pad_cout(ctx, dy, storage_bytes(fdy), rows, d.k, off, &dyp) == ADAPT_OK && fill_wgrad_kpad(aw, d, dyp, fdy, x, fx, dw) == ADAPT_OK &&
            fill_dgrad_kpad(ad, d, dyp, fdy, w, fw, dx) == ADAPT_OK) {
            int s = plan_contraction<OP_DGRAD>(ctx, ad, fdy, fw, ep_dx, off, pd);
            if (s == ADAPT_OK) s = plan_contraction<OP_WGRAD>(ctx, aw, fdy, fx, ep_dw, off, pw);
            if (s == ADAPT_OK) planned = true;
            else if (s != ADAPT_EWORKSPACE) return s;
        }
    }
    if (!planned) {
        aw = ContractArgs{};
        ad = ContractArgs{};
        if (int s = fill_wgrad(aw, d, dy, fdy, x, fx, dw)) return s;
        if (d.n == 0) {                                                                    // dw = 0, no dx
            if (int s = plan_contraction<OP_WGRAD>(ctx, aw, fdy, fx, ep_dw, 0, pw)) return s;
            hipError_t e0 = launch_planned_wgrad(ctx, pw);
            if (e0 == hipSuccess) e0 = finish_planned(ctx, pw);
            return hip_status(ctx, e0);
        }
        if (int s = fill_dgrad(ad, d, dy, fdy, w, fw, dx)) return s;
        if (int s = plan_contraction<OP_DGRAD>(ctx, ad, fdy, fw, ep_dx, 0, pd)) return s;
        if (int s = plan_contraction<OP_WGRAD>(ctx, aw, fdy, fx, ep_dw, 0, pw)) return s;
    }
    hipError_t e = hipSuccess;
    bool paired = false;
    if (pairable(pd, true) && pairable(pw, false) && pd.limbs == pw.limbs) {
        if (pd.tile.bm == 64 && pd.tile.bn == 64) e = launch_pair_d64x64(ctx, pd, pw, &paired);
        else if (pd.tile.bm == 128 && pd.tile.bn == 64) e = launch_pair_d128x64(ctx, pd, pw, &paired);
        else if (pd.tile.bm == 64 && pd.tile.bn == 128) e = launch_pair_d64x128(ctx, pd, pw, &paired);
        else e = launch_pair_d128x128(ctx, pd, pw, &paired);
        if (e == hipSuccess && paired) e = finish_planned(ctx, pw);
    }
    if (!paired) {
        // one after the other; both may use the scratch from its start because the stream orders them
        e = launch_planned_dgrad(ctx, pd);
        if (e == hipSuccess) e = finish_planned(ctx, pd);
        if (e == hipSuccess) e = launch_planned_wgrad(ctx, pw);
        if (e == hipSuccess) e = finish_planned(ctx, pw);
    }
    return hip_status(ctx, e);
}
