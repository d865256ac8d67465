// adapt_workspace_bytes / adapt_reserve_workspace: what a call will take of the context's workspace, from the same
// planning code the call itself runs.
#include "contract_kernel.hpp"

using namespace adapt;

namespace {

constexpr size_t kInvalid = 0;

size_t a256(size_t v) { return (v + 255) & ~(size_t)255; }

// zero-padded copies of a narrow layer's operands (see pad_channels)
size_t pad_bytes(size_t off, size_t rows, int es) { return a256(off) + rows * kPadC * (size_t)es; }

size_t conv_need(adapt_ctx *dry, int call, const adapt_conv_desc &d, adapt_fmt fa, adapt_fmt fb, adapt_fmt fc)
{
    const adapt_epilogue ep = {1, {8, 0}, {ADAPT_RN_HALF_UP, 0, 0}, 0};      // exact output: the widest slabs
    const size_t big = (size_t)1 << 62;
    const bool narrow = d.c < kPadC && d.n > 0;
    const size_t x_rows = (size_t)d.n * d.h * d.w, w_rows = (size_t)d.k * d.r * d.s;
    const size_t dy_rows = (size_t)d.n * ((d.h + 2 * d.pad - d.r) / d.stride + 1) * ((d.w + 2 * d.pad - d.s) / d.stride + 1);
    ContractArgs a = {};
    ContractPlan p;
    size_t need = 0;
    if (call == ADAPT_CALL_CONV_FWD) {                       // operands x (fa), w (fb)
        size_t off = 0;
        if (narrow) {
            off = pad_bytes(pad_bytes(0, x_rows, storage_bytes(fa)), w_rows, storage_bytes(fb));
            if (fill_fwd_padded(a, d, nullptr, fa, nullptr, fb, nullptr) != ADAPT_OK) return kInvalid;
        } else if (fill_fwd(a, d, nullptr, fa, nullptr, fb, nullptr) != ADAPT_OK) return kInvalid;
        if (plan_contraction<OP_FWD>(dry, a, fa, fb, ep, off, p, big) != ADAPT_OK) return kInvalid;
        need = p.ws_end;
    }
    if (call == ADAPT_CALL_CONV_DGRAD || call == ADAPT_CALL_CONV_BACKWARD) {      // operands dy (fa), w (fb)
        size_t off = 0;
        a = ContractArgs{};
        if (narrow) {
            if (call == ADAPT_CALL_CONV_BACKWARD) off = pad_bytes(0, x_rows, storage_bytes(fc));
            off = pad_bytes(off, w_rows, storage_bytes(fb));
            if (fill_dgrad_padded(a, d, nullptr, fa, nullptr, fb, nullptr) != ADAPT_OK) return kInvalid;
        } else if (wants_cout_pad(d) && d.r * d.s <= 32) {   // the copy of dy with zero channels appended, then the plan on it
            off = a256(0) + dy_rows * (size_t)round_up16(d.k) * storage_bytes(fa);
            if (fill_dgrad_kpad(a, d, nullptr, fa, nullptr, fb, nullptr) != ADAPT_OK) return kInvalid;
        } else if (fill_dgrad(a, d, nullptr, fa, nullptr, fb, nullptr) != ADAPT_OK) return kInvalid;
        if (plan_contraction<OP_DGRAD>(dry, a, fa, fb, ep, off, p, big) != ADAPT_OK) return kInvalid;
        need = std::max(need, p.ws_end);
    }
    if (call == ADAPT_CALL_CONV_WGRAD || call == ADAPT_CALL_CONV_BACKWARD) {      // operands dy (fa), x (fb; fc in a backward call)
        const adapt_fmt fx = call == ADAPT_CALL_CONV_BACKWARD ? fc : fb;
        size_t off = 0;
        a = ContractArgs{};
        if (narrow) {
            off = pad_bytes(0, x_rows, storage_bytes(fx));
            if (call == ADAPT_CALL_CONV_BACKWARD) off = pad_bytes(off, w_rows, storage_bytes(fb));
            if (fill_wgrad_padded(a, d, nullptr, fa, nullptr, fx, nullptr) != ADAPT_OK) return kInvalid;
        } else if (wants_cout_pad(d) && (call == ADAPT_CALL_CONV_WGRAD || d.r * d.s <= 32)) {
            off = a256(0) + dy_rows * (size_t)round_up16(d.k) * storage_bytes(fa);
            if (fill_wgrad_kpad(a, d, nullptr, fa, nullptr, fx, nullptr) != ADAPT_OK) return kInvalid;
        } else if (fill_wgrad(a, d, nullptr, fa, nullptr, fx, nullptr) != ADAPT_OK) return kInvalid;
        if (plan_contraction<OP_WGRAD>(dry, a, fa, fx, ep, off, p, big) != ADAPT_OK) return kInvalid;
        need = std::max(need, p.ws_end);
    }
    return need;
}

}  // namespace

// A contraction with an operand above 16 bits runs one narrow contraction per pair of parts (wide.hip): the largest
// need among them, with the query's own call and shapes
static size_t wide_inner_need(const adapt_ctx *ctx, const adapt_workspace_query &q)
{
    adapt_fmt pa[3], pb[3];
    int step;
    const int na = wide_parts(q.fa, pa, &step), nb = wide_parts(q.fb, pb, &step);
    size_t inner = 0;
    for (int i = 0; i < na; ++i)
        for (int j = 0; j < nb; ++j) {
            adapt_workspace_query sub = q;
            sub.fa = pa[i];
            sub.fb = pb[j];
            const size_t need = adapt_workspace_bytes(ctx, &sub);
            if (need == kInvalid) return kInvalid;
            inner = std::max(inner, need);
        }
    return inner;
}

extern "C" size_t adapt_workspace_bytes(const adapt_ctx *ctx, const adapt_workspace_query *q)
{
    if (!q) return kInvalid;
    int num_cu = 0;
    if (ctx) {
        num_cu = ctx->num_cu;
    } else {
        // the current device's size, or (no device: host-side planning) the 256 compute units of an MI355X
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            num_cu = prop.multiProcessorCount;
        } else {
            (void)hipGetLastError();
            num_cu = 256;
        }
    }
    adapt_ctx dry = {};      // plans like a context with unlimited workspace; nothing is launched through it
    dry.num_cu = num_cu;
    const size_t slack = 256;      // alignment of the first block
    switch (q->call) {
        case ADAPT_CALL_QUANTIZE:
            return q->n > ((uint64_t)1 << 40) ? kInvalid : ws_need_quantize(num_cu, q->n) + slack;
        case ADAPT_CALL_QUANTIZE_BATCHED:
            return q->count < 0 ? kInvalid : ws_need_quantize_batched(num_cu, q->count) + slack;
        case ADAPT_CALL_GEMM: {
            if (q->M < 0 || q->N < 0 || q->K < 0 || !fmt_ok_wide(q->fa) || !fmt_ok_wide(q->fb)) return kInvalid;
            if (q->fa.wl > 16 || q->fb.wl > 16) {
                // word lengths above 16: the parts, one exact partial result and the 128-bit sums, after the largest
                // contraction of two 12-bit parts (or of a part and the narrow operand)
                const size_t inner = wide_inner_need(ctx, *q);
                if (inner == kInvalid) return kInvalid;
                const int lda = q->lda ? q->lda : (q->transA ? q->M : q->K), ldb = q->ldb ? q->ldb : (q->transB ? q->K : q->N);
                return std::max<size_t>(inner, (size_t)1 << 20) +
                       ws_need_wide((uint64_t)(q->transA ? q->K : q->M) * lda, q->fa.wl > 16, (uint64_t)(q->transB ? q->N : q->K) * ldb,
                                    q->fb.wl > 16, (uint64_t)q->M * q->N, false) + slack;
            }
            const int lda = q->lda ? q->lda : (q->transA ? q->M : q->K), ldb = q->ldb ? q->ldb : (q->transB ? q->K : q->N);
            ContractArgs a = {};
            fill_gemm(a, q->transA, q->transB, q->M, q->N, q->K, nullptr, q->fa, lda, nullptr, q->fb, ldb, nullptr, q->N);
            ContractPlan p;
            const adapt_epilogue ep = {1, {8, 0}, {ADAPT_RN_HALF_UP, 0, 0}, 0};
            if (plan_contraction<OP_GEMM>(&dry, a, q->fa, q->fb, ep, 0, p, (size_t)1 << 62) != ADAPT_OK) return kInvalid;
            return p.ws_end + slack;
        }
        case ADAPT_CALL_CONV_FWD:
        case ADAPT_CALL_CONV_DGRAD:
        case ADAPT_CALL_CONV_WGRAD:
        case ADAPT_CALL_CONV_BACKWARD: {
            if (q->call != ADAPT_CALL_CONV_BACKWARD && fmt_ok_wide(q->fa) && fmt_ok_wide(q->fb) && (q->fa.wl > 16 || q->fb.wl > 16) &&
                conv_ok(q->conv)) {
                const size_t inner = wide_inner_need(ctx, *q);
                if (inner == kInvalid) return kInvalid;
                const adapt_conv_desc &d = q->conv;
                const uint64_t p = (d.h + 2 * d.pad - d.r) / d.stride + 1, qq = (d.w + 2 * d.pad - d.s) / d.stride + 1;
                const uint64_t nx = (uint64_t)d.n * d.h * d.w * d.c, nw = (uint64_t)d.k * d.r * d.s * d.c, ny = (uint64_t)d.n * p * qq * d.k;
                const uint64_t ea = q->call == ADAPT_CALL_CONV_FWD ? nx : ny, eb = q->call == ADAPT_CALL_CONV_WGRAD ? nx : nw;
                const uint64_t outs = q->call == ADAPT_CALL_CONV_FWD ? ny : q->call == ADAPT_CALL_CONV_DGRAD ? nx : nw;
                return std::max<size_t>(inner, (size_t)1 << 20) + ws_need_wide(ea, q->fa.wl > 16, eb, q->fb.wl > 16, outs, false) + slack;
            }
            if (q->call == ADAPT_CALL_CONV_BACKWARD && fmt_ok_wide(q->fa) && fmt_ok_wide(q->fb) && fmt_ok_wide(q->fc) &&
                (q->fa.wl > 16 || q->fb.wl > 16 || q->fc.wl > 16) && conv_ok(q->conv)) {
                // above 16 bits the backward call runs the two contractions one after the other
                adapt_workspace_query sub = *q;
                sub.call = ADAPT_CALL_CONV_DGRAD;
                const size_t a = adapt_workspace_bytes(ctx, &sub);
                sub.call = ADAPT_CALL_CONV_WGRAD;
                sub.fb = q->fc;
                const size_t b = adapt_workspace_bytes(ctx, &sub);
                return (a == kInvalid || b == kInvalid) ? kInvalid : std::max(a, b);
            }
            if (!fmt_ok(q->fa) || !fmt_ok(q->fb) || !conv_ok(q->conv)) return kInvalid;
            if (q->call == ADAPT_CALL_CONV_BACKWARD && !fmt_ok(q->fc)) return kInvalid;
            const size_t need = conv_need(&dry, q->call, q->conv, q->fa, q->fb, q->fc);
            return need + slack;
        }
        case ADAPT_CALL_KLD_SEARCH:
            if (q->wl_lo < 2 || q->wl_hi > 32 || q->wl_lo > q->wl_hi || q->bins < 2 || q->bins > 65536) return kInvalid;
            return ws_need_kld_search(num_cu, q->n, q->wl_lo, q->wl_hi, q->bins) + slack;
        case ADAPT_CALL_KLD_SEARCH_BATCHED:
            if (q->wl_lo < 2 || q->wl_hi > 32 || q->wl_lo > q->wl_hi || q->count < 0 || (q->count > 0 && !q->kld_items)) return kInvalid;
            for (int t = 0; t < q->count; ++t)
                if (q->kld_items[t].bins < 2 || q->kld_items[t].bins > 65536) return kInvalid;
            return ws_need_kld_search_batched(num_cu, q->kld_items, q->count, q->wl_lo, q->wl_hi) + slack;
        case ADAPT_CALL_SGD_UPDATE:
            return ws_need_sgd_update(num_cu, q->n) + slack;
        case ADAPT_CALL_GRADIENT_DIVERSITY:
            return q->count < 1 ? kInvalid : ws_need_gradient_diversity(q->n, q->count) + slack;
        case ADAPT_CALL_REQUANTIZE_FIT:
            return ws_need_requantize_fit(num_cu, q->n) + slack;
        default:
            return kInvalid;
    }
}

extern "C" int adapt_reserve_workspace(adapt_ctx *ctx, size_t bytes)
{
    if (!ctx) return ADAPT_EINVAL;
    if (bytes + kCtlBytes <= ctx->ws_bytes) return ADAPT_OK;
    hipError_t e = hipStreamSynchronize(ctx->stream);      // nothing in flight may still use the old block
    char *grown = nullptr;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&grown), bytes + kCtlBytes);
    if (e == hipSuccess) e = hipMemset(grown, 0, kCtlBytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (grown) (void)hipFree(grown);
        return hip_status(ctx, e);
    }
    (void)hipFree(ctx->ws);
    ctx->ws = grown;
    ctx->ws_bytes = bytes + kCtlBytes;
    return ADAPT_OK;
}
