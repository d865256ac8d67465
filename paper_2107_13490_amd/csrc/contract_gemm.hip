// C entry point of the gemm contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

extern "C" int adapt_fxp_gemm(adapt_ctx *ctx, int transA, int transB, int M, int N, int K, const void *A, adapt_fmt fa,
                              int lda, const void *B, adapt_fmt fb, int ldb, void *C, int ldc, adapt_epilogue ep)
{
    if (ctx && wants_wide(fa, fb, ep)) {
        if (M < 0 || N < 0 || K < 0) return ADAPT_EINVAL;
        if (M == 0 || N == 0) return ADAPT_OK;
        if (!C || !aligned16(C) || (K > 0 && (!A || !B || !aligned16(A) || !aligned16(B)))) return ADAPT_EINVAL;
        if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return ADAPT_EINVAL;
        if (ldc != N || K == 0) return ADAPT_EUNSUPPORTED;
        const SubContraction sub = [&](const void *pa, adapt_fmt fpa, const void *pb, adapt_fmt fpb, void *c, adapt_epilogue ex) {
            return adapt_fxp_gemm(ctx, transA, transB, M, N, K, pa, fpa, lda, pb, fpb, ldb, c, N, ex);
        };
        return wide_contraction(ctx, A, fa, (uint64_t)(transA ? K : M) * lda, B, fb, (uint64_t)(transB ? N : K) * ldb, (uint64_t)M * N, K, C,
                                ep, sub);
    }
    if (!ctx || !fmt_ok(fa) || !fmt_ok(fb) || M < 0 || N < 0 || K < 0) return ADAPT_EINVAL;
    if (M == 0 || N == 0) return ADAPT_OK;
    if (!C || !aligned16(C) || ldc < N) return ADAPT_EINVAL;
    if (K > 0 && (!A || !B || !aligned16(A) || !aligned16(B))) return ADAPT_EINVAL;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return ADAPT_EINVAL;
    // the kernels index every tensor with 32-bit element offsets
    if ((long long)(transA ? K : M) * lda * storage_bytes(fa) >= (1ll << 32) || (long long)(transB ? N : K) * ldb * storage_bytes(fb) >= (1ll << 32))
        return ADAPT_EUNSUPPORTED;
    ContractArgs a = {};
    fill_gemm(a, transA, transB, M, N, K, A, fa, lda, B, fb, ldb, C, ldc);
    return run_contraction<OP_GEMM>(ctx, a, fa, fb, ep, 0);
}

