// C entry point of the gemm contraction; the kernel template lives in contract_kernel.hpp
#include "contract_kernel.hpp"

using namespace adapt;

extern "C" int adapt_fxp_gemm(adapt_ctx *ctx, int transA, int transB, int M, int N, int K, const void *A, adapt_fmt fa,
                              int lda, const void *B, adapt_fmt fb, int ldb, void *C, int ldc, adapt_epilogue ep)
{
    if (!ctx || !fmt_ok(fa) || !fmt_ok(fb) || M < 0 || N < 0 || K < 0) return ADAPT_EINVAL;
    if (M == 0 || N == 0) return ADAPT_OK;
    if (!C || !aligned16(C) || ldc < N) return ADAPT_EINVAL;
    if (K > 0 && (!A || !B || !aligned16(A) || !aligned16(B))) return ADAPT_EINVAL;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return ADAPT_EINVAL;
    // the kernels index every tensor with 32-bit element offsets
    if ((long long)(transA ? K : M) * lda * storage_bytes(fa) >= (1ll << 32) || (long long)(transB ? N : K) * ldb * storage_bytes(fb) >= (1ll << 32))
        return ADAPT_EUNSUPPORTED;
    ContractArgs a = {};
    a.act = A; a.wgt = B; a.out = C;
    a.M = M; a.N = N; a.K = K;
    a.act_es = storage_bytes(fa); a.wgt_es = storage_bytes(fb);
    // extents: the last row may be shorter than the leading dimension
    a.act_bytes = (uint32_t)((((long long)(transA ? K : M) - 1) * lda + (transA ? M : K)) * a.act_es);
    a.wgt_bytes = (uint32_t)((((long long)(transB ? N : K) - 1) * ldb + (transB ? K : N)) * a.wgt_es);
    a.act_rs = transA ? 1 : lda; a.act_ks = transA ? lda : 1;
    a.wgt_rs = transB ? ldb : 1; a.wgt_ks = transB ? 1 : ldb;
    // vector paths need whole 16-element groups (along k, or along rows) inside the matrix and aligned starts
    a.act_load = !transA ? ((K % 16 == 0 && lda % 16 == 0) ? LOAD_VEC : LOAD_SCALAR)
                         : ((M % 16 == 0 && lda % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR);
    a.wgt_load = transB ? ((K % 16 == 0 && ldb % 16 == 0) ? LOAD_VEC : LOAD_SCALAR)
                        : ((N % 16 == 0 && ldb % 16 == 0) ? LOAD_ROWS : LOAD_SCALAR);
    a.ldc = ldc;
    return run_contraction<OP_GEMM>(ctx, a, fa, fb, ep, 0);
}

