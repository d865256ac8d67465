/* CPU oracle for the integer contractions of AdaPT's fixed-point hot path.
 *
 * TEST INFRASTRUCTURE ONLY: loaded by tests/, the smoke check and the benchmark's
 * cpu_baseline leg; never by the product library.  Shares no code with the HIP path.
 *
 * The paper (Alg. 1, "ForwardPass" on quantized layers; Sec. 3.3 on quantized gradients)
 * does not print a formula for the layer contractions; these are the plain definitions of a
 * zero-padded cross-correlation and of its two adjoints, summed exactly in int64:
 *
 *   fwd  : Y [n,p,q,k] = sum_{r,s,c} X[n, p*st+r-pad, q*st+s-pad, c] * W[k,r,s,c]
 *   dgrad: dX[n,h,w,c] = sum_{k,r,s : h = p*st+r-pad, w = q*st+s-pad} dY[n,p,q,k] * W[k,r,s,c]
 *   wgrad: dW[k,r,s,c] = sum_{n,p,q} dY[n,p,q,k] * X[n, p*st+r-pad, q*st+s-pad, c]
 *   gemm : C [m,n]     = sum_k A[m,k] * B[k,n]
 *
 * Layouts: activations NHWC, weights KRSC, all row-major, operands int32 (holding the
 * fixed-point codes), results int64.  Out-of-range X reads are zero.  Loops run in the
 * order of the definitions; the only parallelism is an OpenMP split over independent outputs.
 */
#include <stdint.h>
#include <string.h>

typedef struct { int n, h, w, c, k, r, s, stride, pad; } conv_shape;

static int out_dim(int in, int pad, int f, int stride) { return (in + 2 * pad - f) / stride + 1; }

void oracle_gemm(int M, int N, int K, const int32_t *A, const int32_t *B, int64_t *C)
{
#pragma omp parallel for
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k)
                acc += (int64_t)A[(size_t)m * K + k] * (int64_t)B[(size_t)k * N + n];
            C[(size_t)m * N + n] = acc;
        }
}

void oracle_conv_fwd(conv_shape d, const int32_t *X, const int32_t *W, int64_t *Y)
{
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
#pragma omp parallel for collapse(2)
    for (int n = 0; n < d.n; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < d.k; ++k) {
                    int64_t acc = 0;
                    for (int r = 0; r < d.r; ++r) {
                        const int h = p * d.stride + r - d.pad;
                        if (h < 0 || h >= d.h) continue;
                        for (int s = 0; s < d.s; ++s) {
                            const int w = q * d.stride + s - d.pad;
                            if (w < 0 || w >= d.w) continue;
                            const int32_t *x = X + (((size_t)n * d.h + h) * d.w + w) * d.c;
                            const int32_t *wt = W + (((size_t)k * d.r + r) * d.s + s) * d.c;
                            for (int c = 0; c < d.c; ++c) acc += (int64_t)x[c] * (int64_t)wt[c];
                        }
                    }
                    Y[(((size_t)n * P + p) * Q + q) * d.k + k] = acc;
                }
}

void oracle_conv_dgrad(conv_shape d, const int32_t *dY, const int32_t *W, int64_t *dX)
{
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
    /* scatter form of the definition: every (n,p,q,k,r,s,c) term lands on dX[n,h,w,c] */
#pragma omp parallel for
    for (int n = 0; n < d.n; ++n) {
        memset(dX + (size_t)n * d.h * d.w * d.c, 0, sizeof(int64_t) * (size_t)d.h * d.w * d.c);
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < d.k; ++k) {
                    const int64_t g = dY[(((size_t)n * P + p) * Q + q) * d.k + k];
                    if (g == 0) continue;
                    for (int r = 0; r < d.r; ++r) {
                        const int h = p * d.stride + r - d.pad;
                        if (h < 0 || h >= d.h) continue;
                        for (int s = 0; s < d.s; ++s) {
                            const int w = q * d.stride + s - d.pad;
                            if (w < 0 || w >= d.w) continue;
                            int64_t *dx = dX + (((size_t)n * d.h + h) * d.w + w) * d.c;
                            const int32_t *wt = W + (((size_t)k * d.r + r) * d.s + s) * d.c;
                            for (int c = 0; c < d.c; ++c) dx[c] += g * (int64_t)wt[c];
                        }
                    }
                }
    }
}

void oracle_conv_wgrad(conv_shape d, const int32_t *dY, const int32_t *X, int64_t *dW)
{
    const int P = out_dim(d.h, d.pad, d.r, d.stride), Q = out_dim(d.w, d.pad, d.s, d.stride);
#pragma omp parallel for collapse(2)
    for (int k = 0; k < d.k; ++k)
        for (int r = 0; r < d.r; ++r)
            for (int s = 0; s < d.s; ++s) {
                int64_t *dw = dW + (((size_t)k * d.r + r) * d.s + s) * d.c;
                for (int c = 0; c < d.c; ++c) dw[c] = 0;
                for (int n = 0; n < d.n; ++n)
                    for (int p = 0; p < P; ++p) {
                        const int h = p * d.stride + r - d.pad;
                        if (h < 0 || h >= d.h) continue;
                        for (int q = 0; q < Q; ++q) {
                            const int w = q * d.stride + s - d.pad;
                            if (w < 0 || w >= d.w) continue;
                            const int64_t g = dY[(((size_t)n * P + p) * Q + q) * d.k + k];
                            const int32_t *x = X + (((size_t)n * d.h + h) * d.w + w) * d.c;
                            for (int c = 0; c < d.c; ++c) dw[c] += g * (int64_t)x[c];
                        }
                    }
            }
}

int oracle_abi_version(void) { return 1; }
