/* adapt_fxp.h - C ABI of the MI355X (gfx950) implementation of AdaPT's fixed-point hot path
 * (Kummer et al., "Adaptive Precision Training (AdaPT)", arXiv 2107.13490).
 *
 * The calls follow the paper's own operations:
 *   Quantize(L, <WL,FL>)             Alg. 1 (last loop), Alg. 3; format of Sec. 2.1 "Fixed-Point
 *                                    Quantization", rounding rule SR of Sec. 3.2
 *   ForwardPass / backward pass      Alg. 1, on quantized layers: integer GEMM and
 *                                    convolution forward / data-gradient / weight-gradient
 *   PushDown(L, WL, FL)              Sec. 3.3 "The PushDown Operation", Alg. 3: KL divergence
 *                                    between the binned distributions of a tensor and of its
 *                                    quantization, over candidate word lengths
 *
 * General rules (every entry point)
 *   - Every tensor pointer and every result pointer is DEVICE memory owned by the caller,
 *     16-byte aligned unless stated otherwise.  The library never frees or keeps caller
 *     memory.  Its only allocations are the context and the context's workspace.
 *   - All work is enqueued on the context's HIP stream and the call returns without
 *     synchronising.  Results are valid in stream order.  Two calls on one context must not
 *     overlap on different streams (they share the workspace).
 *   - Return value: ADAPT_OK (0) or a negative adapt_status.  Nothing is printed, no
 *     exceptions cross the boundary.  On error no kernel of that call has been launched.
 *   - Storage of a tensor in format <wl,fl>: int8_t for wl <= 8 (sign-extended codes),
 *     int16_t for 9 <= wl <= 16, int32_t for 17 <= wl <= 32 (adapt_quantize and the four
 *     contractions take those; every other entry point stops at 16).  The represented value
 *     of code q is q * 2^-fl.
 *   - Layouts: activations NHWC, filters KRSC (Cout, R, S, Cin), row-major, dense.
 */
#ifndef ADAPT_FXP_H
#define ADAPT_FXP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADAPT_OK = 0,
    ADAPT_EINVAL = -1,       /* null / misaligned pointer, size, WL, FL, bins or range out of bounds */
    ADAPT_EUNSUPPORTED = -2, /* valid request this build does not implement (WL > 16 where not stated, dilation, groups) */
    ADAPT_EBOUND = -3,       /* the reduction is too long for one block's int32 accumulators and the workspace
                                cannot hold the partial sums of the splits that would keep them in bounds */
    ADAPT_EHIP = -4,         /* HIP runtime failure (see adapt_error_string / hipGetLastError) */
    ADAPT_EWORKSPACE = -5    /* context workspace too small for this call (see adapt_workspace_bytes) */
} adapt_status;

typedef struct adapt_ctx adapt_ctx; /* opaque: stream, device, workspace */

/* Fixed-point format <WL,FL> (Sec. 2.1, Sec. 3.2): signed, wl total bits, fl fractional bits.
 * 2 <= wl <= 16 (32 where an entry point says so: Sec. 3.3 bounds precision at 32 bits),
 * 0 <= fl <= 31 (fl need not be smaller than wl). */
typedef struct { int wl, fl; } adapt_fmt;

/* Rounding.  ADAPT_SR is the paper's stochastic rounding (Sec. 3.2): round down, or up with
 * probability equal to the fractional distance, decided by 16 random bits per element.
 * ADAPT_RN_HALF_UP (round to nearest, ties up) exists for deterministic tests.
 * Random bits are counter based: element i of a tensor uses 16-bit lane (i mod 8), low half
 * first, of the Philox-4x32-10 block with key (seed lo, seed hi) and counter
 * (i/8 lo, i/8 hi, stream lo, stream hi).  The same (seed, stream) reproduces the same bits. */
typedef enum { ADAPT_RN_HALF_UP = 0, ADAPT_SR = 1 } adapt_round;
typedef struct { int mode; uint64_t seed, stream; } adapt_rng;

/* Convolution geometry: input n x h x w x c, filters k x r x s x c, output n x p x q x k with
 * p = (h + 2 pad - r)/stride + 1, q likewise.  Cross-correlation (no filter flip), zero
 * padding, dilation 1, groups 1, stride >= 1. */
typedef struct { int n, h, w, c, k, r, s, stride, pad; } adapt_conv_desc;

/* What a contraction writes.
 *  raw != 0 : the exact integer accumulator: int32_t if adapt_acc_bits(...) == 32, int64_t if 64,
 *             a 128-bit two's-complement integer (16 bytes, low 8 bytes first) if 128.
 *  raw == 0 : the accumulator converted to `fmt` (storage as for any tensor of that format):
 *             with s = fl_a + fl_b - fmt.fl,
 *               s <= 0      q = acc * 2^-s
 *               1..16       q = (acc + (R16 >> (16-s))) >> s      (R16 = 2^15 for RN_HALF_UP)
 *               s > 16      q = ((acc >> (s-16)) + R16) >> 16
 *             then q = max(q,0) if relu, then saturation to fmt.wl bits.  R16 of output element
 *             i (row-major index in the output tensor) comes from `rng` as described above. */
typedef struct { int raw; adapt_fmt fmt; adapt_rng rng; int relu; } adapt_epilogue;

/* ---- context ------------------------------------------------------------------------------ */

/* Creates a context on the current HIP device.  `hip_stream` is a hipStream_t (NULL = the
 * default stream).  `workspace_bytes` = 0 selects the default (64 MiB).  The workspace holds
 * histograms, split-K partial sums and re-laid-out filters; ADAPT_EWORKSPACE is returned by
 * a call that needs more.  Host pointers in, host pointer out. */
int adapt_create(adapt_ctx **ctx, void *hip_stream, size_t workspace_bytes);
int adapt_destroy(adapt_ctx *ctx);
int adapt_set_stream(adapt_ctx *ctx, void *hip_stream);

/* How much workspace a call takes, from the planning code the call itself runs (the boundary the
 * paper's operations need once they are library calls: Quantize, the layer contractions, PushDown,
 * PushUp and the update all stage partial results on the device).  Fill `call` and the fields that
 * call reads; the others are ignored:
 *   QUANTIZE, SGD_UPDATE, REQUANTIZE_FIT   n
 *   QUANTIZE_BATCHED                       count
 *   GEMM                                   transA, transB, M, N, K, fa, fb, lda, ldb (0 = dense)
 *   CONV_FWD                               conv, fa = format of x, fb = of w
 *   CONV_DGRAD                             conv, fa = dy, fb = w
 *   CONV_WGRAD                             conv, fa = dy, fb = x
 *   CONV_BACKWARD                          conv, fa = dy, fb = w, fc = x
 *   KLD_SEARCH                             n, wl_lo, wl_hi, bins
 *   KLD_SEARCH_BATCHED                     kld_items (HOST array; only n and bins are read), count, wl_lo, wl_hi
 *   GRADIENT_DIVERSITY                     n, count
 * Returns the workspace_bytes with which the call takes its preferred plan (all K splits, padded
 * copies of narrow layers, one batch for up to 24 searches) and returns neither ADAPT_EWORKSPACE nor
 * ADAPT_EBOUND; 0 for a query that is invalid.  With less, contractions use fewer K splits and
 * batched searches smaller batches where they can.  ctx may be NULL: the current device is asked
 * for its number of compute units, and without a device the 256 of an MI355X are assumed (planning
 * on a host without a GPU).  Host pointers; no device work. */
typedef enum {
    ADAPT_CALL_QUANTIZE = 0, ADAPT_CALL_QUANTIZE_BATCHED = 1, ADAPT_CALL_GEMM = 2, ADAPT_CALL_CONV_FWD = 3,
    ADAPT_CALL_CONV_DGRAD = 4, ADAPT_CALL_CONV_WGRAD = 5, ADAPT_CALL_CONV_BACKWARD = 6, ADAPT_CALL_KLD_SEARCH = 7,
    ADAPT_CALL_KLD_SEARCH_BATCHED = 8, ADAPT_CALL_SGD_UPDATE = 9, ADAPT_CALL_GRADIENT_DIVERSITY = 10,
    ADAPT_CALL_REQUANTIZE_FIT = 11
} adapt_call;
struct adapt_kld_item_s;
typedef struct {
    int call;
    uint64_t n;
    int count;
    int transA, transB, M, N, K, lda, ldb;
    adapt_conv_desc conv;
    adapt_fmt fa, fb, fc;
    int wl_lo, wl_hi, bins;
    const struct adapt_kld_item_s *kld_items;
} adapt_workspace_query;
size_t adapt_workspace_bytes(const adapt_ctx *ctx, const adapt_workspace_query *query);
/* Grows the context's workspace to at least `bytes` (never shrinks it).  Synchronises the stream
 * and allocates when it has to grow; call it while setting up, not inside a step. */
int adapt_reserve_workspace(adapt_ctx *ctx, size_t bytes);
const char *adapt_error_string(int status);
/* Library / ABI version (incremented on incompatible changes). */
int adapt_version(void);

/* ---- Quantize (Alg. 1 last loop; Sec. 3.2 SR; Sec. 2.1 format) ------------------------------ */

/* q[i] = quantize(x[i]) for i < n:  y = x * 2^fl, saturated to [-2^(wl-1), 2^(wl-1)-1],
 * t = floor(y * 2^16), q = min((t + R16) >> 16, 2^(wl-1)-1).  NaN gives 0, +-Inf saturate,
 * denormals are not flushed.
 *   x          device, fp32[n]
 *   q          device, int8_t[n] (wl <= 8), int16_t[n] (wl <= 16) or int32_t[n] (wl <= 32: the same rule
 *              with t held in 64 bits)
 *   nnz        device uint64_t, may be NULL: number of non-zero codes (the paper's sp^l is
 *              nnz / n, Sec. 3.4 "Inducing Sparsity")
 *   saturated  device uint64_t, may be NULL: number of elements with x*2^fl outside the range
 * n = 0 is valid (counters are set to 0).  n > 2^40 is ADAPT_EINVAL (per-block counters are
 * 32-bit); x and q must be 16-byte aligned. */
int adapt_quantize(adapt_ctx *ctx, const float *x, size_t n, adapt_fmt fmt, adapt_rng rng,
                   void *q, uint64_t *nnz, uint64_t *saturated);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it) and cannot spare the context's workspace either: adapt_quantize with its scratch (the
 * per-block counter partials, at most 16 KiB) in a 32 KiB array that is part of the library's device
 * image instead of the context's workspace.  Same arguments, results and limits as adapt_quantize
 * (n <= 2^40; ADAPT_EWORKSPACE only on a device with more than 4,000 compute units, ADAPT_EHIP if the
 * array's address could not be taken when the context was created).  It calls no allocating routine
 * and does not touch the workspace.  Every call on one GPU, from any context, shares that GPU's copy of
 * the array: calls that overlap on one GPU (two streams) race on the counters; the codes are unaffected.
 * Nothing in the array needs clearing between calls: every block writes its own partials before they
 * are summed. */
int adapt_quantize_noalloc(adapt_ctx *ctx, const float *x, size_t n, adapt_fmt fmt, adapt_rng rng,
                           void *q, uint64_t *nnz, uint64_t *saturated);

/* One launch for a whole network (the per-layer loop of Alg. 1).  `items` is a HOST array of
 * `count` descriptors (read before the call returns; the pointers inside are device
 * pointers); each tensor is quantized exactly as by adapt_quantize with the item's own format
 * and rng stream (mode and seed are shared).  nnz / saturated of item t are written to
 * counters[2t], counters[2t+1] (device, uint64_t[2*count], may be NULL).  Descriptors travel
 * as kernel arguments, 64 per launch.  Items with 17 <= wl <= 32 (int32_t codes) are taken out of the
 * shared launch and run one after the other, each with a launch of its own. */
typedef struct {
    const float *x; void *q; uint64_t n; int32_t wl, fl; uint64_t stream;
} adapt_quantize_item;
int adapt_quantize_batched(adapt_ctx *ctx, const adapt_quantize_item *items, int count,
                           int mode, uint64_t seed, uint64_t *counters);
/* The same, and the finite range of selected input tensors as a by-product of the pass that
 * reads them: for every t with bit t of range_mask set, ranges[2t], ranges[2t+1] = min and max of
 * the finite elements of item t's x (+inf, -inf if it has none); the other pairs are written as
 * (+inf, -inf).  ranges: device float[2*count] or NULL; count <= 64 when it is given.  The pair of
 * a weight tensor is what adapt_kld_precision_search_ranged takes, so that the precision search
 * needs no range pass.  (Tracking costs a few instructions per element, so it is asked for per
 * tensor: weights, not activations.) */
int adapt_quantize_batched_ranges(adapt_ctx *ctx, const adapt_quantize_item *items, int count,
                                  int mode, uint64_t seed, uint64_t *counters, float *ranges,
                                  uint64_t range_mask);

/* ---- integer contractions (ForwardPass / backward pass of Alg. 1 on quantized tensors) ---- */

/* Common to the four contractions below: operands are device arrays of int8_t (wl <= 8) or
 * int16_t codes, 16-byte aligned, read in place; the output is written per `ep` (exact
 * accumulators: int32_t if adapt_acc_bits() is 32, else int64_t; or requantized codes).  Every
 * tensor must be smaller than 4 GiB (the kernels use 32-bit byte offsets): larger ones return
 * ADAPT_EUNSUPPORTED.  Reductions too long for an int32 accumulator, and weight gradients, are
 * split over K through the context's workspace; the result is bit-identical to the unsplit sum.
 * With too little workspace for the preferred number of splits fewer are taken; ADAPT_EBOUND if
 * even the splits that the int32 accumulators of a block require (K above 65,536 with both
 * operands at most 8 bits, above 32,768 otherwise) do not fit.  Empty outputs (M or N = 0) return ADAPT_OK.
 * Convolutions with fewer than 16 input channels work on zero-padded copies of x and w that
 * they place in the workspace (when it has room; otherwise they gather element by element);
 * results, output shapes and rounding bits are those of the unpadded operands.  When one operand
 * has wl <= 8 and the other 9..16, the int8 operand is multiplied as a single limb. */

/* Word lengths 17..32 (adapt_fxp_gemm, adapt_conv_fwd, adapt_conv_dgrad, adapt_conv_wgrad; operands
 * and / or the requantized output): an operand above 16 bits is int32_t codes; the call splits it
 * into parts the narrow kernels take (17..23 bits: the signed low byte and the rest, a = a1 2^8 +
 * a0; 24..31 bits: the signed low half-word and the rest, a = a1 2^16 + a0; 32 bits: three 11-bit
 * parts a = a2 2^22 + a1 2^11 + a0 with a0, a1 in [0, 2047], a2 = a >> 22), runs the exact
 * contraction of every pair of parts (four for two operands of up to 31 bits, nine for two of 32,
 * two or three with one narrow operand) on the int8 matrix cores, adds the partial results at their
 * power-of-two weights in 128-bit integers and applies the epilogue's rule once; the result is the
 * exact contraction of the full codes, requantized as for any other.  The parts, one partial result (8 bytes per output) and the 128-bit sums (16 bytes
 * per output) live in the workspace (adapt_workspace_bytes counts them).  adapt_fxp_gemm needs
 * ldc == N and K > 0 on this path; adapt_conv_backward and the chain stop at 16 bits. */

/* 32 if K * 2^(wl_a-1) * 2^(wl_b-1) <= 2^31 - 1 (every possible sum fits int32), else 64; 128 when
 * an operand has more than 16 bits. */
int adapt_acc_bits(int64_t K, adapt_fmt a, adapt_fmt b);

/* C[M,N] = op(A)[M,K] . op(B)[K,N], exact over the integers.  Row-major with leading
 * dimensions in elements.  transA = 0: A is M x K (lda >= K); 1: A is stored K x M (lda >= M).
 * transB likewise for B (K x N, ldb >= N; or N x K, ldb >= K).  C is M x N, ldc >= N,
 * element type per `ep`.  The result has fa.fl + fb.fl fractional bits. */
int adapt_fxp_gemm(adapt_ctx *ctx, int transA, int transB, int M, int N, int K,
                   const void *A, adapt_fmt fa, int lda, const void *B, adapt_fmt fb, int ldb,
                   void *C, int ldc, adapt_epilogue ep);

/* y[n,p,q,k]  = sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c] */
int adapt_conv_fwd(adapt_ctx *ctx, adapt_conv_desc d, const void *x, adapt_fmt fx,
                   const void *w, adapt_fmt fw, void *y, adapt_epilogue ep);
/* dx[n,h,w,c] = sum over (k,r,s) and the (p,q) with h = p*stride+r-pad, w = q*stride+s-pad of
 *               dy[n,p,q,k] * w[k,r,s,c] */
int adapt_conv_dgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy,
                     const void *w, adapt_fmt fw, void *dx, adapt_epilogue ep);
/* dw[k,r,s,c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c] */
int adapt_conv_wgrad(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy,
                     const void *x, adapt_fmt fx, void *dw, adapt_epilogue ep);

/* Both gradients of one convolution layer (the backward pass of Alg. 1 for that layer): dx exactly
 * as adapt_conv_dgrad(d, dy, w) with ep_dx and dw exactly as adapt_conv_wgrad(d, dy, x) with ep_dw.
 * When both contractions take a vector path with matching tiles (all word lengths <= 8, or all
 * above 8; channel counts multiples of 16) they share one kernel launch; otherwise the two run one
 * after the other.  Arguments and limits as for the two separate calls. */
int adapt_conv_backward(adapt_ctx *ctx, adapt_conv_desc d, const void *dy, adapt_fmt fdy,
                        const void *w, adapt_fmt fw, const void *x, adapt_fmt fx,
                        void *dx, adapt_epilogue ep_dx, void *dw, adapt_epilogue ep_dw);

/* ---- PushDown: KL-divergence precision search (Sec. 3.3, Alg. 3) --------------------------- */

/* For every candidate word length WL_c = wl_lo..wl_hi with FL_c = WL_c - il (il = integer bits
 * including the sign, kept fixed so that lowering WL only drops fractional bits):
 *   Q   = histogram of the finite elements of w on a grid of power-of-two bins: width 2^e,
 *         edges at multiples of 2^e, e the smallest integer for which the range [min w, max w]
 *         spans nb <= bins bins;
 *   P_c = histogram of quantize(w, <WL_c,FL_c>) on the same bins (values outside go to the end
 *         bins); every candidate uses the same random bits R16(seed, stream, i);
 *   KL_c = sum_b P_c(b) log2(P_c(b) / Q(b)),  P_c(b) = (count + alpha)/(n_finite + alpha nb),
 *         Q likewise.  alpha < 0 selects the default 1/nb; alpha = 0 is the unsmoothed
 *         definition (0 log 0 = 0, +inf where P > 0 = Q).
 * Selection: the smallest WL_c with KL_c < eps, wl_hi if there is none.
 * If w has no finite element or min == max: every KL_c = 0 and wl_lo is selected.
 *   w        device fp32[n]
 *   kld      device double[wl_hi - wl_lo + 1]
 *   sel      device int32_t[2]: selected WL, FL
 *   hist     device uint32_t[(wl_hi - wl_lo + 2) * bins] or NULL: row 0 = counts of Q, row
 *            1 + c = counts of P_c; entries nb..bins-1 of every row are zero
 *   grid     device int64_t[3] or NULL: e, floor(min w / 2^e), nb  (0,0,0 in the degenerate case)
 * Limits: 2 <= wl_lo <= wl_hi <= 32 (above 16 the scaled value is held in 64 bits), 1 <= il, wl_lo - il >= 0, wl_hi - il <= 31,
 * 2 <= bins <= 65536. */
int adapt_kld_precision_search(adapt_ctx *ctx, const float *w, size_t n, int wl_lo, int wl_hi,
                               int il, int bins, double eps, double alpha, adapt_rng rng,
                               double *kld, int32_t *sel, uint32_t *hist, int64_t *grid);

/* The same search with the range already known: `range` = device float[2], (min, max) of the
 * finite elements of w, e.g. as written by adapt_sgd_update_quantize; the range pass over w is
 * skipped.  Elements outside a range that does not bound the tensor are counted in the end
 * bins. */
int adapt_kld_precision_search_ranged(adapt_ctx *ctx, const float *w, size_t n, const float *range,
                                      int wl_lo, int wl_hi, int il, int bins, double eps,
                                      double alpha, adapt_rng rng, double *kld, int32_t *sel,
                                      uint32_t *hist, int64_t *grid);

/* One call for all layers of a network (the loop of Alg. 2 over l in L): the same search on
 * `count` tensors described by a HOST array (read before the call returns; `w` inside is a
 * device pointer); tensor t writes kld[t*ncand ...] and
 * sel[2t], sel[2t+1], with ncand = wl_hi - wl_lo + 1.  il, bins and the rng stream are per
 * tensor; candidate range, eps, alpha, mode and seed are shared. */
typedef struct adapt_kld_item_s {
    const float *w; uint64_t n; int32_t il, bins; uint64_t stream;
} adapt_kld_item;
int adapt_kld_precision_search_batched(adapt_ctx *ctx, const adapt_kld_item *items, int count,
                                       int wl_lo, int wl_hi, double eps, double alpha, int mode,
                                       uint64_t seed, double *kld, int32_t *sel);

/* The batched search with ranges already known (e.g. from adapt_quantize_batched_ranges or
 * adapt_sgd_update_quantize): ranges = HOST array of `count` device pointers, ranges[t] = device
 * float[2] (min, max) of the finite elements of tensor t, or NULL for a tensor whose range the call
 * computes itself.  When every entry is set the range pass over the tensors is skipped.  Elements
 * outside a range that does not bound its tensor are counted in the end bins. */
int adapt_kld_precision_search_batched_ranged(adapt_ctx *ctx, const adapt_kld_item *items,
                                              const float *const *ranges, int count, int wl_lo,
                                              int wl_hi, double eps, double alpha, int mode,
                                              uint64_t seed, double *kld, int32_t *sel);

/* ---- master-weight update fused with re-quantization (Alg. 1: the backward-pass line and the
 *      Quantize loop after it) ------------------------------------------------------------- */

/* Plain SGD on the fp32 master copy with the quantized gradient of the layer, then Quantize:
 *   step = fp32(lr / sqrt(*g_sumsq))  (the gradient divided by its 2-norm, Sec. 3.3 "Dealing with
 *          Fixed-Points Limited Range"; 0 if the sum is 0), or fp32(lr * 2^-fg.fl) if g_sumsq is
 *          NULL (no normalisation)
 *   d  = fma(l2, w, l1 * sign(w))     (derivatives of the L1 / L2 terms of Sec. 3.4; sign(0) = 0)
 *   w1 = fma(-step, c, w)             (c = the gradient code)
 *   w' = fma(-lr, d, w1)              (lr, l1, l2 rounded to fp32 once; three fp32 fused
 *                                      multiply-adds in exactly this order)
 *   q  = quantize(w', fq) as adapt_quantize does, with `rng`
 *   w         device fp32[n], updated in place
 *   g         device codes of the gradient, int8_t[n] (fg.wl <= 8), int16_t[n] (<= 16) or int32_t[n]
 *             (<= 32; converted to fp32 with round-to-nearest-even)
 *   g_sumsq   device or NULL: sum of the squared codes of g (adapt_gradient_diversity writes it as
 *             sums[k], adapt_requantize_fit as sumsq): one uint64_t for fg.wl <= 16, uint64_t[2] (low
 *             word first) for fg.wl > 16, whose nearest double enters the quotient
 *   q         device int8_t[n] (fq.wl <= 8), int16_t[n] (<= 16) or int32_t[n] (<= 32)
 *   counters  device uint64_t[2] or NULL: non-zero codes, saturated elements
 *   range     device float[2] or NULL: min and max of the finite w' (+inf, -inf if there is none)
 * Pointers 16-byte aligned; n <= 2^40. */
typedef struct { double lr, l1, l2; } adapt_sgd_params;
int adapt_sgd_update_quantize(adapt_ctx *ctx, float *w, size_t n, const void *g, adapt_fmt fg,
                              const uint64_t *g_sumsq, adapt_sgd_params opt, adapt_fmt fq,
                              adapt_rng rng, void *q, uint64_t *counters, float *range);

/* ---- PushUp (Sec. 3.3 "The PushUp Operation") ---------------------------------------------- */

/* Gradient diversity of one layer over a lookback window of `count` gradient tensors of n
 * elements each, tensor k held as fixed-point codes g_k = c_k * 2^-fl_k (int8_t for wl <= 8,
 * else int16_t, as written by the contractions' requantizing epilogue):
 *   ds = sum_k ||g_k||_2 / || sum_k g_k ||_2
 * All sums of codes and of squares are exact integers (the codes are aligned to the finest grid
 * of the window before they are added); the norms and the ratio are fp64.
 *   items  HOST array of `count` descriptors, oldest first (read before the call returns; `g`
 *          inside is a device pointer, 16-byte aligned)
 *   sums   device uint64_t[count + 2] or NULL: sum_i c_k[i]^2 for k < count, then the sums of
 *          the low and of the high 32-bit halves of (sum_k c_k[i] * 2^(fl_max - fl_k))^2, so
 *          that the squared norm of the sum is (sums[count+1] * 2^32 + sums[count]) * 4^-fl_max
 *   out    device double[2]: ds (+inf if only the denominator is 0, NaN if both are), and
 *          log ds (natural) when 0 < ds < inf, else 1 (the paper's "otherwise" case)
 * Limits: 1 <= count <= 64, n <= 2^30, and sum_k 2^(wl_k - 1 + fl_max - fl_k) < 2^31 (the element
 * sum is kept in 32 bits); ADAPT_EUNSUPPORTED beyond them.  n = 0 gives NaN and 1.
 * A window with a word length above 16 (int32_t codes for those tensors): the element sum is kept in
 * 64 bits, the limit is sum_k 2^(wl_k - 1 + fl_max - fl_k) < 2^48, and every sum takes 128 bits:
 * sums is then uint64_t[2 (count + 1)], pairs of words, low first: sum_i c_k[i]^2 for k < count, then
 * the sum of the squared aligned element sums. */
typedef struct { const void *g; int32_t wl, fl; } adapt_grad_item;
int adapt_gradient_diversity(adapt_ctx *ctx, const adapt_grad_item *items, int count, size_t n,
                             uint64_t *sums, double *out);

/* The scalar rules of the switch controller.  Host functions: no device, no context.
 * Strategy st of the suggestion rule. */
enum { ADAPT_ST_MIN = 0, ADAPT_ST_MEAN = 1, ADAPT_ST_MAX = 2 };
typedef struct { int wl, fl, s1, s2, s; } adapt_pushup_result;
/* New <WL,FL> of a layer from its diversity `ds` and the PushDown result <wl_min, fl_min>.
 * With L = log ds (natural) if 0 < ds < inf, else 1:
 *   L > 0:  s1 = max(ceil(1/(L - 1)), 1)  (L = 1: wl_cap),  s2 = max(min(32 L^2 - 1, 32) - fl_min, 1)
 *           rounded up, both at most wl_cap;  s = min | ceil(mean) | max of (s1, s2) by `strategy`
 *   else    s = 1
 *   FL = min(fl_min + s, wl_cap), WL = min(max(wl_min, fl_min) + 1, wl_cap), then the buffer bits of
 *   "Dealing with Fixed-Points Limited Range": FL = min(FL, wl_cap - buff),
 *   WL = max(min(FL + buff, wl_cap), WL).  wl_cap is the paper's 32 or the widest length the
 *   caller's kernels take.  ADAPT_EINVAL for arguments out of range. */
int adapt_pushup_suggest(double ds, int wl_min, int fl_min, int strategy, int buff, int wl_cap,
                         adapt_pushup_result *res);
/* "Strategy, Resolution and Lookback": |loss_avg| > |loss_now| gives min; otherwise min -> mean,
 * mean -> max, max stays.  Returns the new strategy. */
int adapt_strategy_next(int strategy, double loss_avg, double loss_now);
/* lb_new = min(max(ceil(lb_upr / ds), lb_lwr), lb_upr) if 0 < ds < inf, else lb_upr; returns
 * ceil(lb_new * gamma + (1 - gamma) * lb). */
int adapt_lookback_next(int lb, double ds, int lb_lwr, int lb_upr, double gamma);
/* r + 1 if lb == lb_upr, r - 1 if lb == lb_lwr (first case wins when both hold), clamped to
 * [r_lwr, r_upr]; r unchanged otherwise. */
int adapt_resolution_next(int r, int lb, int lb_lwr, int lb_upr, int r_lwr, int r_upr);

/* ---- a chained training step (Alg. 1 for one batch) and its element-wise integer operations ---- */

/* The paper states the loop (ForwardPass, backward pass, update, Quantize per layer) and leaves
 * the integer form of ReLU / pooling and the range of fixed-point gradients open; the rules of
 * this library are stated with each call. */

/* 2x2 max-pooling, stride 2, of codes: a[n,i,j,c] = max of y[n,2i..2i+1,2j..2j+1,c] (the code order
 * is the value order).  y: device codes of an n x h x w x c tensor stored as format f (only the
 * storage width of f matters: int8_t, int16_t, or int32_t for 17 <= f.wl <= 32), h and w even; a:
 * device, n x h/2 x w/2 x c, same storage. */
int adapt_maxpool2_fwd(adapt_ctx *ctx, const void *y, adapt_fmt f, int n, int h, int w, int c, void *a);

/* Gradient with respect to a contraction's output from the gradient with respect to the layer's
 * output.  y = the stored layer output before pooling (requantized, after ReLU), n x h x w x c.
 *   pool != 0: da is n x h/2 x w/2 x c; each element goes to the FIRST maximum of its window of y
 *              in the order (0,0),(0,1),(1,0),(1,1); the other three positions get 0
 *   pool == 0: da is n x h x w x c and dy = da
 *   relu != 0: additionally dy = 0 where y <= 0 (the stored output decides the mask)
 * da, y and dy share the storage width of f (f.wl up to 32).  dy must not overlap da or y. */
int adapt_relu_pool_bwd(adapt_ctx *ctx, const void *da, const void *y, adapt_fmt f, int n, int h,
                        int w, int c, int relu, int pool, void *dy);

/* Exact accumulators -> wl-bit codes that keep the leading bits.  Back-propagation is linear in
 * the incoming gradient and the weight update divides a layer's gradient by its 2-norm (Sec. 3.3
 * "Dealing with Fixed-Points Limited Range"), so a gradient tensor may be stored with any
 * power-of-two factor:
 *   shift = max(0, bit_length(max_i |acc[i]|) - (wl - 1))
 *   q[i]  = the contraction epilogue's rule with this shift (SR on the dropped bits, saturation)
 *   acc       device int32_t[n] (acc_bits = 32), int64_t[n] (acc_bits = 64) or 128-bit integers as
 *             pairs of int64_t, low word first (acc_bits = 128: the exact output of a contraction
 *             with an operand above 16 bits)
 *   q         device int8_t[n] (wl <= 8), int16_t[n] (wl <= 16) or int32_t[n] (wl <= 32)
 *   shift     device int32_t or NULL
 *   sumsq     device or NULL: sum of q[i]^2 (what adapt_sgd_update_quantize takes): one uint64_t for
 *             wl <= 16; for wl > 16 the sum may pass 64 bits and is written as uint64_t[2], low word
 *             first
 * Two passes over acc.  n <= 2^40; n = 0 writes shift = 0, sumsq = 0. */
int adapt_requantize_fit(adapt_ctx *ctx, const void *acc, int acc_bits, size_t n, int wl,
                         adapt_rng rng, void *q, int32_t *shift, uint64_t *sumsq);

/* Residual addition of two fixed-point tensors: out = a + b in format fo, i.e. the exact sum with
 * max(fa.fl, fb.fl) fractional bits, then the contraction epilogue's rule with
 * s = max(fa.fl, fb.fl) - fo.fl (SR or round-to-nearest, optional ReLU, saturation).  n <= 2^40.
 * Word lengths up to 32 (int32_t codes above 16 bits; the sum is then formed in 128 bits). */
int adapt_residual_add(adapt_ctx *ctx, const void *a, adapt_fmt fa, const void *b, adapt_fmt fb,
                       size_t n, adapt_fmt fo, adapt_rng rng, int relu, void *out);

/* ---- batch normalisation, global average pooling and gradient merging on fixed-point codes ----
 * The paper trains residual networks with batch normalisation (Sec. 4.1) and does not say how these
 * steps are carried out on codes; the rules below are this library's.  Tensors are NHWC, so the
 * `channels` codes of one position are contiguous ("a row"); channels % 8 == 0, channels <= 4096,
 * rows <= 2^23.  Word lengths go up to 32 in all of these calls (int32_t codes above 16 bits): a call
 * with such a tensor runs the same rules in 128-bit integers (S2 and D2 reach 85 bits, and enter the
 * fp64 formulas as their nearest doubles), one element per thread; it is exact and far from the speed
 * of the calls on int8 / int16 codes.
 *
 * adapt_bn_forward (training mode: statistics of the batch).  Per channel k over the `rows` codes of
 * y (format fy): S1 = sum y, S2 = sum y^2 (exact); in fp64, one rounded operation at a time:
 *   mean = S1/rows, var = max(S2/rows - mean*mean, 0), sig = sqrt(var + eps 4^fy.fl),
 *   alpha = gamma 2^fo.fl / sig, off = beta 2^fo.fl - mean alpha;
 *   FA = clamp(30 - E, 0, 30) where max_k |alpha_k| = f 2^E, 1/2 <= f < 1 (30 if that maximum is 0);
 *   A_k = rint(alpha_k 2^FA) clamped to +-2^30, B_k = rint(off_k 2^FA) clamped to +-2^61;
 *   out = requantize(A_k y + B_k + res 2^(fo.fl + FA - fres.fl), FA) in format fo (the epilogue rule of
 *   the contractions: SR or nearest, optional ReLU, saturation; a negative exponent of the shortcut is
 *   an arithmetic right shift).  res = NULL: no shortcut.
 * gamma, beta: device float[channels] (finite).  state: device, 64-byte aligned,
 * adapt_bn_state_bytes(channels) bytes, written here and read by adapt_bn_backward; layout: a 64-byte
 * header (int32 channels, fl_y, fl_o, FA, FB, 3 reserved; uint64 rows), then mean[K], sig[K], alpha[K]
 * (double), B[K], R[K] (int64), A[K], P[K], Q[K] (int32).  Four launches. */
size_t adapt_bn_state_bytes(int channels);
int adapt_bn_forward(adapt_ctx *ctx, const void *y, adapt_fmt fy, size_t rows, int channels,
                     const float *gamma, const float *beta, double eps, const void *res,
                     adapt_fmt fres, adapt_fmt fo, adapt_rng rng, int relu, void *out, void *state);

/* Backward of the same normalisation from dz, the wl_dz-bit codes of the gradient at its output (any
 * power-of-two scale 2^-e).  D1 = sum dz, D2 = sum dz y (exact);
 *   dgamma = (D2 - mean D1)/sig, dbeta = D1 (device double[channels], in units of 2^-e);
 *   c1 = D1/rows, c2 = dgamma/(rows sig); P = alpha, Q = -(alpha c2), R = alpha (mean c2 - c1);
 *   FB from max(|P|,|Q|) as FA above; codes P^, Q^ (+-2^30), R^ (+-2^61) = rint(. 2^FB);
 *   dy = requantize_fit(P^ dz + Q^ y + R^) in wl_out bits (the rule of adapt_requantize_fit).
 * The gradient with respect to y's values is dy 2^-(e + FB - shift + fo.fl - fy.fl).  shift: device
 * int32 or NULL; e_in / e_out: device int64 or NULL, *e_out = *e_in + FB - shift + fo.fl - fy.fl
 * (e_in = NULL counts as 0).  y, fy, rows, channels as in the forward call.  Five launches. */
int adapt_bn_backward(adapt_ctx *ctx, const void *dz, int wl_dz, const void *y, adapt_fmt fy,
                      size_t rows, int channels, void *state, int wl_out, adapt_rng rng, void *dy,
                      double *dgamma, double *dbeta, int32_t *shift, const int64_t *e_in,
                      int64_t *e_out);

/* gamma[k] = fma(-lr, (float)(dgamma[k] / |dgamma|_2), gamma[k]) and the same for beta, fp32; the
 * norms are summed in channel order in fp64; a zero or non-finite norm leaves that vector alone. */
int adapt_bn_update(adapt_ctx *ctx, float *gamma, float *beta, const double *dgamma,
                    const double *dbeta, int channels, double lr);

/* Global average pooling of an n x hw x c tensor of codes (hw a power of two, c % 8 == 0):
 * out[n, c] = requantize(sum over the hw positions, log2 hw), same format.  Backward: da[n, p, c] =
 * dout[n, c] for every position p; the caller adds log2 hw to the gradient's exponent. */
int adapt_gap_fwd(adapt_ctx *ctx, const void *a, adapt_fmt f, int n, int hw, int c, adapt_rng rng,
                  void *out);
int adapt_gap_bwd(adapt_ctx *ctx, const void *dout, int wl, int n, int hw, int c, void *da);

/* Sum of two gradient tensors a 2^-e_a + b 2^-e_b (codes of wl_a / wl_b bits, exponents in device
 * memory; NULL counts as 0) as wl_out-bit codes: the exact sum on the grid of max(e_a, e_b), then the
 * rule of adapt_requantize_fit; *e_out = max(e_a, e_b) - shift.  If the exponents differ by more than
 * 40, the tensor with the larger exponent (far smaller values) is left out.  b = NULL: a alone is
 * refitted to wl_out bits.  out may be a or b.  Two launches. */
int adapt_grad_add(adapt_ctx *ctx, const void *a, int wl_a, const int64_t *e_a, const void *b,
                   int wl_b, const int64_t *e_b, size_t n, int wl_out, adapt_rng rng, void *out,
                   int32_t *shift, int64_t *e_out);

/* A feed-forward chain of convolution / fully connected layers (FC: h = w = r = s = 1, pad 0, c =
 * the flattened NHWC input), each optionally followed by ReLU (fused into the contraction's
 * epilogue) and then by 2x2/2 max-pooling.  All layers share the batch size conv.n, and the
 * output of layer l has as many elements per sample as layer l+1 reads. */
typedef struct { adapt_conv_desc conv; int relu, pool; } adapt_layer_desc;
typedef struct adapt_net adapt_net; /* opaque, host */

/* Per-layer record the step keeps in the workspace (device memory). */
typedef struct {
    uint64_t g_sumsq;            /* sum of the squared weight-gradient codes */
    uint64_t g_sumsq_hi;         /* its bits above 64: written only for gradient codes above 16 bits */
    uint64_t nnz, saturated;     /* of the re-quantized weights (adapt_net_update) */
    float range_lo, range_hi;    /* finite range of the updated master weights */
    int32_t shift_w, shift_a;    /* shifts chosen for the weight gradient / the data gradient handed down */
    int32_t reserved[4];
} adapt_net_stats;

enum { ADAPT_NT_INPUT = 0,   /* quantized network input (layer ignored) */
       ADAPT_NT_Y = 1,       /* layer output before pooling */
       ADAPT_NT_A = 2,       /* layer output (after pooling); the last layer's are the logits */
       ADAPT_NT_DY = 3,      /* gradient w.r.t. the contraction output */
       ADAPT_NT_DA = 4,      /* gradient w.r.t. the layer output (not written for the last layer) */
       ADAPT_NT_QW = 5,      /* weight codes */
       ADAPT_NT_G = 6,       /* weight-gradient codes */
       ADAPT_NT_STATS = 7,   /* adapt_net_stats */
       ADAPT_NT_YC = 8,      /* batch-norm layers: the convolution output that is normalised */
       ADAPT_NT_DYC = 9,     /* gradient w.r.t. the convolution output (= NT_DY without batch norm) */
       ADAPT_NT_BN = 10,     /* batch-norm layers: the state of adapt_bn_forward (bytes) */
       ADAPT_NT_EXP = 11,    /* int64[4]: exponents of the gradient codes of the last backward pass: of NT_DA
                              * (for the last layer: dlogits_fl), of NT_DYC after batch norm, of NT_G, one spare */
       ADAPT_NT_DGAMMA = 12, /* batch-norm layers: double[k], gradient of gamma in units of 2^-e(NT_DA) */
       ADAPT_NT_DBETA = 13 };

/* Hyper-parameters of the precision switch (Sec. 3.3 "Strategy, Resolution and Lookback"): bounds and
 * start values of the lookback lb^l and the resolution r^l (the number of bins of the KL search),
 * the lookback momentum gamma, the KL threshold eps, the buffer bits, the candidate word lengths
 * of PushDown and the start strategy (ADAPT_ST_*).  1 <= lb_lwr <= lb_init <= lb_upr <= 64,
 * 2 <= r_lwr <= r_init <= r_upr <= 65536, 0 <= gamma <= 1, eps >= 0, 1 <= buff <= 15,
 * 2 <= wl_lo <= wl_hi <= 16. */
typedef struct {
    int lb_lwr, lb_upr, lb_init;
    int r_lwr, r_upr, r_init;
    double gamma, eps;
    int buff, wl_lo, wl_hi, strategy_init;
} adapt_switch_params;

/* A network as a graph of layers (the residual networks of Sec. 4.1): layer l is a convolution of
 * the output of layer `src` (-1: the layer before, or the network input for layer 0), optionally
 * followed by batch normalisation (bn; with it the ReLU comes after the normalisation and `res` >= 0
 * adds the output of layer `res` inside it: adapt_bn_forward), then ReLU, then 2x2 max-pooling (pool)
 * or global average pooling (gap: adapt_gap_fwd).  src, res < l; every layer but the last needs a
 * consumer, at most four.  Backward, a layer's output gradient is the sum of what its consumers hand
 * back: the first contribution is stored (a convolution's data gradient as the fitting pass wrote
 * it; a shortcut's gradient refitted with adapt_grad_add alone), later ones are added with
 * adapt_grad_add; exponents stay in device memory
 * (ADAPT_NT_EXP).  Random streams of the additional steps: rng.stream + 2^20 + 8 l + slot with slot
 * 0 = batch-norm output, 1 = batch-norm data gradient, 2 = average pooling, 3 + k = the k-th contribution
 * to the gradient of layer l's output. */
typedef struct { adapt_conv_desc conv; int relu, pool, bn, src, res, gap; } adapt_node_desc;
size_t adapt_graph_workspace_bytes(const adapt_node_desc *nodes, int count, int lb_upr);
/* As adapt_net_create.  gammas, betas: HOST arrays of `count` device float[k] pointers (read for the
 * layers with bn; the arrays may be NULL when no layer has it), owned by the caller and updated in
 * place by adapt_net_update (adapt_bn_update with the step's learning rate).  bn_eps >= 0. */
int adapt_graph_create(adapt_ctx *ctx, const adapt_node_desc *nodes, int count, float *const *weights,
                       float *const *gammas, float *const *betas, double bn_eps,
                       const adapt_switch_params *sp, void *workspace, size_t workspace_bytes,
                       adapt_net **out);

/* Bytes of device workspace the chain needs (activations, gradients, codes of weights and
 * gradients at int16 storage so that word lengths may change, two accumulator buffers, and
 * lb_upr + 1 gradient tensors per layer for the lookback windows, into one of which the backward
 * pass writes; lb_upr = 0 without precision switching);
 * 0 if the description is invalid (count outside 1..64, unequal batch sizes, shapes that do not
 * chain, pooling of an odd-sized map, lb_upr outside 0..64). */
size_t adapt_net_workspace_bytes(const adapt_layer_desc *layers, int count, int lb_upr);

/* layers, weights: HOST arrays of `count` entries; weights[l] = device fp32 master weights of layer
 * l (KRSC), owned by the caller and updated in place by adapt_net_update.  sp: HOST, or NULL for a
 * chain without adapt_net_precision_switch.  workspace: device, 256-byte aligned, owned by the
 * caller, must outlive the net.  Formats start as <8,4>. */
int adapt_net_create(adapt_ctx *ctx, const adapt_layer_desc *layers, int count,
                     float *const *weights, const adapt_switch_params *sp, void *workspace,
                     size_t workspace_bytes, adapt_net **net);
/* The same chain or graph laid out for word lengths up to wl_max (16 or 32; for callers that cannot tell in advance how far
 * PushUp will go, Sec. 3.3 caps it at 32): with 32 every code buffer holds int32_t storage and the accumulator
 * buffers 128-bit integers, adapt_net_set_format and the switch parameters' wl_hi may go up to 32, PushUp's cap is
 * 32, tensors of layers above 16 bits are int32_t (adapt_net_tensor reports 4-byte elements), the loss gradient
 * handed to adapt_net_backward is int32_t when the last layer has more than 16 bits, and adapt_net_stats holds the
 * 128-bit sum of squares in g_sumsq / g_sumsq_hi.  A window whose gradients have more than 16 bits follows
 * adapt_gradient_diversity's rule for such windows (bound 2^48).  Contractions with an operand above 16 bits are
 * composed of narrower parts (see adapt_acc_bits): correct, and several times slower than the native ones. */
size_t adapt_net_workspace_bytes_wide(const adapt_layer_desc *layers, int count, int lb_upr, int wl_max);
size_t adapt_graph_workspace_bytes_wide(const adapt_node_desc *nodes, int count, int lb_upr, int wl_max);
int adapt_graph_create_wide(adapt_ctx *ctx, const adapt_node_desc *nodes, int count, float *const *weights,
                            float *const *gammas, float *const *betas, double bn_eps,
                            const adapt_switch_params *sp, int wl_max, void *workspace,
                            size_t workspace_bytes, adapt_net **out);
int adapt_net_create_wide(adapt_ctx *ctx, const adapt_layer_desc *layers, int count,
                          float *const *weights, const adapt_switch_params *sp, int wl_max,
                          void *workspace, size_t workspace_bytes, adapt_net **out);
int adapt_net_destroy(adapt_net *net);
/* <WL,FL> of layer l: its weights, its output activations, and (WL only) its gradients. */
int adapt_net_set_format(adapt_net *net, int layer, adapt_fmt f);
/* Where a tensor of the chain lives: byte offset into the workspace, element count, bytes per
 * element (for reading results; host pointers out). */
int adapt_net_tensor(const adapt_net *net, int layer, int which, size_t *offset, size_t *count,
                     int *elem_bytes);

/* Random streams: every call takes (mode, seed, stream0); layer l uses stream0 + 8 l + slot with
 * slot 0 = forward output, 1 = data gradient handed down, 2 = weight gradient, 3 = re-quantized
 * weights, 4 = network input (l = 0), 5 = first quantization of the weights, 6 = PushDown.
 * A call that fails returns the failing step's status; steps enqueued before it have run. */

/* Quantize of every layer's master weights into its format (one launch). */
int adapt_net_quantize_weights(adapt_net *net, adapt_rng rng);
/* x: device fp32, the batch in NHWC.  a_{-1} = quantize(x, format of layer 0); per layer
 * y = requantize(ReLU(conv(a, W^))) into the layer's format, a = maxpool(y). */
int adapt_net_forward(adapt_net *net, const float *x, adapt_rng rng);
/* dlogits: device codes (storage of the last layer's format, its word length) of the loss gradient
 * with respect to the last layer's output, dlogits_fl = their fractional bits (any scale works
 * for the update; the precision switch compares gradients of several batches, so keep it
 * consistent).  Per layer, last to first: dy = adapt_relu_pool_bwd(da, y); exact
 * dW = wgrad(dy, a_prev) and, above the first layer, exact da_prev = dgrad(dy, W^); both through
 * adapt_requantize_fit (dW to the layer's word length, da_prev to the previous layer's).  Needs a
 * forward pass since the last format change or update. */
int adapt_net_backward(adapt_net *net, const void *dlogits, int dlogits_fl, adapt_rng rng);

/* PrecisionSwitch (Alg. 2), between the backward pass and the update.  `loss` is this batch's loss.
 *   strategy   adapt_strategy_next(strategy, mean of the last ceil(mean_l lb^l) earlier losses, loss);
 *              unchanged on the first call
 *   per layer  the weight-gradient codes join the layer's window (at most lb_upr entries, oldest
 *              dropped) with the exponent that follows from the fitting shifts (kept in device memory,
 *              ADAPT_NT_EXP; on a plain chain:
 *                e(dy_last) = dlogits_fl, e(g_l) = e(dy_l) + FL(a_{l-1}) - shift_w(l),
 *                e(dy_{l-1}) = e(dy_l) + FL(W^_l) - shift_a(l));
 *              ds = adapt_gradient_diversity of the most recent min(len, lb^l) entries with
 *              fl_k = e_k - min e.  The aligned sum of the window is kept in 32-bit integers: while
 *              sum_k 2^(wl_k - 1 + max e - e_k) reaches 2^31 the oldest of these entries is left out
 *              (the newest always stays); `used` reports how many entered;
 *              lb^l = adapt_lookback_next, r^l = adapt_resolution_next;
 *              if len >= lb^l: PushDown = the KL search (batched over the layers that switch; it takes the
 *              range of the weights from the last adapt_net_update, so master weights that the caller
 *              rewrites must be followed by adapt_net_quantize_weights) on the master weights with
 *              il = WL - FL, candidates max(wl_lo, il)..wl_hi, r^l bins, stream slot 6, its
 *              selection limited to the current WL; PushUp = adapt_pushup_suggest with wl_cap 16;
 *              the layer takes the new format and its window is emptied.
 * The call synchronises the stream once for the diversities and, when a layer switches, once more
 * for the selections.  A call that returns an error has changed nothing (strategy, loss history,
 * windows, lookbacks, resolutions and formats are as before) and may be repeated; a second call
 * after the same backward pass is ADAPT_EINVAL.  The update
 * that follows quantizes the weights in the new formats; a forward pass is needed before the next
 * backward pass.  report: HOST array of `count` entries or NULL; strategy: HOST or NULL. */
typedef struct {
    double ds;
    int32_t wl, fl, lb, res, switched, wl_min, fl_min, used;
} adapt_switch_report;
int adapt_net_precision_switch(adapt_net *net, double loss, adapt_rng rng,
                               adapt_switch_report *report, int *strategy);
/* Per layer adapt_sgd_update_quantize with the gradient codes and their sum of squares (the step
 * has length lr per layer) and rng stream rng.stream + 8 l + 3; writes the new weight codes and the
 * stats record; gamma and beta of the layers with batch normalisation as adapt_bn_update does.
 * The results are those of the per-layer calls bit for bit, enqueued as one launch for all gamma /
 * beta and one launch pair for the weights of all layers with codes of at most 16 bits (per-layer
 * launches for the others).  ADAPT_EINVAL, with nothing enqueued, before the first backward pass;
 * ADAPT_EWORKSPACE when the context's workspace cannot hold the batch's per-block partials (the
 * same 16 KiB per layer on a 256-CU device that adapt_net_quantize_weights takes). */
int adapt_net_update(adapt_net *net, adapt_sgd_params opt, adapt_rng rng);

/* ---- the paper's performance model (Sec. 4.1 "Performance Model") --------------------------- */

/* One layer at one training step: ops = multiply-adds of a forward pass, sp = fraction of
 * non-zero weights (nnz / numel as adapt_quantize reports it), wl = its word length, numel = its
 * number of weights, lookback and resolution as the switch controller holds them.  Host functions;
 * NaN for arguments out of range. */
typedef struct { double ops, sp, numel; int wl, lookback, resolution; } adapt_perf_layer;
/* Bound on the operations of one PushDown: 2 log2(32 - 8) r 3 numel. */
double adapt_perf_pushdown_ops(int resolution, double numel);
/* Bound on the operations of one PushUp: (lb + 1) numel + 1. */
double adapt_perf_pushup_ops(int lookback, double numel);
/* One step's term of the training-cost bound: sum_l ops_l (sp_l WL_l + 32 / accs) (quantized
 * sparse forward pass, 32-bit dense backward pass, accs gradient-accumulation steps). */
double adapt_perf_step_cost(const adapt_perf_layer *layers, int count, int accs);
/* One step's term of the overhead bound: sum_l 32 (sp_l pd_l + pu_l) / (accs lb_l). */
double adapt_perf_step_overhead(const adapt_perf_layer *layers, int count, int accs);
/* sz = sum_l sp_l WL_l (taken at the last step), and one step's term of mem = mean over steps of
 * sum_l (sp_l WL_l + 32). */
double adapt_perf_model_size(const adapt_perf_layer *layers, int count);
double adapt_perf_step_memory(const adapt_perf_layer *layers, int count);
/* SU = bs_other costs_other / (bs_ours costs_ours). */
double adapt_perf_speedup(double bs_other, double costs_other, double bs_ours, double costs_ours);

#ifdef __cplusplus
}
#endif
#endif /* ADAPT_FXP_H */
