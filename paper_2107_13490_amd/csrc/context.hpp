// Library context: stream, device facts and the single workspace allocation.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "adapt_fxp.h"

// Where a contraction with an exact output leaves the largest magnitude of each of its blocks' outputs, for the
// fitting requantization that follows it in the chained step (which then needs no pass of its own over the
// accumulators).  Armed by the chained step around a contraction call (part != null), filled in by the launch.
struct adapt_amax_sink {
    unsigned long long *part;      // device: room for `capacity` maxima
    unsigned long long *zero;      // device word the producing launch clears (the sum the fitting pass adds to), or null
    int capacity;
    int count;                     // maxima the last launch stored; 0: none (not armed, nothing launched), -1: more than fit
};

struct adapt_ctx {
    hipStream_t stream;
    int device;
    int num_cu;
    // Device workspace.  The first kCtlBytes hold small control words (tickets of the
    // "last block finishes" reductions; zero at creation and re-zeroed by whoever uses them),
    // the rest is scratch for the call in flight.
    char *ws;
    size_t ws_bytes;
    hipError_t last_hip_error;
    // kernels whose dynamic LDS limit this context has already raised above the 64 KiB default
    std::vector<const void *> big_lds_kernels;
    // this device's copy of the static scratch array of adapt_quantize_noalloc (null if its address could not be taken)
    void *static_scratch;
    // [0]: forward / data-gradient / GEMM contractions, [1]: weight gradients
    adapt_amax_sink amax[2];
};

namespace adapt {

constexpr size_t kCtlBytes = 4096;
constexpr size_t kStaticScratchBytes = 32 * 1024;      // static scratch of the entry point that allocates nothing
hipError_t static_scratch_address(void **ptr);         // of the current device's copy
constexpr size_t kDefaultWorkspace = (size_t)64 << 20;

}  // namespace adapt
#include <functional>
namespace adapt {
// Contraction with operands or an output of 17..32 bits, composed of exact contractions of 11-bit parts (wide.hip).
// sub(a_part, fa, b_part, fb, c, exact epilogue) runs one of them; elems_*: codes in each operand's allocation.
typedef std::function<int(const void *, adapt_fmt, const void *, adapt_fmt, void *, adapt_epilogue)> SubContraction;
int wide_contraction(adapt_ctx *ctx, const void *a, adapt_fmt fa, uint64_t elems_a, const void *b, adapt_fmt fb, uint64_t elems_b,
                     uint64_t outputs, int64_t k_total, void *out, adapt_epilogue ep, const SubContraction &sub);
size_t ws_need_wide(uint64_t elems_a, bool wide_a, uint64_t elems_b, bool wide_b, uint64_t outputs, bool raw);
// formats of the parts an operand is split into (lowest first), their weight step in bits; returns their number
int wide_parts(adapt_fmt f, adapt_fmt fmt[3], int *step);
// The fitting requantization with 128-bit accumulators or an output above 16 bits (wide_ops.hip); arguments as in
// adapt_requantize_fit, plus the exponent bookkeeping of the chained step (*e_out = (e_in ? *e_in : 0) + e_add - shift).
int requantize_fit_wide(adapt_ctx *ctx, const void *acc, int acc_bits, size_t n, int wl, adapt_rng rng, void *q, int32_t *shift,
                        uint64_t *sumsq, const long long *e_in, long long e_add, long long *e_out);

inline char *scratch(adapt_ctx *c) { return c->ws + kCtlBytes; }
inline size_t scratch_bytes(const adapt_ctx *c) { return c->ws_bytes - kCtlBytes; }
inline uint32_t *ticket(adapt_ctx *c, int slot) { return reinterpret_cast<uint32_t *>(c->ws) + slot; }

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int hip_status(adapt_ctx *c, hipError_t e)
{
    if (e == hipSuccess) return ADAPT_OK;
    c->last_hip_error = e;
    return ADAPT_EHIP;
}

// A kernel that wants more than 64 KiB of dynamic LDS needs the limit raised once before its first launch;
// the context remembers which kernels it has done that for (no process-wide state).
inline hipError_t allow_big_lds(adapt_ctx *c, const void *kernel, size_t lds_bytes)
{
    if (lds_bytes <= 64 * 1024) return hipSuccess;
    for (const void *k : c->big_lds_kernels)
        if (k == kernel) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e == hipSuccess) c->big_lds_kernels.push_back(kernel);
    return e;
}

// Bytes of scratch the calls of each source file take at most for the given sizes (adapt_workspace_bytes)
size_t ws_need_quantize(int num_cu, uint64_t n);
size_t ws_need_quantize_batched(int num_cu, int count);
size_t ws_need_kld_search(int num_cu, uint64_t n, int wl_lo, int wl_hi, int bins);
size_t ws_need_kld_search_batched(int num_cu, const adapt_kld_item *items, int count, int wl_lo, int wl_hi);
size_t ws_need_sgd_update(int num_cu, uint64_t n);
size_t ws_need_gradient_diversity(uint64_t n, int count);
size_t ws_need_requantize_fit(int num_cu, uint64_t n);

inline bool fmt_ok(adapt_fmt f) { return f.wl >= 2 && f.wl <= 16 && f.fl >= 0 && f.fl <= 31; }
inline int storage_bytes(adapt_fmt f) { return f.wl <= 8 ? 1 : f.wl <= 16 ? 2 : 4; }      // int8, int16 or int32 codes
// word lengths 17..32 (int32 codes): only the entry points that say so take them
// true when a contraction with these formats takes the composed path for word lengths above 16
inline bool wants_wide(adapt_fmt fa, adapt_fmt fb, const adapt_epilogue &ep) { return fa.wl > 16 || fb.wl > 16 || (!ep.raw && ep.fmt.wl > 16); }
inline bool fmt_ok_wide(adapt_fmt f) { return f.wl >= 2 && f.wl <= 32 && f.fl >= 0 && f.fl <= 31; }

}  // namespace adapt
