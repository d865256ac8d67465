// Updates of all layers of a chained step in one launch each (Alg. 1: the backward-pass line and the per-layer
// Quantize loop; batch-normalisation parameters as in the per-layer call).  Results are those of the per-layer
// entry points bit for bit: every element's arithmetic and rounding bits depend on its index in its own tensor only.
#pragma once
#include <cstddef>
#include <cstdint>

#include "adapt_fxp.h"

struct adapt_ctx;

namespace adapt {

constexpr int kUpdateMaxItems = 32;      // tensors per launch (descriptors travel in the kernel arguments)

// One layer of adapt_sgd_update_quantize; codes of at most 16 bits on both sides
struct SgdBatchItem {
    float *w;
    const void *g;
    void *q;
    const uint64_t *g_sumsq;      // device, or null
    uint64_t n;
    uint64_t seed, stream;
    uint64_t *counters;           // device: nnz, saturated; or null
    float *range;                 // device: min, max of the finite new weights; or null
    int8_t es_g, es_q;            // bytes per gradient / weight code: 1 or 2
    int8_t fl_g;
    int8_t wl, fl;                // format of the weight codes
};

// Enqueues the fused update of `count` layers: one launch for the element work and one for the totals per
// kUpdateMaxItems layers.  ADAPT_EWORKSPACE when the context's scratch cannot hold the per-block partials (nothing is
// enqueued then).
int sgd_update_batch(adapt_ctx *ctx, const SgdBatchItem *items, int count, adapt_sgd_params opt, int mode);

// One layer of adapt_bn_update
struct BnUpdateItem {
    float *gamma, *beta;
    const double *dgamma, *dbeta;
    int channels;
};

// Enqueues the parameter updates of `count` normalisation layers, one block per layer
int bn_update_batch(adapt_ctx *ctx, const BnUpdateItem *items, int count, double lr);

}  // namespace adapt
