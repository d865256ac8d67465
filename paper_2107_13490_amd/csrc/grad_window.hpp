// Window descriptions of the gradient-diversity kernels (Sec. 3.3 "The PushUp Operation"), shared by
// the stand-alone entry point and the chained step.
#pragma once
#include <cstddef>
#include <cstdint>

#include "adapt_fxp.h"

namespace adapt {

constexpr int kGdMaxTensors = 64;
constexpr int kGdMaxLayers = 64;         // layers of a chained step

// what the kernels read: tensors oldest first, each with its alignment to the finest grid
struct GradWindow {
    const void *g[kGdMaxTensors];
    uint8_t es[kGdMaxTensors];            // element bytes: 1, 2 or 4
    uint8_t shift[kGdMaxTensors];         // fl_max - fl_k
    int8_t fl[kGdMaxTensors];
    int count;
    int fl_max;
};

// Chained step, written by the host into pinned memory: the window of one layer, oldest first, whose
// last entry is this batch's gradient.  exp[k] is the exponent e of entry k (value = code * 2^-e);
// the last entry's is not known to the host: the device takes it from the record the backward pass wrote.
struct ChainLayerIn {
    const void *g[kGdMaxTensors];
    long long exp[kGdMaxTensors];
    uint8_t wl[kGdMaxTensors];
    int count;
};

// Chained step, written by the device into pinned memory
struct ChainLayerOut {
    double ds, log_ds;
    long long exp_new;                    // exponent of this batch's gradient
    int used;                             // entries that entered the sums (the newest `used` of the window)
    int pad;
};

}  // namespace adapt

struct adapt_ctx;

namespace adapt {

// Enqueues the diversities of all layers of a chained step: in / out are host-pinned, device-visible
// arrays of nlayers records, e_g[l * e_stride] the exponent of layer l's newest gradient in device
// memory, win device scratch for nlayers window descriptions, n[l] the element count of layer l's gradient.
int gradient_diversity_chain(adapt_ctx *ctx, const ChainLayerIn *in, int nlayers, const size_t *n, const long long *e_g, size_t e_stride,
                             GradWindow *win, ChainLayerOut *out);

}  // namespace adapt
