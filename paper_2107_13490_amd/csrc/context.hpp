// Library context: stream, device facts and the single workspace allocation.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "adapt_fxp.h"

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
};

namespace adapt {

constexpr size_t kCtlBytes = 4096;
constexpr size_t kDefaultWorkspace = (size_t)64 << 20;

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

inline bool fmt_ok(adapt_fmt f) { return f.wl >= 2 && f.wl <= 16 && f.fl >= 0 && f.fl <= 31; }
inline int storage_bytes(adapt_fmt f) { return f.wl <= 8 ? 1 : 2; }

}  // namespace adapt
