// Context management and the small host-only entry points of the C ABI.
#include <new>

#include "common.hpp"
#include "context.hpp"

using namespace adapt;

extern "C" int adapt_version(void) { return 1; }

extern "C" const char *adapt_error_string(int status)
{
    switch (status) {
        case ADAPT_OK: return "ok";
        case ADAPT_EINVAL: return "invalid argument (null or misaligned pointer, size or format out of range)";
        case ADAPT_EUNSUPPORTED: return "unsupported request";
        case ADAPT_EBOUND: return "exact result does not fit the accumulator or output type";
        case ADAPT_EHIP: return "HIP runtime error";
        case ADAPT_EWORKSPACE: return "context workspace too small";
        default: return "unknown status";
    }
}

extern "C" int adapt_create(adapt_ctx **out, void *hip_stream, size_t workspace_bytes)
{
    if (!out) return ADAPT_EINVAL;
    *out = nullptr;
    adapt_ctx *c = new (std::nothrow) adapt_ctx();
    if (!c) return ADAPT_EHIP;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->last_hip_error = hipSuccess;
    hipError_t e = hipGetDevice(&c->device);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) { delete c; return ADAPT_EHIP; }
    c->num_cu = prop.multiProcessorCount;
    c->ws_bytes = (workspace_bytes ? workspace_bytes : kDefaultWorkspace) + kCtlBytes;
    e = hipMalloc(reinterpret_cast<void **>(&c->ws), c->ws_bytes);
    if (e == hipSuccess) e = hipMemset(c->ws, 0, kCtlBytes);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { if (c->ws) (void)hipFree(c->ws); delete c; return ADAPT_EHIP; }
    // the current device's copy of the static scratch array (see adapt_quantize_noalloc); a failure here only
    // disables that entry point
    if (static_scratch_address(&c->static_scratch) != hipSuccess) {
        c->static_scratch = nullptr;
        (void)hipGetLastError();
    }
    *out = c;
    return ADAPT_OK;
}

extern "C" int adapt_destroy(adapt_ctx *c)
{
    if (!c) return ADAPT_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    hipError_t f = hipFree(c->ws);
    delete c;
    return (e == hipSuccess && f == hipSuccess) ? ADAPT_OK : ADAPT_EHIP;
}

extern "C" int adapt_set_stream(adapt_ctx *c, void *hip_stream)
{
    if (!c) return ADAPT_EINVAL;
    c->stream = static_cast<hipStream_t>(hip_stream);
    return ADAPT_OK;
}

extern "C" int adapt_acc_bits(int64_t K, adapt_fmt a, adapt_fmt b)
{
    if (K < 0 || !fmt_ok_wide(a) || !fmt_ok_wide(b)) return ADAPT_EINVAL;
    if (a.wl > 16 || b.wl > 16) return 128;                  // the composed path for wide operands sums in 128 bits
    // K * 2^(wl_a-1) * 2^(wl_b-1) <= 2^31 - 1, evaluated without overflow (K < 2^63, shift <= 30)
    const int sh = a.wl + b.wl - 2;
    const int64_t lim = ((int64_t)1 << 31) - 1;
    return (K <= (lim >> sh)) ? 32 : 64;
}

