"""Helpers of the GPU parity tests: the HIP path is reached only through the C-ABI binding."""
import numpy as np
import torch

import paper_2107_13490_amd as pkg

_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        _ctx = pkg.Context()
    return _ctx


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def u64(t):
    return host(t).view(np.uint64)


def oracle_quantize(x, wl, fl, seed, stream):
    """The oracle's quantizer (SR) over a large tensor: slices of 2^20 elements, each with the rounding bits of its
    own index range, spread over the host's cores.  Returns int64 codes of x's shape."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from oracle import fxp_oracle as orc
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.empty(flat.size, dtype=np.int64)
    step = 1 << 20

    def part(a):
        b = min(flat.size, a + step)
        bits = orc.r16(seed, stream, np.arange(a, b, dtype=np.uint64))
        out[a:b] = orc.quantize_with_bits(flat[a:b], wl, fl, bits)[0]

    with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1))) as pool:
        list(pool.map(part, range(0, flat.size, step)))
    return out.reshape(np.shape(x))
