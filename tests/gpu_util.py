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
