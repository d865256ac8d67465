"""GPU parity of the entry point that allocates nothing (adapt_quantize_noalloc, scratch in a static device array)
against adapt_quantize: identical codes and counters, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import paper_2107_13490_amd as pkg
import workloads as wk

from gpu_util import ctx, dev, host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,fl", [(8, 5), (12, 9)])
def test_quantize_noalloc_equals_quantize_on_two_calls_in_a_row(wl, fl):
    c = ctx()
    for n, stream in (((1 << 22) + 37, 3), (70001, 4), (5, 5)):      # the later calls are smaller than the first
        x = dev(wk.normal((n,), 1.0, 17, stream))
        x[:3] = torch.tensor([float("nan"), float("inf"), -1e9], device="cuda")[:min(3, n)]
        want_q, want_cnt = c.quantize(x, wl, fl, pkg.SR, 9, stream)
        out = torch.full((n,), 77, dtype=c.storage_dtype(wl), device="cuda")
        cnt = torch.full((2,), -1, dtype=torch.int64, device="cuda")
        before = torch.cuda.memory_allocated()
        c.quantize_noalloc(x, wl, fl, pkg.SR, 9, stream, out, cnt)
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out, want_q)
        assert np.array_equal(host(cnt), host(want_cnt))


def test_quantize_noalloc_argument_checks_and_other_contexts_share_the_array():
    c = ctx()
    x = dev(wk.normal((4096,), 1.0, 18, 1))
    out = torch.empty(4096, dtype=torch.int8, device="cuda")
    cnt = torch.zeros(2, dtype=torch.int64, device="cuda")
    with pytest.raises(pkg.AdaptError):
        c.quantize_noalloc(x, 33, 5, pkg.SR, 0, 0, out, cnt)
    with pytest.raises(pkg.AdaptError):
        c.quantize_noalloc(x[1:], 8, 5, pkg.SR, 0, 0, out, cnt)          # misaligned input
    tiny = pkg.Context(workspace_bytes=256)                               # no room for partials in its workspace: not needed
    tiny.quantize_noalloc(x, 8, 5, pkg.SR, 1, 2, out, cnt)
    want_q, want_cnt = c.quantize(x, 8, 5, pkg.SR, 1, 2)
    assert torch.equal(out, want_q) and np.array_equal(host(cnt), host(want_cnt))
    e = torch.empty(0, dtype=torch.float32, device="cuda")
    c.quantize_noalloc(e, 8, 5, pkg.SR, 0, 0, torch.empty(0, dtype=torch.int8, device="cuda"), cnt)
    assert host(cnt).tolist() == [0, 0]
    tiny.close()
