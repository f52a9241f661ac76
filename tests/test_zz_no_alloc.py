"""GPU test of sx_expand_topk_static, the entry point for callers that cannot allocate: same results as
sx_expand_topk (they share the kernels) with the candidates staged in the library's fixed device array.
Two calls in a row, the second with a smaller input, so that what the first call left in the shared
array is seen not to leak into the second; then the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as wl
from helpers import dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sx():
    import paper_2406_02532_amd as m
    return m


def _both(sx, N, V, k, B, seed):
    logits, cum = wl.gen_expand_inputs(N, V, seed=seed, max_depth=16)
    lg, cm = to_dev(logits), to_dev(cum)
    ref = sx.expand_topk(lg, cm, k, B)[:4]
    outs = (torch.full((B,), -7, dtype=torch.int32, device=dev()), torch.full((B,), -7, dtype=torch.int32, device=dev()),
            torch.full((B,), float("nan"), dtype=torch.float32, device=dev()), torch.full((1,), -7, dtype=torch.int32, device=dev()))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = sx.expand_topk_static(lg, cm, k, B, *outs)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    n = int(ref[3].item())
    assert int(got[3].item()) == n == min(B, N * k)
    for a, b in zip(got[:3], ref[:3]):                       # same kernels on the same inputs: bit for bit
        assert torch.equal(a[:n], b[:n])


def test_static_scratch_matches_workspace_entry_point_twice(sx):
    _both(sx, N=2048, V=32000, k=32, B=2048, seed=11)        # exactly the limit: 65536 candidates
    _both(sx, N=37, V=1000, k=5, B=64, seed=12)              # smaller, ragged, right after: stale entries must not show
    _both(sx, N=3, V=50000, k=7, B=100, seed=13)             # B above N*k: every candidate comes back, streaming kernel


def test_static_scratch_rejects_what_does_not_fit(sx):
    one = C.c_void_p(256)   # never dereferenced: the size check comes before any launch
    L = sx.lib
    assert L.sx_expand_topk_static(one, one, 2049, 32000, 32, 2048, one, one, one, one, None) == -2
    assert L.sx_expand_topk_static(one, one, 300, 32000, 256, 2048, one, one, one, one, None) == -2
    assert L.sx_expand_topk_static(None, one, 4, 100, 2, 4, one, one, one, one, None) == -1
