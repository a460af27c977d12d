"""GPU: the entry point that allocates nothing (anszp_decode_static_plan keeps its plan in device memory of the
library's own) against anszp_decode_planned with a caller's plan buffer: same outputs, same status words, on
two calls in a row, the second with a smaller input; a third call reuses the plan the second one wrote."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(w):
    d = B.to_device(B.pack_workload(w))
    want, got = B.alloc_out(d), B.alloc_out(d)
    want.view(torch.uint8).fill_(0xA5)
    got.view(torch.uint8).fill_(0xA5)
    a_want, a_got = B.decode_args(d, want), B.decode_args(d, got)
    B.decode_planned_raw(a_want, B.plan_decode(a_want))
    st_want = d.read_status()
    d.status.zero_()
    return d, want, got, a_got, st_want


def test_static_plan_equals_callers_plan():
    first, second = W.config3(), W.config2()           # 369 chunks (large geometry), then 686 shorter ones of fewer symbols (small geometry)
    assert second.numel < first.numel
    for w in (first, second):
        d, want, got, args, st_want = _both(w)
        B.decode_static_plan_raw(args, True)
        assert d.read_status() == st_want == (0, 0)
        assert torch.equal(want.view(torch.uint8), got.view(torch.uint8))
    # the array still holds the second call's plan
    got.view(torch.uint8).fill_(0x5A)
    B.decode_static_plan_raw(args, False)
    assert d.read_status() == (0, 0)
    assert torch.equal(want.view(torch.uint8), got.view(torch.uint8))
    # a smaller input still: one chunk
    d, want, got, args, st_want = _both(W.tiny(n=1500))
    B.decode_static_plan_raw(args, True)
    assert d.read_status() == st_want == (0, 0)
    assert torch.equal(want.view(torch.uint8), got.view(torch.uint8))


def test_static_plan_limits():
    w = W.tiny(n=64 * 4200, chunk_size=64)              # 4200 chunks: more than the array holds
    d = B.to_device(B.pack_workload(w))
    out = B.alloc_out(d)
    args = B.decode_args(d, out)
    assert args.n_chunks > 4096
    with torch.cuda.device("cuda:0"):
        rc = B.lib().anszp_decode_static_plan(C.byref(args), 1, torch.cuda.current_stream().cuda_stream)
    assert rc != 0 and "range" in B.strerror(rc).lower()
    torch.cuda.synchronize()
    assert d.read_status() == (0, 0)
