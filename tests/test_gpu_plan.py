"""GPU: a decode with a prepared work assignment (anszp_plan_decode / anszp_decode_planned) gives what the oracle
gives, bit for bit, and the same status words as anszp_decode; plans that do not fit are refused or harmless."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

from helpers import host_from_oracle, oracle_encode, oracle_expected

pytestmark = pytest.mark.gpu


def _workloads():
    return {"tiny": W.tiny(), "config1": W.config1(), "config2": W.config2(), "config3": W.config3(),
            "channel_grouped": W.channel_grouped(), "ragged": W.tiny(seed=11, n=70001, bitwidth=3, n_streams=48)}


@pytest.mark.parametrize("name", ["tiny", "config1", "config2", "config3", "channel_grouped", "ragged"])
def test_planned_decode_equals_the_oracle(orc, name):
    w = _workloads()[name]
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.alloc_out(d)
    args = B.decode_args(d, out)
    assert B.plan_bytes(args.n_chunks) >= 128 and B.plan_bytes(args.n_chunks) % 128 == 0
    plan = B.plan_decode(args)
    for _ in range(2):                                   # a plan serves any number of launches
        out.view(torch.uint8).fill_(0xA5)
        B.decode_planned_raw(args, plan)
        assert d.read_status() == (0, 0)
        got = B.bits_of(out)[:w.numel]
        bad = np.nonzero(got != expect)[0]
        assert len(bad) == 0, f"{len(bad)} mismatches, first at {bad[:5]}"


def test_plan_outlives_the_descriptor_array(orc):
    # the plan holds the descriptors it was made from: scribbling over the array afterwards changes nothing
    w = W.config2()
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.alloc_out(d)
    args = B.decode_args(d, out)
    plan = B.plan_decode(args)
    torch.cuda.synchronize()
    d.chunks.view(torch.uint8).fill_(0xFF)
    out.view(torch.uint8).fill_(0xA5)
    B.decode_planned_raw(args, plan)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)


def test_corrupt_streams_are_flagged_alike(orc):
    w = W.config2()
    c = oracle_encode(orc, w)
    h = host_from_oracle(c, w)
    h.payload[len(h.payload) // 3] ^= 0x00100400
    h.stream_hdr[17] ^= 0x5
    d = B.to_device(h)
    out_a, out_b = B.alloc_out(d), B.alloc_out(d)
    out_a.view(torch.uint8).fill_(0xA5)
    out_b.view(torch.uint8).fill_(0xA5)
    B.decode_raw(B.decode_args(d, out_a))
    st_a = d.read_status()
    d.status.zero_()
    args = B.decode_args(d, out_b)
    B.decode_planned_raw(args, B.plan_decode(args))
    st_b = d.read_status()
    assert st_a == st_b and st_a[0] != 0
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))


def test_plans_that_do_not_fit(orc):
    w2, w3 = W.config2(), W.config3()
    d2, d3 = B.to_device(B.pack_workload(w2)), B.to_device(B.pack_workload(w3))
    out2, out3 = B.alloc_out(d2), B.alloc_out(d3)
    a2, a3 = B.decode_args(d2, out2), B.decode_args(d3, out3)
    plan2 = B.plan_decode(a2)
    # another container (other number of chunks, other kernel geometry): refused on the device, nothing written
    big = torch.zeros(max(plan2.numel(), B.plan_bytes(a3.n_chunks)), dtype=torch.uint8, device="cuda:0")
    big[:plan2.numel()] = plan2
    out3.view(torch.uint8).fill_(0xA5)
    B.decode_planned_raw(a3, big)
    st = d3.read_status()
    assert st[0] == B.ST_BAD_DESC and st[1] >= 1
    assert bool((out3.view(torch.uint8) == 0xA5).all())
    # host-side refusals: no plan, a plan that is too small, a misaligned one
    stream = torch.cuda.current_stream().cuda_stream
    L = B.lib()
    assert L.anszp_decode_planned(C.byref(a2), None, 0, stream) == B.lib().anszp_decode_planned(C.byref(a2), None, 1 << 20, stream) != 0
    assert B.strerror(L.anszp_decode_planned(C.byref(a2), plan2.data_ptr(), plan2.numel() - 128, stream)) == B.strerror(L.anszp_plan_decode(C.byref(a2), plan2.data_ptr(), 64, stream))
    assert L.anszp_decode_planned(C.byref(a2), plan2.data_ptr() + 4, plan2.numel(), stream) != 0
    assert L.anszp_plan_bytes(1 << 31) == 0
    torch.cuda.synchronize()
    assert d2.read_status() == (0, 0)


def test_launches_that_need_no_plan(orc):
    # chunks too long for the look-ahead kernel go to the streaming kernel: the plan is neither written nor read
    w = W.config4(n_blocks=1, d_model=512, d_ff=1024)
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.alloc_out(d)
    args = B.decode_args(d, out)
    plan = torch.full((max(16, B.plan_bytes(args.n_chunks)),), 0x5A, dtype=torch.uint8, device="cuda:0")
    with torch.cuda.device("cuda:0"):
        assert B.lib().anszp_plan_decode(C.byref(args), plan.data_ptr(), plan.numel(), torch.cuda.current_stream().cuda_stream) == 0
    B.decode_planned_raw(args, plan)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)
    assert bool((plan == 0x5A).all())


@pytest.mark.parametrize("name", ["config2", "config3"])
def test_many_launches_all_give_the_oracle_s_bits(orc, name):
    """The hand-overs between a chunk's wavefronts depend on timing; 300 launches in a row (planned and not, back
    to back, so that launches overlap each other's tails) must each leave exactly the oracle's bits and clean
    status words."""
    w = _workloads()[name]
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.alloc_out(d)
    args = B.decode_args(d, out)
    plan = B.plan_decode(args)
    B.decode_planned_raw(args, plan)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)
    want = out.view(torch.int16).clone()
    for i in range(300):
        out.view(torch.uint8).fill_(0x5A)
        if i % 3 == 2:
            B.decode_raw(args)
        else:
            B.decode_planned_raw(args, plan)
        assert bool(torch.equal(out.view(torch.int16), want)), f"launch {i} differs"
    assert d.read_status() == (0, 0)
