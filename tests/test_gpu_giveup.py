"""GPU: the bounded waits of the decode kernels.  With the bound lowered from the host (anszp_test_set_spin_limit) a
hand-over that is not satisfied at once is given up: the launch must report ANSZP_ST_INTERNAL, drain (every wavefront
leaves: the call returns and the device stays usable) and write nothing outside the output; with the default bound
back, the same container decodes to the oracle's bits.  No kernel is made to hang or fault: every wait still ends."""
import numpy as np
import pytest
import torch

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

from helpers import host_from_oracle, oracle_encode, oracle_expected

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["lookahead_large", "lookahead_small", "streaming"])
def test_a_wait_that_gives_up_drains_the_launch(orc, name):
    w = {"lookahead_large": W.tiny(seed=3, n=400000, bitwidth=6, n_streams=64, chunk_size=65536, table_log=12, p0=0.75),
         "lookahead_small": W.config2(),
         "streaming": W.config4(n_blocks=1, d_model=512, d_ff=1024)}[name]
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    guard = 4096
    buf = torch.full((w.numel + 2 * guard,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    out = buf[guard:guard + w.numel].view(torch.bfloat16)
    try:
        B.lib().anszp_test_set_spin_limit(1)
        B.decode(d, out=out)
        torch.cuda.synchronize()
        st = d.read_status()
        assert st[0] & B.ST_INTERNAL and st[1] >= 1, st
        assert bool((buf[:guard] == 0x5A5A).all()) and bool((buf[guard + w.numel:] == 0x5A5A).all())
    finally:
        B.lib().anszp_test_set_spin_limit(0)
    # a few polls are not enough either; the launch still drains
    try:
        B.lib().anszp_test_set_spin_limit(4)
        d.status.zero_()
        B.decode(d, out=out)
        torch.cuda.synchronize()
        assert d.read_status()[0] in (0, B.ST_INTERNAL)
    finally:
        B.lib().anszp_test_set_spin_limit(0)
    d.status.zero_()
    buf.fill_(0x5A5A)
    B.decode(d, out=out)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)
