"""Streams that follow the input channels of a layer (Sec. III-B, end of Sec. II-A): weights stored
[cin / 64][cout][kh][kw][64], one chunk per group of 64 input channels, so that stream k of a chunk is input
channel 64 g + k.  The symbols' statistics differ from channel to channel, so the storage order matters to
what every stream holds.  Containers come from the ORACLE's encoder; the GPU decodes them through the C ABI
(look-ahead kernel for the chunks that fit its window, streaming kernel for the long ones) and every weight is
compared with the oracle's."""
import numpy as np
import pytest
import torch

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

from helpers import host_from_oracle, oracle_encode, oracle_expected

pytestmark = pytest.mark.gpu


def test_channel_grouped_streams_decode_to_the_oracles_weights(orc):
    w = W.channel_grouped()
    # the layout does what it says: stream k of a chunk holds one input channel, and channels differ
    lay = w.layers[0]
    t = lay.tensor()
    flat = lay.symbols()
    assert np.array_equal(W.from_channel_groups(flat, lay.shape), t)
    group0 = flat[:lay.group_symbols]
    for k in (0, 17, 63):
        assert np.array_equal(group0[k::64], t[:, k].reshape(-1))
    share = (t == lay.zero_point).mean(axis=(0, 2, 3))
    assert share.max() - share.min() > 0.25

    c = oracle_encode(orc, w)
    assert list(c.chunk_nsym[:2]) == [lay.group_symbols] * 2
    words = c.chunk_payload_words
    assert words.max() > B.LOOKAHEAD_WINDOW_WORDS > words.min()          # both kernels get chunks
    # streams of one chunk differ in length as their channels differ in compressibility
    first = (c.stream_hdr[:64] >> 16).astype(np.int64)
    assert first.max() > 1.5 * first.min()
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.alloc_out(d)
    out.view(torch.uint8).fill_(0xA5)
    B.decode_by_chunk_size(d, out=out)
    assert d.read_status() == (0, 0)
    got = B.bits_of(out)[:w.numel]
    bad = np.nonzero(got != expect)[0]
    assert len(bad) == 0, f"{len(bad)} mismatches, first at {bad[:5]}"
    # the library's own packer writes the same container for this layout
    h = B.pack_workload(w)
    assert np.array_equal(h.payload, c.payload) and np.array_equal(h.stream_hdr, c.stream_hdr)
    # and one call per kernel gives the same weights (every variant decodes every chunk, if slowly)
    for variant in (B.VARIANT_STEPWISE, B.VARIANT_STREAMING, B.VARIANT_MERGED):
        out2 = B.alloc_out(d)
        B.decode(d, out=out2, variant=variant)
        assert d.read_status() == (0, 0)
        assert np.array_equal(B.bits_of(out2)[:w.numel], expect), f"variant {variant}"
