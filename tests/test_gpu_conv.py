"""GPU parity of the fused decode + convolution entry point: anszp_conv_fused through the C ABI on
containers the ORACLE's encoder produced, against the fp64 convolution oracle applied to the
generated symbols and activations."""
import numpy as np
import pytest
import torch

from oracle import conv_oracle as CO
from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

from helpers import host_from_oracle, oracle_encode

pytestmark = pytest.mark.gpu


def _layer(shape, bitwidth, p0, seed, scale=0.03125, channel_scales=None):
    z = 1 << (bitwidth - 1)
    cout, cin, kh, kw = shape
    lay = W.Layer("conv", shape, bitwidth, z, scale, W.peaked_geometric_pmf(1 << bitwidth, z, p0), seed)
    if channel_scales is not None:
        lay.channel_len = cin * kh * kw
        lay.channel_scales = channel_scales
    return lay


def _case(orc, shape, B_, H, Wd, stride, pad, bitwidth=4, p0=0.7, n_streams=64, table_log=12, seed=1, per_channel=False,
          x_layout="nhwc", y_layout="nhwc"):
    cout, cin, kh, kw = shape
    K = cin * kh * kw
    rows = B.conv_rows_per_chunk(K)
    cs = None
    if per_channel:
        cs = (0.01 + 0.002 * np.arange(cout)).astype(np.float32)
    lay = _layer(shape, bitwidth, p0, seed, channel_scales=cs)
    w = W.Workload("conv_case", [lay], table_log, n_streams, rows * K, "bf16")
    c = oracle_encode(orc, w)                                   # the oracle's encoder, the oracle's bytes
    d = B.to_device(host_from_oracle(c, w))
    codes, values = W.bf16_activations(B_ * H * Wd * cin, seed + 100)
    x = torch.from_numpy(codes.view(np.int16).reshape(B_, H, Wd, cin)).to("cuda:0").view(torch.bfloat16)
    if x_layout == "c8":
        x = B.to_c8(x)
    y = B.conv_fused(d, 0, 0, rows, x, shape, stride, pad, x_layout=x_layout, y_layout=y_layout)
    status = d.read_status()
    if y_layout == "c8":
        y = B.from_c8(y)
    got = y.cpu().numpy().astype(np.float64)

    sym = lay.symbols().reshape(cout, kh, kw, cin)              # order [cout][kh][kw][cin]
    q = sym.astype(np.int64) - lay.zero_point
    x64 = values.astype(np.float64).reshape(B_, H, Wd, cin)
    if per_channel:
        wts = q.astype(np.float64) * cs.astype(np.float64)[:, None, None, None]
    else:
        wts = CO.dequantized_weights(sym, lay.zero_point, lay.scale, sym.shape)
    want = CO.conv2d_nhwc(x64, wts, stride, pad)
    return status, got, want, CO.conv2d_nhwc(np.abs(x64), np.abs(wts), stride, pad)


def _check(status, got, want, magnitude):
    assert status == (0, 0), status
    assert got.shape == want.shape
    # every product is exact in fp32 (bf16 x 8-bit integer); what remains is fp32 summation: a few units
    # in the last place of the sum of magnitudes, and one rounding by the scale
    bound = 2.0 ** -20 * magnitude + 1e-30
    worst = np.max(np.abs(got - want) - bound)
    assert worst <= 0, f"beyond the summation bound by {worst}"
    # the stated bar of the fused variant: max error relative to the output's scale <= 1e-2
    assert np.max(np.abs(got - want)) <= 1e-2 * np.max(np.abs(want))


@pytest.mark.parametrize("shape,B_,H,Wd,stride,pad", [
    ((32, 64, 1, 1), 2, 9, 7, 1, 0),          # pointwise
    ((16, 32, 3, 3), 3, 10, 10, 1, 1),        # 300 output pixels: a ragged last block of 64
    ((48, 64, 3, 3), 1, 13, 11, 2, 1),        # stride 2
    ((64, 3, 7, 7), 2, 20, 20, 2, 3),         # first layer: 3 input channels, K = 147
    ((16, 128, 1, 1), 2, 9, 9, 2, 0),         # strided pointwise (downsample)
    ((16, 8, 3, 3), 1, 6, 5, 1, 1),           # 8 input channels: a tap is a quarter of an MFMA's k
    ((32, 40, 3, 3), 1, 7, 7, 1, 1),          # 40 input channels: the last 32 k of a tap are partly beyond it
    ((16, 512, 3, 3), 1, 7, 7, 1, 1),         # K = 4608: the largest panel
    ((16, 5, 2, 2), 1, 5, 5, 1, 0),           # odd everything, no padding
    ((64, 256, 3, 3), 2, 7, 7, 1, 1),         # K = 2304: two row tiles per workgroup is what fits on chip
    ((128, 64, 3, 3), 2, 9, 9, 1, 1),         # four row tiles per workgroup, two such panels
])
def test_convolution_shapes(orc, shape, B_, H, Wd, stride, pad):
    _check(*_case(orc, shape, B_, H, Wd, stride, pad))


@pytest.mark.parametrize("shape,B_,H,Wd,stride,pad,layout", [
    ((64, 256, 1, 1), 2, 14, 14, 1, 0, "c8"),     # pointwise, four steps' loads in flight, bf16 panel of four row tiles
    ((32, 1024, 1, 1), 1, 7, 7, 1, 0, "c8"),      # pointwise, byte panel widened to bf16 in place
    ((64, 128, 1, 1), 2, 9, 9, 2, 0, "c8"),       # strided pointwise through the ring of loads
    ((64, 64, 1, 1), 1, 30, 30, 1, 0, "nhwc"),    # 900 pixels, 57 column tiles: two rounds of tiles, two steps in flight
    ((32, 128, 3, 3), 3, 9, 9, 2, 1, "c8"),       # several taps through the ring: stride 2, taps outside the image
    ((64, 64, 3, 3), 2, 12, 12, 1, 1, "c8"),      # several taps through the ring: one group of two steps per tap
    ((32, 128, 3, 3), 5, 7, 7, 1, 1, "c8"),       # patch in LDS: a round of pixels spans five images
    ((16, 512, 3, 3), 9, 7, 7, 1, 1, "c8"),       # patch in LDS, K = 4608, sixteen steps, 441 pixels
    ((64, 128, 3, 3), 2, 30, 30, 1, 1, "nhwc"),   # patch in LDS: 1800 pixels, several workgroups and rounds, rows of 30
    ((32, 256, 3, 3), 1, 17, 5, 1, 1, "c8"),      # patch in LDS: narrow images, rows shorter than a column tile
    ((64, 3, 7, 7), 2, 24, 24, 2, 3, "nhwc"),     # 3 channels, image rows of 144 bytes staged in LDS with their padding
    ((32, 3, 3, 3), 3, 16, 16, 1, 1, "nhwc"),     # the same over three images, stride 1
    ((16, 5, 2, 2), 1, 9, 8, 1, 0, "nhwc"),       # 5 channels, no padding, a 2 x 2 kernel
    ((16, 12, 5, 5), 2, 40, 40, 3, 2, "nhwc"),    # 12 channels, stride 3, 392 pixels: K = 300 spans ten steps
    ((32, 64, 1, 3), 2, 8, 9, 1, 1, "c8"),        # a kernel of one row of three taps (a kernel row's taps loaded together)
    ((16, 128, 5, 3), 1, 9, 9, 2, 1, "c8"),       # five kernel rows of three taps, stride 2
    ((16, 64, 3, 5), 1, 9, 9, 1, 2, "c8"),        # five taps wide: the ring with the taps outermost
    ((128, 64, 3, 3), 1, 40, 40, 1, 1, "c8"),     # four row tiles, 1600 pixels: two column tiles per wavefront, several rounds
])
def test_shapes_of_the_pipelined_contractions(orc, shape, B_, H, Wd, stride, pad, layout):
    _check(*_case(orc, shape, B_, H, Wd, stride, pad, seed=shape[1] + H, x_layout=layout, y_layout=layout))


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        k = int(rng.choice([1, 3]))
        cin = int(rng.choice([8, 32, 64, 96, 128, 160, 192, 256, 320]))
        cout = int(rng.choice([16, 32, 48, 64, 128]))
        stride = int(rng.choice([1, 2]))
        pad = 0 if k == 1 else int(rng.choice([0, 1]))
        h, w = int(rng.integers(k + 2, 19)), int(rng.integers(k + 2, 19))
        batch = int(rng.integers(1, 5))
        layout = str(rng.choice(["c8", "nhwc"]))
        cases.append(((cout, cin, k, k), batch, h, w, stride, pad, layout, int(rng.integers(1, 9)), float(rng.choice([0.5, 0.8, 0.93])), 1000 + i))
    return cases


@pytest.mark.parametrize("shape,B_,H,Wd,stride,pad,layout,bitwidth,p0,seed", _random_cases(36, 20240611))
def test_seeded_random_shapes(orc, shape, B_, H, Wd, stride, pad, layout, bitwidth, p0, seed):
    """Channel counts, kernel sizes, strides, image sizes, batches, layouts and alphabets drawn from a seeded generator:
    every way the kernel has of addressing the activations, with ragged pixel counts."""
    _check(*_case(orc, shape, B_, H, Wd, stride, pad, bitwidth=bitwidth, p0=p0, seed=seed, x_layout=layout, y_layout=layout))


@pytest.mark.parametrize("bitwidth,p0,n_streams,table_log", [(1, 0.9, 64, 12), (8, 0.75, 64, 12), (3, 0.3, 32, 10), (5, 0.8, 7, 9)])
def test_alphabets_streams_and_table_sizes(orc, bitwidth, p0, n_streams, table_log):
    _check(*_case(orc, (32, 32, 3, 3), 2, 8, 8, 1, 1, bitwidth=bitwidth, p0=p0, n_streams=n_streams,
                  table_log=table_log, seed=bitwidth))


def test_scale_per_output_channel(orc):
    _check(*_case(orc, (32, 16, 3, 3), 2, 6, 6, 1, 1, per_channel=True))


def test_bf16_output_is_the_fp32_output_rounded(orc):
    shape, K = (32, 32, 3, 3), 288
    rows = B.conv_rows_per_chunk(K)
    lay = _layer(shape, 4, 0.7, 11)
    w = W.Workload("conv_case", [lay], 12, 64, rows * K, "bf16")
    d = B.to_device(host_from_oracle(oracle_encode(orc, w), w))
    codes, values = W.bf16_activations(2 * 9 * 9 * 32, 12)
    x = torch.from_numpy(codes.view(np.int16).reshape(2, 9, 9, 32)).to("cuda:0").view(torch.bfloat16)
    y32 = B.conv_fused(d, 0, 0, rows, x, shape, 1, 1)
    y16 = B.conv_fused(d, 0, 0, rows, x, shape, 1, 1, y_dtype="bf16")
    assert d.read_status() == (0, 0)
    assert y16.dtype == torch.bfloat16
    assert torch.equal(y16, y32.to(torch.bfloat16))               # round to nearest even of the same fp32 sums
    sym = lay.symbols().reshape(32, 3, 3, 32)
    want = CO.conv2d_nhwc(values.astype(np.float64).reshape(2, 9, 9, 32),
                          CO.dequantized_weights(sym, lay.zero_point, lay.scale, sym.shape), 1, 1)
    got = y16.float().cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want) - 2.0 ** -8 * np.abs(want)) <= 1e-6 * np.max(np.abs(want))
    assert np.max(np.abs(got - want)) <= 1e-2 * np.max(np.abs(want))


@pytest.mark.parametrize("shape,B_,H,Wd,stride,pad", [
    ((32, 64, 1, 1), 2, 9, 7, 1, 0), ((64, 32, 3, 3), 2, 10, 11, 1, 1), ((48, 64, 3, 3), 1, 13, 11, 2, 1),
    ((32, 40, 3, 3), 1, 7, 7, 1, 1), ((16, 512, 3, 3), 1, 7, 7, 1, 1), ((64, 256, 3, 3), 2, 7, 7, 1, 1),
])
@pytest.mark.parametrize("x_layout,y_layout", [("c8", "c8"), ("nhwc", "c8"), ("c8", "nhwc")])
def test_channel_blocked_layouts(orc, shape, B_, H, Wd, stride, pad, x_layout, y_layout):
    _check(*_case(orc, shape, B_, H, Wd, stride, pad, x_layout=x_layout, y_layout=y_layout))


def test_first_layer_reads_an_image_and_writes_channel_blocks(orc):
    _check(*_case(orc, (64, 3, 7, 7), 2, 20, 20, 2, 3, y_layout="c8"))


def test_many_pixels_several_splits(orc):
    # 2 * 40 * 40 = 3200 output pixels: 50 blocks of 64 spread over workgroups and wavefronts
    _check(*_case(orc, (64, 32, 3, 3), 2, 40, 40, 1, 1, seed=9))


def test_chunk_whose_words_exceed_the_staging_buffer(orc):
    # a table that gives the layer's only symbol one state in 4096: every weight costs 12 bits, a chunk of one
    # output channel (4608 weights) 1728 words, more than a wavefront stages on chip: decoded from global memory
    shape, K = (16, 512, 3, 3), 4608
    sym = np.ones(16 * K, dtype=np.uint8)
    freqs = np.zeros(256, dtype=np.uint32)
    freqs[0], freqs[1] = 4095, 1
    c = orc.encode_layers([sym], 12, 64, K, freqs=[freqs])
    assert int(c.chunk_payload_words.max()) > 1280
    lay = W.Layer("rare", shape, 1, 0, 0.5, np.array([0.0, 1.0]), 0)
    w = W.Workload("rare", [lay], 12, 64, K, "bf16")
    d = B.to_device(host_from_oracle(c, w))
    codes, values = W.bf16_activations(1 * 5 * 5 * 512, 21)
    x = torch.from_numpy(codes.view(np.int16).reshape(1, 5, 5, 512)).to("cuda:0").view(torch.bfloat16)
    y = B.conv_fused(d, 0, 0, 1, x, shape, 1, 1)
    status = d.read_status()
    x64 = values.astype(np.float64).reshape(1, 5, 5, 512)
    wts = CO.dequantized_weights(sym, 0, 0.5, (16, 3, 3, 512))
    _check(status, y.cpu().numpy().astype(np.float64), CO.conv2d_nhwc(x64, wts, 1, 1),
           CO.conv2d_nhwc(np.abs(x64), np.abs(wts), 1, 1))


def test_corrupt_stream_is_reported(orc):
    shape, K = (16, 32, 3, 3), 288
    rows = 8                                    # 36 symbols per stream: the flipped bits are bits a stream reads, not its padding
    lay = _layer(shape, 4, 0.7, 3)
    w = W.Workload("conv_case", [lay], 12, 64, rows * K, "bf16")
    c = oracle_encode(orc, w)
    h = host_from_oracle(c, w)
    h.payload[len(h.payload) // 2] ^= 0x00F0F000
    d = B.to_device(h)
    codes, _ = W.bf16_activations(1 * 6 * 6 * 32, 4)
    x = torch.from_numpy(codes.view(np.int16).reshape(1, 6, 6, 32)).to("cuda:0").view(torch.bfloat16)
    y = B.conv_fused(d, 0, 0, rows, x, shape, 1, 1)
    bits, count = d.read_status()
    assert bits & (B.ST_BAD_STATE | B.ST_BAD_LENGTH) and count >= 1
    assert torch.isfinite(y).all()


@pytest.mark.parametrize("shape", [(16, 32, 3, 3), (16, 256, 3, 3)])        # bf16 panel, byte panel
@pytest.mark.parametrize("field,value", [("n_symbols", 17), ("layer_id", 1), ("payload_offset", 1 << 40),
                                         ("payload_offset", 2), ("payload_words", 1 << 30), ("stream_offset", 0xFFFFFF00)])
def test_chunk_descriptor_that_does_not_fit_is_skipped(orc, shape, field, value):
    cout, cin, kh, kw = shape
    K = cin * kh * kw
    rows = B.conv_rows_per_chunk(K)
    lay = _layer(shape, 4, 0.7, 31)
    w = W.Workload("conv_case", [lay], 12, 64, rows * K, "bf16")
    h = host_from_oracle(oracle_encode(orc, w), w)
    h.chunks[field][len(h.chunks) - 1] = value
    d = B.to_device(h)
    codes, _ = W.bf16_activations(1 * 6 * 6 * cin, 32)
    x = torch.from_numpy(codes.view(np.int16).reshape(1, 6, 6, cin)).to("cuda:0").view(torch.bfloat16)
    y = B.conv_fused(d, 0, 0, rows, x, shape, 1, 1)
    bits, count = d.read_status()
    assert bits & B.ST_BAD_DESC and count >= 1
    assert torch.isfinite(y).all()


def test_rejected_arguments(orc):
    lay = _layer((16, 32, 1, 1), 4, 0.7, 5)
    w = W.Workload("conv_case", [lay], 12, 64, 16 * 32, "bf16")
    d = B.to_device(host_from_oracle(oracle_encode(orc, w), w))
    x = torch.zeros((1, 4, 4, 32), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(B.AnszpError):
        B.conv_fused(d, 0, 0, 16, x, (24, 32, 1, 1), 1, 0)          # cout not a multiple of 16
    with pytest.raises(B.AnszpError):
        B.conv_fused(d, 0, 0, 3, x, (16, 32, 1, 1), 1, 0)           # rows per chunk must divide 16
    a = B.conv_args(d, 0, 0, 16, x, (16, 32, 1, 1), 1, 0, torch.empty((1, 4, 4, 16), dtype=torch.float32, device="cuda:0"))
    a.x_layout = 7
    with pytest.raises(B.AnszpError):
        B.conv_fused_raw(a)                                        # unknown layout
    with pytest.raises(B.AnszpError):
        B.conv_fused(d, 0, 0, 16, x, (16, 32, 5, 5), 1, 0)          # kernel larger than the padded image
    big = torch.zeros((1, 4, 4, 1024), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(B.AnszpError):
        B.conv_fused(d, 0, 0, 1, big, (16, 1024, 3, 3), 1, 1)       # K = 9216 > 4608
    assert d.read_status() == (0, 0)


def test_bf16_panel_does_not_depend_on_stale_lds(orc):
    """Short rows (K <= 576) keep the panel as bf16 values, and the contraction reads it beyond what decoding
    writes (a row's columns from K to its end, the bytes behind the last row).  Those reads meet activations
    that are zero; whatever an earlier kernel left there must not turn 0 * x into NaN.  A helper kernel first
    fills every CU's LDS with +Inf (0x7F80) or NaN (0xFFFF) patterns."""
    import ctypes as C
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gpu_helpers", "liblds_fill.so")
    assert os.path.exists(path), "tests/gpu_helpers/liblds_fill.so is missing: run python -m paper_2406_06237_amd.build"
    helper = C.CDLL(path)
    helper.lds_fill.argtypes = [C.c_uint32, C.c_void_p, C.c_void_p]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    for pattern in (0x7F807F80, 0xFFFFFFFF, 0x7F80FF80):
        for shape, size, stride, pad in (((64, 3, 7, 7), 20, 2, 3), ((32, 40, 3, 3), 11, 1, 1), ((16, 8, 1, 1), 9, 1, 0)):
            assert helper.lds_fill(pattern, sink.data_ptr(), None) == 0
            torch.cuda.synchronize()
            layout = "c8" if shape[1] % 8 == 0 else "nhwc"
            status, got, want, mag = _case(orc, shape, 2, size, size, stride, pad, seed=pattern & 0xFFF, x_layout=layout)
            assert np.isfinite(got).all(), f"pattern {pattern:#x}, shape {shape}: non-finite outputs"
            _check(status, got, want, mag)
    assert int(sink[0]) == 0


def test_launches_replayed_from_a_captured_graph(orc):
    """Callers may capture the launches of several layers into a graph (after one eager call per kernel, which sets
    the kernel's LDS limit): every replay, with eager work and synchronisations between, must leave what the eager
    launches left."""
    cases = [((64, 128, 1, 1), 1, 0), ((32, 128, 3, 3), 1, 1), ((32, 64, 3, 3), 2, 1)]
    calls, outs, keep = [], [], []
    for i, (shape, stride, pad) in enumerate(cases):
        cout, cin, kh, kw = shape
        K = cin * kh * kw
        rows = B.conv_rows_per_chunk(K)
        lay = _layer(shape, 4, 0.8, 50 + i)
        w = W.Workload("conv_case", [lay], 12, 64, rows * K, "bf16")
        d = B.to_device(host_from_oracle(oracle_encode(orc, w), w))
        codes, _ = W.bf16_activations(2 * 10 * 10 * cin, 60 + i)
        x = B.to_c8(torch.from_numpy(codes.view(np.int16).reshape(2, 10, 10, cin)).to("cuda:0").view(torch.bfloat16))
        ho = (10 + 2 * pad - kh) // stride + 1
        y = torch.empty(B.conv_out_shape(2, ho, ho, cout, "c8"), dtype=torch.bfloat16, device="cuda:0")
        calls.append((d, B.conv_args(d, 0, 0, rows, x, shape, stride, pad, y, "c8", "c8")))
        outs.append(y)
        keep.append(x)                                        # the arguments hold addresses, not tensors

    def step():
        for _, a in calls:
            B.conv_fused_raw(a)

    step()
    torch.cuda.synchronize()
    want = [y.clone() for y in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(4):
        for y in outs:
            y.view(torch.int16).fill_(0x7FC0)                 # NaN patterns: a replay must overwrite every element
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for y, ref in zip(outs, want):
            assert torch.equal(y.view(torch.int16), ref.view(torch.int16))
        step()                                                # eager work between the replays
        torch.cuda.synchronize()
    for d, _ in calls:
        assert d.read_status() == (0, 0)
