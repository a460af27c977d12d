"""GPU parity: libanszp's decode + dequant through the C ABI against the CPU oracle, element by
element and bit for bit, on containers the ORACLE's encoder produced."""
import numpy as np
import pytest
import torch

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

from helpers import host_from_oracle, oracle_encode, oracle_expected

pytestmark = pytest.mark.gpu


def _run(orc, w, out_dtype=None):
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w, out_dtype)
    d = B.to_device(host_from_oracle(c, w))
    variants = [None, B.VARIANT_STEPWISE, B.VARIANT_MERGED, B.VARIANT_STEPWISE_SHARED, B.VARIANT_STREAMING]
    if w.table_log <= 8:
        variants.append(B.VARIANT_BYTE_TABLE)       # the 3 l-byte table of Sec. II-A holds at most 256 states
    for variant in variants:
        out = B.alloc_out(d, out_dtype)
        out.view(torch.uint8).fill_(0xA5)
        B.decode(d, out=out, out_dtype=out_dtype, variant=variant)
        status = d.read_status()
        got = B.bits_of(out)[:w.numel]
        assert status == (0, 0), f"variant {variant}: status {status}"
        bad = np.nonzero(got != expect)[0]
        assert len(bad) == 0, (f"variant {variant}: {len(bad)} mismatches, first at {bad[:5]}: "
                               f"got {got[bad[:5]]} want {expect[bad[:5]]}")
    return d, out


def test_config1_single_conv_fp32(orc):
    _run(orc, W.config1())


@pytest.mark.parametrize("dtype", ["u8", "f32", "bf16"])
@pytest.mark.parametrize("N,chunk,n,R,b,p0", [
    (64, 2048, 5000, 10, 4, 0.8), (64, 65536, 65536 + 1000, 12, 8, 0.7), (32, 16384, 40000, 11, 3, 0.6),
    (1, 3000, 7001, 10, 4, 0.5), (7, 100, 999, 9, 2, 0.9), (64, 4096, 40, 8, 5, 0.75),
    (64, 1024, 3 * 1024, 12, 1, 0.95), (33, 555, 5555, 6, 6, 0.3), (64, 128, 1, 5, 4, 0.8),
])
def test_ragged_geometries(orc, dtype, N, chunk, n, R, b, p0):
    w = W.tiny(seed=n, n=n, bitwidth=b, n_streams=N, chunk_size=chunk, table_log=R, p0=p0, out_dtype=dtype)
    _run(orc, w)


def test_single_symbol_layer_and_flat_distribution(orc):
    z = 4
    lay = W.Layer("const", (10000,), 3, z, 0.5, np.eye(1, 8, z)[0], 5)
    flat = W.Layer("flat", (20000,), 8, 128, 0.01, np.ones(256) / 256, 6)
    w = W.Workload("mix", [lay, flat, lay], 12, 64, 4096, "bf16")
    _run(orc, w)
    _run(orc, w, "f32")


def test_per_channel_scales(orc):
    w = W.config4(n_blocks=1, d_model=256, d_ff=704)
    w.chunk_size = 32768
    _run(orc, w)
    _run(orc, w, "f32")
    # channel length that is not a multiple of the stream count
    rng = np.random.default_rng(1)
    lay = W.Layer("odd", (37, 101), 4, 8, 0.0, W.laplace_pmf(16, 8, 1.0), 9, channel_len=101,
                  channel_scales=rng.uniform(0.005, 0.05, 37).astype(np.float32))
    w2 = W.Workload("odd", [lay, lay], 10, 64, 1000, "bf16")
    _run(orc, w2)
    # a layer with a scale per channel and no scales to read: every chunk is refused, nothing is written as zeros
    d = B.to_device(host_from_oracle(oracle_encode(orc, w2), w2))
    for variant in (None, B.VARIANT_STEPWISE, B.VARIANT_MERGED, B.VARIANT_STEPWISE_SHARED, B.VARIANT_STREAMING):
        out = B.alloc_out(d)
        out.view(torch.uint8).fill_(0xA5)
        a = B.decode_args(d, out)
        a.scales, a.n_scales = None, 0
        B.decode_raw(a, d.device, variant)
        st = d.read_status()
        assert st[0] == B.ST_BAD_DESC and st[1] == len(d.host.chunks), f"variant {variant}: {st}"
        assert bool((out.view(torch.uint8) == 0xA5).all()), f"variant {variant} wrote weights without scales"
        d.status.zero_()
    # too few scales for the last channels
    a = B.decode_args(d, B.alloc_out(d))
    a.n_scales = a.n_scales - 1
    B.decode_raw(a, d.device)
    assert d.read_status()[0] == B.ST_BAD_DESC


def test_config2_resnet18(orc):
    _run(orc, W.config2())


def test_config3_resnet50(orc):
    _run(orc, W.config3())


def test_config4_one_block_at_real_shapes(orc):
    """One of config 4's 32 identical blocks (4 of 4096x4096 and 3 of 4096x11008, 262,144-symbol chunks,
    per-output-channel scales): every chunk has the full-size geometry of the whole set."""
    w = W.config4(n_blocks=1)
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.decode(d)
    assert d.read_status() == (0, 0)
    got = B.bits_of(out)[:w.numel]
    assert np.array_equal(got, expect)
    # the merged kernel forced onto the same chunks (they exceed its window and fall back inside it)
    idx = np.random.default_rng(0).integers(0, w.numel, size=200000)
    out2 = B.decode(d, variant=B.VARIANT_MERGED)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out2)[:w.numel][idx], expect[idx])
    # the kernel the full set gets (24,704 chunks: the automatic choice is the streaming kernel), forced here
    out3 = B.decode(d, variant=B.VARIANT_STREAMING)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out3)[:w.numel], expect)


def test_many_large_chunks_take_the_streaming_kernel(orc):
    """More than 4096 chunks whose words exceed the on-chip window: the automatic choice is the streaming
    kernel (fourteen chunks per workgroup, several layers per workgroup at layer boundaries, per-channel
    scales, a ragged last chunk per layer) and must decode every element."""
    w = W.config4(n_blocks=1)
    w.chunk_size = 49152 - 64 * 3          # 4096 x 4096 and 4096 x 11008 are not multiples: ragged tails
    c = oracle_encode(orc, w)
    assert len(c.chunk_nsym) >= 4096 and c.payload.size / len(c.chunk_nsym) > 3584
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    out = B.decode(d)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)


@pytest.mark.parametrize("dtype", ["u8", "f32", "bf16"])
def test_no_dominant_symbol_ragged(orc, dtype):
    """64 streams and no state that reads zero bits: the streaming kernel's split into decoding and loading
    wavefronts, with a ragged last step, in every output type."""
    w = W.tiny(seed=3, n=5 * 8192 + 37, bitwidth=5, n_streams=64, chunk_size=8192, table_log=10, p0=0.3, out_dtype=dtype)
    _run(orc, w)


def test_streaming_workgroups_spanning_many_layers(orc):
    """800 layers of one chunk each: a workgroup of the streaming kernel gets chunks of three or four layers, more
    than the two tables it stages."""
    rng = np.random.default_rng(5)
    layers = []
    for i in range(800):
        b = int(rng.integers(2, 6))
        z = 1 << (b - 1)
        layers.append(W.Layer(f"l{i}", (64 * int(rng.integers(3, 9)) + int(rng.integers(0, 64)),), b, z,
                              float(rng.uniform(0.005, 0.05)), W.peaked_geometric_pmf(1 << b, z, float(rng.uniform(0.2, 0.9))), 100 + i))
    w = W.Workload("many_layers", layers, 8, 64, 1024, "bf16")
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    d = B.to_device(host_from_oracle(c, w))
    for variant in (B.VARIANT_STREAMING, B.VARIANT_STEPWISE_SHARED):
        out = B.alloc_out(d)
        out.view(torch.uint8).fill_(0xA5)
        B.decode(d, out=out, variant=variant)
        assert d.read_status() == (0, 0), f"variant {variant}"
        assert np.array_equal(B.bits_of(out)[:w.numel], expect), f"variant {variant}"


@pytest.mark.parametrize("R", [6, 7, 8])
def test_byte_tables_on_the_device_equal_the_oracles(orc, R):
    """Sec. II-A: the look-up table is 3 l bytes (symbol, nb_bits, newX, one byte each; 192 bytes for 64 states).
    The bytes anszp_build_tables_device and anszp_build_tables leave in device memory equal the oracle's table
    byte for byte at l = 64, 128, 256, and decoding through them (the byte-table kernel) gives the oracle's
    weights on the odd-bin set."""
    w = W.resnet50_odd_bins()
    w.layers = w.layers[:12]
    w.table_log = R
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    h = host_from_oracle(c, w)
    d = B.to_device(h)
    L = 1 << R
    on_device = d.tables.cpu().numpy().view(np.uint32).reshape(len(w.layers), -1)
    built = B.build_tables_device(torch.from_numpy(np.ascontiguousarray(h.freqs).astype(np.int32)).cuda(), R)
    built = built.cpu().numpy().view(np.uint32).reshape(len(w.layers), -1)
    for i in range(len(w.layers)):
        want = orc.decode_table_bytes(h.freqs[i], R)
        assert len(want) == 3 * L
        assert np.array_equal(B.split_table(on_device[i])["bytes"], want)
        assert np.array_equal(B.split_table(built[i])["bytes"], want)
    out = B.alloc_out(d)
    out.view(torch.uint8).fill_(0xA5)
    B.decode(d, out=out, variant=B.VARIANT_BYTE_TABLE)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)
    # larger tables have no byte form: the variant is refused
    w2 = W.tiny(n=1000, chunk_size=512, table_log=9)
    d2 = B.to_device(host_from_oracle(oracle_encode(orc, w2), w2))
    with pytest.raises(B.AnszpError) as e:
        B.decode(d2, variant=B.VARIANT_BYTE_TABLE)
    assert e.value.code == -2


@pytest.mark.parametrize("R", [6, 8])
def test_odd_bin_alphabets_with_small_tables(orc, R):
    """The alphabets the paper describes (odd bin counts 13..31, zero-point in the middle) coded with the
    table sizes of its Sec. III-B study (64 and 256 states)."""
    w = W.resnet50_odd_bins()
    w.layers = w.layers[:24]
    w.table_log = R
    _run(orc, w)


def test_library_packer_output_decodes_too(orc):
    """The same weights compressed by the library's own host packer."""
    w = W.tiny(n=70000, chunk_size=8192, table_log=11, p0=0.85)
    h = B.pack_workload(w)
    d = B.to_device(h)
    out = B.decode(d)
    assert d.read_status() == (0, 0)
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)


def test_dequant_zp_alone(orc):
    import torch
    rng = np.random.default_rng(2)
    q = rng.integers(0, 256, size=100003, dtype=np.uint8)
    qd = torch.from_numpy(q).cuda()
    for dt in ("f32", "bf16"):
        got = B.bits_of(B.dequant_zp(qd, 128, 0.0173, dt))
        want = orc.dequant(q, 128, 0.0173, dt)
        assert np.array_equal(got, want.view(np.uint32) if dt == "f32" else want)
    scales = rng.uniform(0.001, 0.1, size=1001).astype(np.float32)
    got = B.bits_of(B.dequant_zp(qd, 7, 0.0, "bf16", 100, torch.from_numpy(scales).cuda()))
    assert np.array_equal(got, orc.dequant(q, 7, 0.0, "bf16", 100, scales))
    # tie and denormal cases of the bf16 rounding
    for pattern in (0x3F808000, 0x3F818000, 0x00000007, 0x7F000000 // 255):
        s = float(np.array([pattern], np.uint32).view(np.float32)[0])
        small = torch.arange(0, 256, dtype=torch.uint8).cuda()
        for dt in ("f32", "bf16"):
            got = B.bits_of(B.dequant_zp(small, 3, s, dt))
            want = orc.dequant(np.arange(256, dtype=np.uint8), 3, s, dt)
            assert np.array_equal(got, want.view(np.uint32) if dt == "f32" else want)


def test_tables_built_on_the_device_equal_the_host_tables(orc):
    """anszp_build_tables_device against anszp_build_tables_host, word for word, over the frequency rows of the
    benchmark sets and of edge cases (one symbol, two symbols, all 256, a dominant symbol, ties between symbols of
    equal frequency), at several table sizes; a row that is not normalised is reported and yields zeros; and a
    container decodes with device-built tables."""
    import torch
    rng = np.random.default_rng(11)
    for R in (1, 5, 8, 10, 12):
        L = 1 << R
        rows = []
        one = np.zeros(256, np.uint32); one[7] = L; rows.append(one)
        if L >= 2:
            two = np.zeros(256, np.uint32); two[3] = L // 2; two[200] = L - L // 2; rows.append(two)
            dom = np.zeros(256, np.uint32); dom[8] = L - 1; dom[9] = 1; rows.append(dom)
        if L >= 256:
            flat = np.full(256, L // 256, np.uint32); rows.append(flat)
        for _ in range(12):
            k = int(rng.integers(1, min(L, 256) + 1))
            counts = np.zeros(256, np.uint64)
            counts[rng.choice(256, size=k, replace=False)] = rng.integers(1, 1000, size=k).astype(np.uint64) ** int(rng.integers(1, 4))
            rows.append(B.normalize_freqs(counts, R))
        freqs = np.stack(rows)
        want = B.build_tables_host(freqs, R)
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        got = B.build_tables_device(torch.from_numpy(freqs.astype(np.int32)).cuda(), R, status)
        assert np.array_equal(got.cpu().numpy().view(np.uint32).reshape(want.shape), want), f"table_log {R}"
        assert status.cpu().tolist() == [0, 0]
    # not normalised: zeros and a status bit, the other tables of the call are unaffected
    bad = np.stack([B.normalize_freqs(np.arange(256, dtype=np.uint64) + 1, 10)] * 3)
    bad[1, 0] += 1
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    got = B.build_tables_device(torch.from_numpy(bad.astype(np.int32)).cuda(), 10, status).cpu().numpy().view(np.uint32).reshape(3, -1)
    want = B.build_tables_host(bad[[0, 2]], 10)
    assert np.array_equal(got[[0, 2]], want) and not got[1].any()
    assert status.cpu().tolist() == [B.ST_BAD_FREQ, 1]
    # decode with device-built tables
    w = W.config2()
    c = oracle_encode(orc, w)
    _, expect = oracle_expected(orc, c, w)
    h = host_from_oracle(c, w)
    d = B.to_device(h)
    d.tables = B.build_tables_device(torch.from_numpy(np.ascontiguousarray(h.freqs).astype(np.int32)).cuda(), h.table_log)
    out = B.decode(d)
    assert d.read_status() == (0, 0)
    assert np.array_equal(B.bits_of(out)[:w.numel], expect)


@pytest.mark.parametrize("p0", [0.7, 0.3])
def test_corruption_is_flagged_not_fatal(orc, p0):
    """Damaged inputs set status bits; nothing is read or written outside the buffers.  With p0 = 0.3 no state
    reads zero bits, and the streaming kernel works with its loading wavefronts."""
    import torch
    w = W.tiny(n=50000, chunk_size=4096, table_log=10, p0=p0)
    c = oracle_encode(orc, w)
    good = host_from_oracle(c, w)

    def status_of(h):
        worst = (0, 0)
        for variant in (B.VARIANT_STEPWISE, B.VARIANT_MERGED, B.VARIANT_STEPWISE_SHARED, B.VARIANT_STREAMING):
            d = B.to_device(h)
            guard = torch.full((w.numel + 4096,), 0x5A5A, dtype=torch.int16, device="cuda").view(torch.bfloat16)
            B.decode_raw(B.decode_args(d, guard), d.device, variant)
            st = d.read_status()
            assert bool((guard[w.numel:].view(torch.int16) == 0x5A5A).all()), "wrote past the output"
            if variant == B.VARIANT_STEPWISE:
                worst = st
            else:
                assert (st[0] != 0) == (worst[0] != 0), f"variants disagree: {worst} vs {st}"
        return worst

    assert status_of(good) == (0, 0)
    import copy
    h = copy.deepcopy(good); h.payload[len(h.payload) // 2] ^= np.uint32(0x10)
    assert status_of(h)[0] & (B.ST_BAD_STATE | B.ST_BAD_LENGTH)
    h = copy.deepcopy(good); h.stream_hdr[5] ^= np.uint32(1)
    assert status_of(h)[0] & (B.ST_BAD_STATE | B.ST_BAD_LENGTH)
    h = copy.deepcopy(good); h.stream_hdr[7] += np.uint32(1 << 16)
    assert status_of(h)[0] != 0
    h = copy.deepcopy(good); h.payload = h.payload[: len(h.payload) // 2].copy()
    assert status_of(h)[0] & B.ST_BAD_DESC
    h = copy.deepcopy(good); h.chunks["out_offset"][3] = w.numel
    assert status_of(h)[0] & B.ST_BAD_DESC
    h = copy.deepcopy(good); h.chunks["layer_id"][0] = 9
    assert status_of(h)[0] & B.ST_BAD_DESC
    h = copy.deepcopy(good); h.chunks["stream_offset"][-1] = len(h.stream_hdr)
    assert status_of(h)[0] & B.ST_BAD_DESC
    h = copy.deepcopy(good); h.chunks["n_symbols"][2] += 1
    st = status_of(h)
    assert st[0] != 0 and st[1] >= 1
