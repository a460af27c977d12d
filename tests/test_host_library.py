"""CPU-side checks of libanszp: the ABI surface and the host entry points (no GPU calls).

The library's table builder and packer are written independently of the oracle; both follow
the same container definition, so their outputs must agree bit for bit.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2406_06237_amd import binding as B
from paper_2406_06237_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "anszp.h")).read()
    declared = sorted(set(re.findall(r"\b(anszp_[a-z_0-9]+)\s*\(", header)))
    assert declared == sorted(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.version() == 100
    assert B.strerror(0) == "ok" and "range" in B.strerror(-2)


def test_struct_layouts_match_header():
    # sizes and offsets as the C compiler lays the header's structs out
    src = ('#include <stdio.h>\n#include <stddef.h>\n#include "anszp.h"\nint main(void){printf("%zu %zu %zu %zu %zu %zu\\n",'
           'sizeof(anszp_decode_args_t), offsetof(anszp_decode_args_t, status), offsetof(anszp_decode_args_t, out),'
           'sizeof(anszp_chunk_t), sizeof(anszp_layer_t), offsetof(anszp_decode_args_t, chunks));return 0;}')
    import subprocess, tempfile
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(src)
        subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", os.path.join(d, "t"), os.path.join(d, "t.c")])
        got = [int(v) for v in subprocess.check_output([os.path.join(d, "t")]).split()]
    assert got == [C.sizeof(B.DecodeArgs), B.DecodeArgs.status.offset, B.DecodeArgs.out.offset,
                   B.CHUNK_DTYPE.itemsize, B.LAYER_DTYPE.itemsize, B.DecodeArgs.chunks.offset]
    assert B.CHUNK_DTYPE.fields["out_offset"][1] == 8 and B.CHUNK_DTYPE.fields["payload_words"][1] == 24
    assert B.LAYER_DTYPE.fields["scales_offset"][1] == 16 and B.LAYER_DTYPE.fields["out_base"][1] == 24


def _random_freqs(rng, R, max_syms=40):
    L = 1 << R
    A = int(rng.integers(1, min(L, max_syms) + 1))
    cuts = np.sort(rng.choice(np.arange(1, L), size=A - 1, replace=False)) if A > 1 else np.array([], int)
    f = np.zeros(256, dtype=np.uint32)
    f[np.sort(rng.choice(256, size=A, replace=False))] = np.diff(np.concatenate(([0], cuts, [L])))
    return f


@pytest.mark.parametrize("R", [1, 2, 5, 8, 10, 11, 12])
def test_tables_equal_oracle_tables(orc, R):
    rng = np.random.default_rng(100 + R)
    rows = [_random_freqs(rng, R) for _ in range(6)]
    L = 1 << R
    peaked = np.zeros(256, dtype=np.uint32)
    peaked[9] = L - min(3, L - 1)
    rest = L - int(peaked[9])
    for i in range(rest):
        peaked[10 + i] = 1
    rows.append(peaked)
    single = np.zeros(256, dtype=np.uint32)
    single[200] = L
    rows.append(single)
    tables = B.build_tables_host(np.stack(rows), R)
    for row, t in zip(rows, tables):
        f = B.split_table(t)
        sym, nb, newX = orc.decode_table(row, R)
        assert np.array_equal(f["sym"], sym) and np.array_equal(f["nb"], nb) and np.array_equal(f["newX"], newX)
        # the three-bytes-per-state table of Sec. II-A, for tables it can hold (at most 256 states)
        if L <= 256:
            assert np.array_equal(f["bytes"], orc.decode_table_bytes(row, R))
        else:
            assert not f["bytes"].any()


def _lookahead_decode(t, words, x0, n, dominant):
    """Decode n symbols with the look-ahead entries only (pure Python), returning symbols, symbols emitted,
    bits consumed, the last index, and whether the last look-up started in an entry marked as state 0."""
    bits = int.from_bytes(np.asarray(words, dtype=np.uint32).tobytes(), "little")

    def peek(pos, k):                                   # next k stream bits, first bit on top
        v = 0
        for i in range(k):
            v = (v << 1) | ((bits >> (pos + i)) & 1)
        return v

    pos, out = 0, []
    idx = 2 * x0 + peek(0, 1)
    while len(out) < n:
        T, c = int(t["la_bits"][idx]), int(t["la_count"][idx])
        assert int(t["la_state0"][idx]) == (1 if idx >> 1 == 0 else 0)
        out.extend([dominant] * (c - 1))
        out.append(int(t["la_sym"][idx]))
        idx = int(t["la_base"][idx]) + peek(pos, T + 1)
        pos += T
        assert 0 <= idx < len(t["la_bits"])
    return np.array(out[:n], dtype=np.uint8), len(out), pos, idx


@pytest.mark.parametrize("R", [2, 3, 6, 8, 11, 12])
def test_lookahead_entries_decode_what_the_oracle_encodes(orc, R):
    """The look-ahead half of a table is the paper's automaton with steps merged: decoding oracle-encoded
    streams with it alone must give back the symbols, read exactly the stream's bits and end in state 0."""
    L = 1 << R
    rng = np.random.default_rng(40 + R)
    cases = []
    for p0 in (0.3, 0.55, 0.7, 0.76, 0.9, 0.97):
        A = int(rng.integers(2, min(L, 40) + 1))
        pmf = W.peaked_geometric_pmf(A, A // 2, p0)
        cases.append(pmf)
    cases.append(np.eye(1, 5, 2)[0])                    # single symbol
    for pmf in cases:
        n = 3000
        sym = W.sample_symbols(pmf, n, int(rng.integers(1 << 30)))
        f = orc.normalize(np.bincount(sym, minlength=256), R)
        t = B.split_table(B.build_tables_host(f[None, :], R)[0])
        assert np.all(t["la_pad"] == 0) and np.all(t["zero"] == 0) and np.all(t["la_base_rem"] == 0)
        assert int(t["la_bits"].max()) <= 12 and int(t["la_count"].max()) <= 8
        assert np.array_equal(t["la_shift"], 31 - t["la_bits"]) and np.array_equal(t["la_count_low"], t["la_count"])
        dominant = int(np.argmax(f)) if f.max() > L // 2 else 255
        for length in (n, 1, 2, 7, 100):
            words, x0 = orc.encode_stream(sym[:length], f, R)
            out, emitted, pos, idx = _lookahead_decode(t, words, x0, length, dominant)
            assert np.array_equal(out, sym[:length])
            # an entry never passes through state 0, so every stream ends where an entry ends
            assert emitted == length
            _, _, total = orc.decode_stream(words, x0, length, f, R)
            assert pos == total and idx >> 1 == 0
        # entries with and without look-ahead agree when there is no dominant symbol
        if f.max() <= L // 2:
            assert np.all(t["la_count"] == 1)
            la = B.build_tables_host(f[None, :], R)[0][4 * L:8 * L].reshape(L, 2, 2)
            assert np.array_equal(la[1:, 0], la[1:, 1])
            assert np.array_equal(t["la_bits"].reshape(L, 2)[:, 0], t["nb"])
            assert np.array_equal(t["la_sym"].reshape(L, 2)[:, 0], t["sym"])
            assert np.array_equal(t["la_base"].reshape(L, 2)[:, 0], 2 * t["newX"].astype(np.int32))


def test_normalize_equals_oracle(orc):
    rng = np.random.default_rng(5)
    for R in (4, 8, 10, 12):
        for _ in range(25):
            A = int(rng.integers(1, min(1 << R, 256) + 1))
            counts = np.zeros(256, dtype=np.uint64)
            counts[rng.choice(256, size=A, replace=False)] = rng.integers(1, 10 ** int(rng.integers(1, 9)), size=A)
            assert np.array_equal(B.normalize_freqs(counts, R), orc.normalize(counts, R))
    with pytest.raises(B.AnszpError):
        B.normalize_freqs(np.zeros(256, dtype=np.uint64), 8)
    with pytest.raises(B.AnszpError):
        B.normalize_freqs(np.ones(256, dtype=np.uint64), 13)


@pytest.mark.parametrize("N,chunk,n,R", [(1, 36864, 36864, 10), (32, 16384, 50000, 11), (64, 65536, 140001, 12),
                                          (64, 1024, 37, 6), (5, 333, 4000, 9), (64, 4096, 0, 8)])
def test_packer_equals_oracle_encoder(orc, N, chunk, n, R):
    w = W.tiny(seed=n + N, n=max(n, 1), bitwidth=5, p0=0.83)
    sym = w.layers[0].symbols()[:n]
    if n == 0:
        h = B.pack_layers([sym], R, N, chunk, [16], [0.1], freqs=[np.eye(1, 256, 3, dtype=np.uint32)[0] << R])
        assert len(h.chunks) == 0 and len(h.payload) == 0
        return
    h = B.pack_layers([sym, sym[::-1].copy()], R, N, chunk, [16, 16], [0.1, 0.2])
    c = orc.encode_layers([sym, sym[::-1].copy()], R, N, chunk)
    assert np.array_equal(h.freqs, c.freqs)
    assert np.array_equal(h.stream_hdr, c.stream_hdr)
    assert np.array_equal(h.payload, c.payload)
    assert np.array_equal(h.chunks["layer_id"], c.chunk_layer)
    assert np.array_equal(h.chunks["n_symbols"], c.chunk_nsym)
    assert np.array_equal(h.chunks["out_offset"], c.chunk_out_off)
    assert np.array_equal(h.chunks["payload_offset"], c.chunk_payload_off)
    assert np.array_equal(h.chunks["payload_words"], c.chunk_payload_words)
    assert np.array_equal(h.chunks["stream_offset"], c.chunk_stream_off)
    assert np.array_equal(h.layers["out_base"], c.layer_out_base)


def test_host_error_codes():
    lib = B.lib()
    f = np.zeros(256, dtype=np.uint32)
    f[0] = 255
    t = np.zeros(B.table_words(1, 8), dtype=np.uint32)
    assert lib.anszp_build_tables_host(f.ctypes.data, 1, 8, t.ctypes.data) == -3          # sum != 2^R
    f[0] = 256
    assert lib.anszp_build_tables_host(f.ctypes.data, 1, 8, t.ctypes.data) == 0
    assert lib.anszp_build_tables_host(f.ctypes.data, 1, 13, t.ctypes.data) == -2
    assert lib.anszp_build_tables_host(None, 1, 8, t.ctypes.data) == -1
    assert lib.anszp_build_tables_host(f.ctypes.data, 0, 8, t.ctypes.data) == -2
    with pytest.raises(B.AnszpError) as e:
        B.pack_layer(np.array([0, 1], dtype=np.uint8), f, 8, 64, 1024)                    # symbol 1 has f = 0
    assert e.value.code == -4
    with pytest.raises(B.AnszpError) as e:
        B.pack_layer(np.array([0], dtype=np.uint8), f, 8, 65, 1024)
    assert e.value.code == -2
    with pytest.raises(B.AnszpError) as e:
        B.pack_layer(np.array([0], dtype=np.uint8), f, 8, 64, 1024, payload_word_offset=2)
    assert e.value.code == -2
    # decode argument validation happens before any GPU call
    a = B.DecodeArgs()
    assert lib.anszp_decode(None, None) == -1
    assert lib.anszp_decode(C.byref(a), None) == 0            # zero chunks: nothing to do
    a.n_chunks = 1
    assert lib.anszp_decode(C.byref(a), None) == -1           # NULL pointers
    lay = np.zeros(1, dtype=B.LAYER_DTYPE)
    assert lib.anszp_dequant_zp(None, 0, lay.ctypes.data, None, 0, None, 3, None) == -2
    assert lib.anszp_dequant_zp(None, 0, lay.ctypes.data, None, 0, None, 1, None) == 0
    assert lib.anszp_dequant_zp(None, 5, lay.ctypes.data, None, 0, None, 1, None) == -1


def test_table_size_study_trend():
    """Sec. III-B on the synthetic odd-bin ResNet-50 (first layers only, for speed): the gap to the entropy
    bound grows as the table shrinks, and parallel streams cost little once only the paper's per-stream
    cost (the final state) is counted."""
    from paper_2406_06237_amd import table_size_study as T
    rows, bound, numel = T.study(states=(64, 128, 256, 4096), max_layers=14)
    single = {st: total for st, g, total, _, _ in rows if g.startswith("single")}
    assert single[64] > single[128] > single[256] > single[4096] >= bound * 0.999
    assert single[4096] < bound * 1.01 and single[256] < bound * 1.12
    for st, g, total, paper_like, streams in rows:
        if not g.startswith("single"):
            assert total > single[st]                                  # framing is not free
            assert paper_like < single[st] * 1.03, (st, g, paper_like / single[st])


def test_stream_grouping_geometries():
    """Sec. III-B grouping (a stream per input channel) against the benchmark's chunks on config 3: about as many
    streams, hence about the same bytes, but streams up to 4.5 times as long."""
    from paper_2406_06237_amd import stream_grouping_study as S
    w, cs = S.containers()
    size = {k: 4 * len(h.payload) + 4 * len(h.stream_hdr) for k, h in cs.items()}
    streams = {k: int(np.count_nonzero(h.stream_hdr >> 16)) for k, h in cs.items()}
    assert sum(int(c) for c in cs["by channel"].chunks["n_symbols"]) == w.numel
    assert abs(size["by channel"] / size["benchmark"] - 1.0) < 0.01
    assert abs(streams["by channel"] / streams["benchmark"] - 1.0) < 0.06
    assert int(cs["by channel"].chunks["n_symbols"].max()) // 64 == 4608
    assert int(cs["benchmark"].chunks["n_symbols"].max()) // 64 == 1024


def test_conv_packing_geometry():
    """Host side of the fused decode + convolution path: chunks follow the rows of the GEMM panels."""
    assert [B.conv_rows_per_chunk(k) for k in (64, 147, 256, 512, 576, 1024, 1152, 2048, 2304, 4608)] == \
           [16, 16, 16, 8, 4, 4, 2, 2, 1, 1]
    for k in (20, 64, 147, 576, 1152, 4608):
        r = B.conv_rows_per_chunk(k)
        assert 16 % r == 0 and (r == 1 or r * k <= 4096)
    shapes = [(32, 16, 3, 3), (16, 64, 1, 1)]
    rng = np.random.default_rng(3)
    syms = [rng.integers(0, 4, size=int(np.prod(s))).astype(np.uint8) for s in shapes]
    h, first, rows = B.pack_conv_layers(syms, shapes, 10, 64, [2, 2], [0.5, 0.25], [2, 2])
    assert rows == [B.conv_rows_per_chunk(144), B.conv_rows_per_chunk(64)]
    assert first == [0, 32 // rows[0]]
    assert len(h.chunks) == 32 // rows[0] + 16 // rows[1]
    assert list(h.chunks["n_symbols"][:first[1]]) == [rows[0] * 144] * first[1]
    assert list(h.chunks["n_symbols"][first[1]:]) == [rows[1] * 64] * (16 // rows[1])
    assert np.all(h.chunks["payload_offset"] % 4 == 0)
    with pytest.raises(ValueError):
        B.pack_conv_layers([syms[0][:-1]], [shapes[0]], 10, 64, [2], [0.5])
    with pytest.raises(ValueError):
        B.pack_conv_layers([np.zeros(24 * 16, np.uint8)], [(24, 16, 1, 1)], 10, 64, [0], [1.0])   # cout not a multiple of 16
    geo = W.resnet50_conv_geometry()
    assert len(geo) == 53 and geo[0][1:] == ((64, 3, 7, 7), 2, 3, 224)
    assert all(co % 64 == 0 and ci * kh * kw <= 4608 for _, (co, ci, kh, kw), _, _, _ in geo)
    macs = sum(co * ci * kh * kw * (((s + 2 * p - kh) // st + 1) ** 2) for _, (co, ci, kh, kw), st, p, s in geo)
    assert macs == 4087136256                                  # multiply-adds per 224 x 224 image
