"""ctypes front end of the CPU oracle (ans_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports this package and
this package never imports the GPU library.  It marshals numpy arrays into the
C functions and stitches per-layer results into one container; all arithmetic
of the method lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ans_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None

E_CORRUPT = -5


def build(force: bool = True) -> str:
    """Compile ans_oracle.c with gcc into liborc.so (plain -O2, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra",
                               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm", "-lpthread"])
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=True)
        _lib = C.CDLL(_LIB)
        _lib.orc_encode_stream.restype = C.c_int64
        _lib.orc_encode_layer.restype = C.c_int64
        _lib.orc_entropy_bits.restype = C.c_double
        _lib.orc_cross_entropy_bits.restype = C.c_double
    return _lib


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def normalize(counts: np.ndarray, R: int) -> np.ndarray:
    c = np.zeros(256, dtype=np.uint64)
    c[:len(counts)] = counts
    f = np.zeros(256, dtype=np.uint32)
    rc = lib().orc_normalize(_p(c, C.c_uint64), C.c_int(R), _p(f, C.c_uint32))
    if rc:
        raise ValueError(f"orc_normalize failed: {rc}")
    return f


def _f256(f):
    out = np.zeros(256, dtype=np.uint32)
    out[:len(f)] = f
    return out


def spread(f: np.ndarray, R: int) -> np.ndarray:
    f = _f256(f)
    out = np.zeros(1 << R, dtype=np.uint8)
    rc = lib().orc_spread(_p(f, C.c_uint32), C.c_int(R), _p(out, C.c_uint8))
    if rc:
        raise ValueError(f"orc_spread failed: {rc}")
    return out


def decode_table(f: np.ndarray, R: int):
    """(sym[L] u8, nb[L] u8, newX[L] u16): the three fields of Sec. II-A's table."""
    f = _f256(f)
    L = 1 << R
    sym = np.zeros(L, dtype=np.uint8)
    nb = np.zeros(L, dtype=np.uint8)
    newX = np.zeros(L, dtype=np.uint16)
    rc = lib().orc_build_decode_table(_p(f, C.c_uint32), C.c_int(R), _p(sym, C.c_uint8),
                                      _p(nb, C.c_uint8), _p(newX, C.c_uint16))
    if rc:
        raise ValueError(f"orc_build_decode_table failed: {rc}")
    return sym, nb, newX


def decode_table_bytes(f: np.ndarray, R: int) -> np.ndarray:
    f = _f256(f)
    lut = np.zeros(3 << R, dtype=np.uint8)
    n = lib().orc_build_decode_table_bytes(_p(f, C.c_uint32), C.c_int(R), _p(lut, C.c_uint8))
    if n < 0:
        raise ValueError(f"orc_build_decode_table_bytes failed: {n}")
    return lut[:n]


def encode_map(f: np.ndarray, R: int):
    f = _f256(f)
    enc = np.zeros(1 << R, dtype=np.uint16)
    base = np.zeros(256, dtype=np.uint32)
    rc = lib().orc_build_encode_map(_p(f, C.c_uint32), C.c_int(R), _p(enc, C.c_uint16), _p(base, C.c_uint32))
    if rc:
        raise ValueError(f"orc_build_encode_map failed: {rc}")
    return enc, base


def encode_stream(symbols: np.ndarray, f: np.ndarray, R: int):
    """Encode one stream; returns (words u32[], initial decoder state)."""
    symbols = _u8(symbols)
    f = _f256(f)
    enc, base = encode_map(f, R)
    cap = (len(symbols) * R + 31) // 32 + 1
    words = np.zeros(cap, dtype=np.uint32)
    x0 = C.c_uint16(0)
    n = lib().orc_encode_stream(_p(symbols, C.c_uint8), C.c_uint64(0), C.c_uint64(1),
                                C.c_uint64(len(symbols)), _p(f, C.c_uint32), C.c_int(R),
                                _p(enc, C.c_uint16), _p(base, C.c_uint32),
                                _p(words, C.c_uint32), C.c_uint64(cap), C.byref(x0))
    if n < 0:
        raise ValueError(f"orc_encode_stream failed: {n}")
    return words[:n].copy(), int(x0.value)


def decode_stream(words: np.ndarray, init_state: int, count: int, f: np.ndarray, R: int):
    """Decode one stream; returns (symbols, rc, bits_read)."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    wbuf = words if len(words) else np.zeros(1, dtype=np.uint32)
    sym, nb, newX = decode_table(f, R)
    out = np.zeros(max(count, 1), dtype=np.uint8)
    bits = C.c_uint64(0)
    rc = lib().orc_decode_stream(_p(wbuf, C.c_uint32), C.c_uint64(len(words)), C.c_uint16(init_state),
                                 C.c_uint64(count), C.c_int(R), _p(sym, C.c_uint8), _p(nb, C.c_uint8),
                                 _p(newX, C.c_uint16), _p(out, C.c_uint8), C.c_uint64(0), C.c_uint64(1),
                                 C.byref(bits))
    return out[:count], rc, int(bits.value)


@dataclass
class Container:
    """A compressed multi-layer weight set as plain arrays (see ans_oracle.c, 'Layer container')."""
    R: int
    N: int
    chunk_size: int
    freqs: np.ndarray                 # [n_layers, 256] u32, each row sums to 2^R
    layer_numel: np.ndarray           # [n_layers] u64
    layer_out_base: np.ndarray        # [n_layers] u64
    chunk_layer: np.ndarray           # [n_chunks] u32
    chunk_nsym: np.ndarray            # [n_chunks] u32
    chunk_out_off: np.ndarray         # [n_chunks] u64 (element index in the flat output)
    chunk_payload_off: np.ndarray     # [n_chunks] u64 (32-bit words)
    chunk_payload_words: np.ndarray   # [n_chunks] u32
    chunk_stream_off: np.ndarray      # [n_chunks] u32
    stream_hdr: np.ndarray            # [n_chunks * N] u32
    payload: np.ndarray               # u32 words

    @property
    def n_chunks(self) -> int:
        return len(self.chunk_layer)

    @property
    def numel(self) -> int:
        return int(self.layer_numel.sum())

    def compressed_bits(self) -> int:
        """Payload words actually owned by streams, plus one 32-bit header per stream."""
        return int(self.chunk_payload_words.astype(np.uint64).sum()) * 32 + 32 * len(self.stream_hdr)


def encode_layer(symbols: np.ndarray, f: np.ndarray, R: int, N: int, chunk_size: int):
    symbols = _u8(symbols)
    f = _f256(f)
    n = len(symbols)
    n_chunks = (n + chunk_size - 1) // chunk_size
    cap = (n * R + 31) // 32 + n_chunks * (N + 4) + 8
    nsym = np.zeros(n_chunks, dtype=np.uint32)
    poff = np.zeros(n_chunks, dtype=np.uint64)
    pwords = np.zeros(n_chunks, dtype=np.uint32)
    hdr = np.zeros(n_chunks * N, dtype=np.uint32)
    payload = np.zeros(cap, dtype=np.uint32)
    used = lib().orc_encode_layer(_p(symbols, C.c_uint8), C.c_uint64(n), _p(f, C.c_uint32), C.c_int(R),
                                  C.c_uint32(N), C.c_uint32(chunk_size), _p(nsym, C.c_uint32),
                                  _p(poff, C.c_uint64), _p(pwords, C.c_uint32), _p(hdr, C.c_uint32),
                                  _p(payload, C.c_uint32), C.c_uint64(cap))
    if used < 0:
        raise ValueError(f"orc_encode_layer failed: {used}")
    return nsym, poff, pwords, hdr, payload[:used].copy()


def encode_layers(layer_symbols: Sequence[np.ndarray], R: int, N: int, chunk_size,
                  freqs: Sequence[np.ndarray] | None = None) -> Container:
    """Histogram + normalise each layer (unless freqs are given), encode, and concatenate.  chunk_size: one
    number for all layers, or one per layer."""
    sizes = [int(chunk_size)] * len(layer_symbols) if np.isscalar(chunk_size) else [int(v) for v in chunk_size]
    fr, c_layer, c_nsym, c_out, c_poff, c_pw, c_soff, hdrs, pays = [], [], [], [], [], [], [], [], []
    numel, out_base = [], []
    elem = 0
    words = 0
    streams = 0
    for li, sym in enumerate(layer_symbols):
        sym = _u8(sym)
        if freqs is None:
            f = normalize(np.bincount(sym, minlength=256).astype(np.uint64), R)
        else:
            f = _f256(freqs[li])
        nsym, poff, pw, hdr, pay = encode_layer(sym, f, R, N, sizes[li])
        nc = len(nsym)
        fr.append(f)
        numel.append(len(sym))
        out_base.append(elem)
        c_layer.append(np.full(nc, li, dtype=np.uint32))
        c_nsym.append(nsym)
        c_out.append(elem + np.arange(nc, dtype=np.uint64) * np.uint64(sizes[li]))
        c_poff.append(poff + np.uint64(words))
        c_pw.append(pw)
        c_soff.append((streams + np.arange(nc, dtype=np.uint64) * N).astype(np.uint32))
        hdrs.append(hdr)
        pays.append(pay)
        elem += len(sym)
        words += len(pay)
        streams += nc * N
    cat = np.concatenate
    return Container(R, N, max(sizes) if sizes else 0, np.stack(fr).astype(np.uint32),
                     np.array(numel, dtype=np.uint64), np.array(out_base, dtype=np.uint64),
                     cat(c_layer), cat(c_nsym), cat(c_out).astype(np.uint64), cat(c_poff).astype(np.uint64),
                     cat(c_pw), cat(c_soff), cat(hdrs), cat(pays) if words else np.zeros(0, np.uint32))


def tables_for(container: Container):
    L = 1 << container.R
    nl = len(container.freqs)
    tsym = np.zeros(nl * L, dtype=np.uint8)
    tnb = np.zeros(nl * L, dtype=np.uint8)
    tnx = np.zeros(nl * L, dtype=np.uint16)
    for li in range(nl):
        s, n, x = decode_table(container.freqs[li], container.R)
        tsym[li * L:(li + 1) * L] = s
        tnb[li * L:(li + 1) * L] = n
        tnx[li * L:(li + 1) * L] = x
    return tsym, tnb, tnx


def decode_dequant(container: Container, zero_points, scales, channel_len=None, channel_scales=None,
                   out_dtype: str = "bf16", n_threads: int = 1, tables=None):
    """Decode every chunk and dequantise.  Returns (symbols u8, weights, rc).

    weights is float32 for out_dtype "f32", uint16 bit patterns for "bf16",
    None for "u8".  channel_scales: list (per layer) of float32 arrays or None.
    """
    c = container
    nl = len(c.freqs)
    tsym, tnb, tnx = tables if tables is not None else tables_for(c)
    z = np.ascontiguousarray(zero_points, dtype=np.uint32)
    sc = np.ascontiguousarray(scales, dtype=np.float32)
    cl = np.zeros(nl, dtype=np.uint32) if channel_len is None else np.ascontiguousarray(channel_len, dtype=np.uint32)
    soff = np.zeros(nl, dtype=np.uint64)
    flat = [np.zeros(1, dtype=np.float32)]
    acc = 0
    if channel_scales is not None:
        flat = []
        for li in range(nl):
            soff[li] = acc
            if channel_scales[li] is not None:
                a = np.ascontiguousarray(channel_scales[li], dtype=np.float32)
                flat.append(a)
                acc += len(a)
        if not flat:
            flat = [np.zeros(1, dtype=np.float32)]
    all_scales = np.concatenate(flat)
    n = c.numel
    out_sym = np.zeros(max(n, 1), dtype=np.uint8)
    code = {"u8": 0, "f32": 1, "bf16": 2}[out_dtype]
    out = {0: np.zeros(1, np.uint8), 1: np.zeros(max(n, 1), np.float32), 2: np.zeros(max(n, 1), np.uint16)}[code]
    payload = c.payload if len(c.payload) else np.zeros(1, np.uint32)
    rc = lib().orc_decode_dequant(
        C.c_uint64(c.n_chunks), _p(c.chunk_layer, C.c_uint32), _p(c.chunk_nsym, C.c_uint32),
        _p(c.chunk_out_off, C.c_uint64), _p(c.chunk_payload_off, C.c_uint64), _p(c.chunk_stream_off, C.c_uint32),
        _p(c.stream_hdr, C.c_uint32), _p(payload, C.c_uint32), C.c_uint64(len(c.payload)), C.c_int(c.R), C.c_uint32(c.N),
        _p(tsym, C.c_uint8), _p(tnb, C.c_uint8), _p(tnx, C.c_uint16),
        _p(z, C.c_uint32), _p(sc, C.c_float), _p(cl, C.c_uint32), _p(soff, C.c_uint64),
        _p(c.layer_out_base, C.c_uint64), _p(all_scales, C.c_float),
        _p(out_sym, C.c_uint8), out.ctypes.data_as(C.c_void_p), C.c_int(code), C.c_int(n_threads))
    return out_sym[:n], (None if code == 0 else out[:n]), rc


def dequant(symbols: np.ndarray, zero_point: int, scale: float, out_dtype: str = "bf16",
            channel_len: int = 0, channel_scales: np.ndarray | None = None) -> np.ndarray:
    q = _u8(symbols)
    n = len(q)
    cs = np.ascontiguousarray(channel_scales if channel_scales is not None else np.zeros(1), dtype=np.float32)
    if out_dtype == "f32":
        out = np.zeros(n, dtype=np.float32)
        lib().orc_dequant_f32(_p(q, C.c_uint8), C.c_uint64(0), C.c_uint64(n), C.c_uint64(0),
                              C.c_uint32(zero_point), C.c_float(scale), C.c_uint32(channel_len),
                              _p(cs, C.c_float), C.c_uint64(0), _p(out, C.c_float))
    else:
        out = np.zeros(n, dtype=np.uint16)
        lib().orc_dequant_bf16(_p(q, C.c_uint8), C.c_uint64(0), C.c_uint64(n), C.c_uint64(0),
                               C.c_uint32(zero_point), C.c_float(scale), C.c_uint32(channel_len),
                               _p(cs, C.c_float), C.c_uint64(0), _p(out, C.c_uint16))
    return out


def entropy_bits(counts: np.ndarray) -> float:
    c = np.zeros(256, dtype=np.uint64)
    c[:len(counts)] = counts
    return float(lib().orc_entropy_bits(_p(c, C.c_uint64)))


def cross_entropy_bits(counts: np.ndarray, f: np.ndarray, R: int) -> float:
    c = np.zeros(256, dtype=np.uint64)
    c[:len(counts)] = counts
    f = _f256(f)
    return float(lib().orc_cross_entropy_bits(_p(c, C.c_uint64), _p(f, C.c_uint32), C.c_int(R)))
