"""Thin ctypes binding of libanszp.so (declared in include/anszp.h).

Argument marshalling only: every step of the decode path (table staging, tANS decode,
dequantisation, stores) runs in the library's HIP kernels, and the container is built by the
library's host packer.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library is missing or the call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libanszp.so")

OUT_U8, OUT_F32, OUT_BF16 = 0, 1, 2
OUT_CODES = {"u8": OUT_U8, "f32": OUT_F32, "bf16": OUT_BF16}
ST_BAD_DESC, ST_BAD_STATE, ST_BAD_LENGTH, ST_INTERNAL, ST_BAD_FREQ, ST_BAD_SYMBOL, ST_NO_SPACE = 1, 2, 4, 8, 16, 32, 64
MAX_TABLE_LOG, MAX_STREAMS, ALPHABET = 12, 64, 256

CHUNK_DTYPE = np.dtype([("layer_id", "<u4"), ("n_symbols", "<u4"), ("out_offset", "<u8"),
                        ("payload_offset", "<u8"), ("payload_words", "<u4"), ("stream_offset", "<u4")])
LAYER_DTYPE = np.dtype([("scale", "<f4"), ("zero_point", "<u4"), ("bitwidth", "<u4"), ("channel_len", "<u4"),
                        ("scales_offset", "<u8"), ("out_base", "<u8")])
JOB_DTYPE = np.dtype([("first_symbol", "<u8"), ("n_symbols", "<u8"), ("chunk_size", "<u4"), ("first_chunk", "<u4"),
                      ("reserved", "<u4", (2,))])
assert CHUNK_DTYPE.itemsize == 32 and LAYER_DTYPE.itemsize == 32 and JOB_DTYPE.itemsize == 32


class DecodeArgs(C.Structure):
    _fields_ = [("tables", C.c_void_p), ("n_tables", C.c_uint32), ("table_log", C.c_uint32),
                ("n_streams", C.c_uint32), ("out_dtype", C.c_uint32),
                ("chunks", C.c_void_p), ("n_chunks", C.c_uint64),
                ("stream_hdr", C.c_void_p), ("n_stream_hdr", C.c_uint64),
                ("payload", C.c_void_p), ("payload_words", C.c_uint64),
                ("layers", C.c_void_p), ("scales", C.c_void_p), ("n_scales", C.c_uint64),
                ("out", C.c_void_p), ("out_elems", C.c_uint64), ("status", C.c_void_p)]


class ConvArgs(C.Structure):
    _fields_ = [("tables", C.c_void_p), ("n_tables", C.c_uint32), ("table_log", C.c_uint32),
                ("n_streams", C.c_uint32), ("layer_id", C.c_uint32),
                ("chunks", C.c_void_p), ("n_chunks", C.c_uint64),
                ("stream_hdr", C.c_void_p), ("n_stream_hdr", C.c_uint64),
                ("payload", C.c_void_p), ("payload_words", C.c_uint64),
                ("layers", C.c_void_p), ("scales", C.c_void_p), ("n_scales", C.c_uint64),
                ("rows_per_chunk", C.c_uint32), ("batch", C.c_uint32), ("in_h", C.c_uint32), ("in_w", C.c_uint32),
                ("cin", C.c_uint32), ("cout", C.c_uint32), ("kh", C.c_uint32), ("kw", C.c_uint32),
                ("stride", C.c_uint32), ("pad", C.c_uint32),
                ("x", C.c_void_p), ("y", C.c_void_p), ("y_dtype", C.c_uint32), ("x_layout", C.c_uint32),
                ("y_layout", C.c_uint32), ("status", C.c_void_p)]


class AnszpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None
EXPORTS = ["anszp_version", "anszp_strerror", "anszp_normalize_freqs", "anszp_build_tables_host",
           "anszp_build_tables", "anszp_build_tables_device", "anszp_pack_bound", "anszp_pack_layer", "anszp_decode", "anszp_decode_variant",
           "anszp_dequant_zp", "anszp_conv_fused", "anszp_pack_layer_device",
           "anszp_plan_bytes", "anszp_plan_decode", "anszp_decode_planned", "anszp_decode_static_plan",
           "anszp_pack_layers_device", "anszp_test_set_spin_limit"]


def lib():
    """Load libanszp.so (build it first with `python -m paper_2406_06237_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run __graft_entry__.build()")
        # PyTorch brings its own HIP runtime: load it first, so that the library binds to the same
        # one (two runtimes in one process do not share devices, streams or allocations)
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        L.anszp_strerror.restype = C.c_char_p
        L.anszp_strerror.argtypes = [C.c_int]
        L.anszp_normalize_freqs.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
        L.anszp_build_tables_host.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.anszp_build_tables.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.anszp_build_tables_device.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.anszp_pack_bound.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_uint32, C.c_void_p, C.c_void_p]
        L.anszp_pack_layer.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int, C.c_int, C.c_uint32,
                                       C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.anszp_decode.argtypes = [C.POINTER(DecodeArgs), C.c_void_p]
        L.anszp_decode_variant.argtypes = [C.POINTER(DecodeArgs), C.c_int, C.c_void_p]
        L.anszp_plan_bytes.restype = C.c_uint64
        L.anszp_plan_bytes.argtypes = [C.c_uint64]
        L.anszp_plan_decode.argtypes = [C.POINTER(DecodeArgs), C.c_void_p, C.c_uint64, C.c_void_p]
        L.anszp_decode_planned.argtypes = [C.POINTER(DecodeArgs), C.c_void_p, C.c_uint64, C.c_void_p]
        L.anszp_decode_static_plan.argtypes = [C.POINTER(DecodeArgs), C.c_int, C.c_void_p]
        L.anszp_dequant_zp.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint64,
                                       C.c_void_p, C.c_int, C.c_void_p]
        L.anszp_conv_fused.argtypes = [C.POINTER(ConvArgs), C.c_void_p]
        L.anszp_pack_layer_device.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int, C.c_int, C.c_uint32, C.c_uint32,
                                              C.c_uint64, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.anszp_pack_layers_device.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_int, C.c_int,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.anszp_test_set_spin_limit.argtypes = [C.c_uint32]
        L.anszp_test_set_spin_limit.restype = None
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().anszp_strerror(code).decode()


def _check(rc: int, where: str):
    if rc != 0:
        raise AnszpError(rc, where)


def version() -> int:
    return lib().anszp_version()


# ----------------------------------------------------------------------------- host entry points
def normalize_freqs(counts: np.ndarray, table_log: int) -> np.ndarray:
    c = np.zeros(ALPHABET, dtype=np.uint64)
    c[:len(counts)] = counts
    f = np.zeros(ALPHABET, dtype=np.uint32)
    _check(lib().anszp_normalize_freqs(c.ctypes.data, table_log, f.ctypes.data), "anszp_normalize_freqs")
    return f


TABLE_WORDS_PER_STATE = 8     # a table of L states occupies 8 L words (see anszp.h)


def table_words(n_tables: int, table_log: int) -> int:
    return (n_tables * TABLE_WORDS_PER_STATE) << table_log


def build_tables_host(freqs: np.ndarray, table_log: int) -> np.ndarray:
    freqs = np.ascontiguousarray(freqs, dtype=np.uint32).reshape(-1, ALPHABET)
    tables = np.zeros(table_words(len(freqs), max(0, min(table_log, 20))), dtype=np.uint32)
    _check(lib().anszp_build_tables_host(freqs.ctypes.data, len(freqs), table_log, tables.ctypes.data),
           "anszp_build_tables_host")
    return tables.reshape(len(freqs), -1)


def split_table(tables: np.ndarray):
    """Fields of a table (or stack of tables): the byte table (tables of at most 256 states), the paper's
    triple per state and the look-ahead entries."""
    t = np.asarray(tables, dtype=np.uint32)
    L = t.shape[-1] // TABLE_WORDS_PER_STATE
    lo = t[..., 2 * L:3 * L]
    la = t[..., 4 * L:8 * L]
    first, second = la[..., 0::2], la[..., 1::2]
    base8 = second.astype(np.int32)
    return {"newX": (lo & 0xFFFF).astype(np.uint16), "nb": ((lo >> 16) & 0xFF).astype(np.uint8),
            "sym": (lo >> 24).astype(np.uint8),
            "bytes": np.ascontiguousarray(t[..., :L]).view(np.uint8)[..., :3 * L],
            "la_bits": ((first >> 24) & 15).astype(np.uint8), "la_shift": (first & 31).astype(np.uint8),
            "la_pad": (((first >> 5) & 15) | (((first >> 12) & 15) << 4)).astype(np.uint8),
            "la_sym": ((first >> 16) & 0xFF).astype(np.uint8), "la_count": (((first >> 28) & 7) + 1).astype(np.uint8),
            "la_count_low": (((first >> 9) & 7) + 1).astype(np.uint8), "la_state0": (first >> 31).astype(np.uint8),
            "la_base": base8 // 8, "la_base_rem": base8 % 8,
            "zero": np.concatenate([t[..., L:2 * L], t[..., 3 * L:4 * L]], axis=-1)}


@dataclass
class HostContainer:
    table_log: int
    n_streams: int
    chunk_size: int
    out_dtype: str
    freqs: np.ndarray        # [n_layers, 256] u32
    layers: np.ndarray       # LAYER_DTYPE [n_layers]
    chunks: np.ndarray       # CHUNK_DTYPE [n_chunks]
    stream_hdr: np.ndarray   # u32
    payload: np.ndarray      # u32
    scales: np.ndarray       # f32 (per-channel scales of all layers, possibly empty)
    numel: int

    def compressed_bytes(self) -> int:
        """Bytes a decode has to read: stream words, stream headers."""
        return int(self.chunks["payload_words"].astype(np.uint64).sum()) * 4 + 4 * len(self.stream_hdr)


def pack_layer(symbols: np.ndarray, freqs: np.ndarray, table_log: int, n_streams: int, chunk_size: int,
               layer_id: int = 0, out_offset: int = 0, payload_word_offset: int = 0, stream_offset: int = 0):
    sym = np.ascontiguousarray(symbols, dtype=np.uint8)
    f = np.zeros(ALPHABET, dtype=np.uint32)
    f[:len(freqs)] = freqs
    nc, cap = C.c_uint64(0), C.c_uint64(0)
    _check(lib().anszp_pack_bound(len(sym), table_log, n_streams, chunk_size, C.addressof(nc), C.addressof(cap)),
           "anszp_pack_bound")
    chunks = np.zeros(nc.value, dtype=CHUNK_DTYPE)
    hdr = np.zeros(nc.value * n_streams, dtype=np.uint32)
    payload = np.zeros(cap.value + 4, dtype=np.uint32)
    used = C.c_uint64(0)
    _check(lib().anszp_pack_layer(sym.ctypes.data, len(sym), f.ctypes.data, table_log, n_streams, chunk_size,
                                  layer_id, out_offset, payload_word_offset, stream_offset,
                                  chunks.ctypes.data, hdr.ctypes.data, payload.ctypes.data, len(payload),
                                  C.addressof(used)), "anszp_pack_layer")
    return chunks, hdr, payload[:used.value].copy()


def pack_layers(layer_symbols: Sequence[np.ndarray], table_log: int, n_streams: int, chunk_size: int,
                zero_points: Sequence[int], scales: Sequence[float], bitwidths: Optional[Sequence[int]] = None,
                channel_len: Optional[Sequence[int]] = None,
                channel_scales: Optional[Sequence[Optional[np.ndarray]]] = None,
                out_dtype: str = "bf16", freqs: Optional[Sequence[np.ndarray]] = None,
                chunk_sizes: Optional[Sequence[int]] = None) -> HostContainer:
    """Compress a list of layers into one container with the library's host packer (chunk_sizes: one chunk
    size per layer instead of chunk_size for all)."""
    nl = len(layer_symbols)
    layers = np.zeros(nl, dtype=LAYER_DTYPE)
    fr, ch, hd, pl, sc = [], [], [], [], []
    elem = words = streams = n_sc = 0
    for li, sym in enumerate(layer_symbols):
        sym = np.ascontiguousarray(sym, dtype=np.uint8)
        f = (normalize_freqs(np.bincount(sym, minlength=ALPHABET), table_log) if freqs is None
             else np.ascontiguousarray(freqs[li], dtype=np.uint32))
        chunks, hdr, payload = pack_layer(sym, f, table_log, n_streams, chunk_sizes[li] if chunk_sizes is not None else chunk_size,
                                          li, elem, words, streams)
        layers[li] = (scales[li], zero_points[li], bitwidths[li] if bitwidths is not None else 8,
                      channel_len[li] if channel_len is not None else 0, n_sc, elem)
        if channel_len is not None and channel_len[li]:
            cs = np.ascontiguousarray(channel_scales[li], dtype=np.float32)
            sc.append(cs)
            n_sc += len(cs)
        fr.append(f); ch.append(chunks); hd.append(hdr); pl.append(payload)
        elem += len(sym); words += len(payload); streams += len(hdr)
    cat = np.concatenate
    return HostContainer(table_log, n_streams, chunk_size, out_dtype, np.stack(fr), layers, cat(ch), cat(hd),
                         cat(pl) if words else np.zeros(0, np.uint32),
                         cat(sc) if sc else np.zeros(0, np.float32), elem)


def pack_workload(w) -> HostContainer:
    """Compress a workloads.Workload."""
    L = w.layers
    return pack_layers(w.symbols(), w.table_log, w.n_streams, w.chunk_size,
                       [l.zero_point for l in L], [l.scale for l in L], [l.bitwidth for l in L],
                       [l.channel_len for l in L], [l.channel_scales for l in L], w.out_dtype,
                       chunk_sizes=getattr(w, "chunk_sizes", None))


# --------------------------------------------------------------------------- device entry points
def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("libanszp device entry points need a GPU (torch.cuda.is_available() is False)")
    return torch


def _dev(arr: np.ndarray, device):
    """Copy a numpy array to the device as raw bytes (at least 16 bytes so the pointer is valid)."""
    torch = _torch()
    raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
    if raw.size < 16:
        raw = np.concatenate([raw, np.zeros(16 - raw.size, np.uint8)])
    return torch.from_numpy(raw.copy()).to(device)


def _stream_ptr(torch, device):
    return C.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def build_tables(freqs: np.ndarray, table_log: int, device="cuda:0"):
    """anszp_build_tables into a new device tensor (uint8 view of n_tables * 8 * 2^table_log uint32)."""
    torch = _torch()
    freqs = np.ascontiguousarray(freqs, dtype=np.uint32).reshape(-1, ALPHABET)
    with torch.cuda.device(device):
        tables = torch.empty(table_words(len(freqs), table_log) * 4, dtype=torch.uint8, device=device)
        _check(lib().anszp_build_tables(freqs.ctypes.data, len(freqs), table_log, tables.data_ptr(),
                                        _stream_ptr(torch, device)), "anszp_build_tables")
    return tables


def build_tables_device(freqs_dev, table_log: int, status=None):
    """anszp_build_tables_device: freqs_dev is an int32/uint32-valued device tensor of n_tables x 256 entries;
    returns the tables as a new device tensor (int32 view of n_tables * 8 * 2^table_log words)."""
    torch = _torch()
    device = freqs_dev.device
    n_tables = freqs_dev.numel() // ALPHABET
    with torch.cuda.device(device):
        tables = torch.empty(table_words(n_tables, table_log), dtype=torch.int32, device=device)
        _check(lib().anszp_build_tables_device(freqs_dev.data_ptr(), n_tables, table_log, tables.data_ptr(),
                                               status.data_ptr() if status is not None else None,
                                               _stream_ptr(torch, device)), "anszp_build_tables_device")
    return tables


_TORCH_OUT = {"u8": "uint8", "f32": "float32", "bf16": "bfloat16"}


@dataclass
class DeviceContainer:
    host: HostContainer
    device: str
    tables: object
    layers: object
    chunks: object
    stream_hdr: object
    payload: object
    scales: object
    status: object

    def read_status(self):
        torch = _torch()
        torch.cuda.synchronize(self.device)
        st = self.status.cpu().numpy().view(np.uint32)
        return int(st[0]), int(st[1])


def to_device(h: HostContainer, device="cuda:0") -> DeviceContainer:
    """Upload a container and build its decode tables on the device."""
    torch = _torch()
    tables = build_tables(h.freqs, h.table_log, device)
    return DeviceContainer(h, device, tables, _dev(h.layers, device), _dev(h.chunks, device),
                           _dev(h.stream_hdr, device), _dev(h.payload, device), _dev(h.scales, device),
                           torch.zeros(2, dtype=torch.int32, device=device))


def alloc_out(d: DeviceContainer, out_dtype: Optional[str] = None):
    torch = _torch()
    dt = getattr(torch, _TORCH_OUT[out_dtype or d.host.out_dtype])
    return torch.empty(max(d.host.numel, 8), dtype=dt, device=d.device)


def decode_args(d: DeviceContainer, out, out_dtype: Optional[str] = None) -> DecodeArgs:
    h = d.host
    a = DecodeArgs()
    a.tables = d.tables.data_ptr(); a.n_tables = len(h.freqs); a.table_log = h.table_log
    a.n_streams = h.n_streams; a.out_dtype = OUT_CODES[out_dtype or h.out_dtype]
    a.chunks = d.chunks.data_ptr(); a.n_chunks = len(h.chunks)
    a.stream_hdr = d.stream_hdr.data_ptr(); a.n_stream_hdr = len(h.stream_hdr)
    a.payload = d.payload.data_ptr(); a.payload_words = len(h.payload)
    a.layers = d.layers.data_ptr(); a.scales = d.scales.data_ptr(); a.n_scales = len(h.scales)
    a.out = out.data_ptr(); a.out_elems = h.numel; a.status = d.status.data_ptr()
    return a


VARIANT_AUTO, VARIANT_STEPWISE, VARIANT_MERGED, VARIANT_STEPWISE_SHARED, VARIANT_STREAMING, VARIANT_BYTE_TABLE = 0, 1, 2, 3, 4, 5


def decode_raw(args: DecodeArgs, device="cuda:0", variant: Optional[int] = None):
    """anszp_decode (or anszp_decode_variant) on torch's current stream of `device`."""
    torch = _torch()
    with torch.cuda.device(device):
        if variant is None:
            _check(lib().anszp_decode(C.byref(args), _stream_ptr(torch, device)), "anszp_decode")
        else:
            _check(lib().anszp_decode_variant(C.byref(args), variant, _stream_ptr(torch, device)),
                   "anszp_decode_variant")


def plan_bytes(n_chunks: int) -> int:
    return int(lib().anszp_plan_bytes(n_chunks))


def plan_decode(args: DecodeArgs, device="cuda:0"):
    """anszp_plan_decode into a new device buffer (returned as a torch uint8 tensor)."""
    torch = _torch()
    plan = torch.empty(max(16, plan_bytes(args.n_chunks)), dtype=torch.uint8, device=device)
    with torch.cuda.device(device):
        _check(lib().anszp_plan_decode(C.byref(args), plan.data_ptr(), plan.numel(), _stream_ptr(torch, device)), "anszp_plan_decode")
    return plan


def decode_planned_raw(args: DecodeArgs, plan, device="cuda:0"):
    """anszp_decode_planned on torch's current stream of `device`."""
    torch = _torch()
    with torch.cuda.device(device):
        _check(lib().anszp_decode_planned(C.byref(args), plan.data_ptr(), plan.numel(), _stream_ptr(torch, device)), "anszp_decode_planned")


def decode_static_plan_raw(args: DecodeArgs, replan: bool, device="cuda:0"):
    """anszp_decode_static_plan on torch's current stream of `device`."""
    torch = _torch()
    with torch.cuda.device(device):
        _check(lib().anszp_decode_static_plan(C.byref(args), 1 if replan else 0, _stream_ptr(torch, device)), "anszp_decode_static_plan")


LOOKAHEAD_WINDOW_WORDS = 11096     # stream words of one chunk the look-ahead kernel can hold on chip (a chunk that has a workgroup to itself)


def decode_by_chunk_size(d: DeviceContainer, out=None, out_dtype: Optional[str] = None):
    """Decode a container whose chunks differ much in size (streams that follow the input channels: a chunk is a
    group of 64 channels of its layer) with two calls of anszp_decode: one over the chunks whose stream words fit
    the look-ahead kernel's on-chip window, one over the others with the streaming kernel
    (a call decodes all its chunks with one kernel; the descriptors of a call may be any subset in any order).  Returns the output tensor."""
    torch = _torch()
    if out is None:
        out = alloc_out(d, out_dtype)
    words = d.host.chunks["payload_words"]
    parts = [(np.nonzero(words <= LOOKAHEAD_WINDOW_WORDS)[0], VARIANT_MERGED),
             (np.nonzero(words > LOOKAHEAD_WINDOW_WORDS)[0], VARIANT_STREAMING)]
    keep = []
    for idx, variant in parts:
        if len(idx) == 0:
            continue
        sub = _dev(np.ascontiguousarray(d.host.chunks[idx]), d.device)
        keep.append(sub)
        a = decode_args(d, out, out_dtype)
        a.chunks = sub.data_ptr()
        a.n_chunks = len(idx)
        decode_raw(a, d.device, variant)
    torch.cuda.synchronize(d.device)                   # the descriptor copies live until both calls are done
    return out


def decode(d: DeviceContainer, out=None, out_dtype: Optional[str] = None, variant: Optional[int] = None):
    """Decode + dequantise the whole container; returns the output tensor (first numel elements valid)."""
    if out is None:
        out = alloc_out(d, out_dtype)
    decode_raw(decode_args(d, out, out_dtype), d.device, variant)
    return out


def dequant_zp(symbols, zero_point: int, scale: float, out_dtype: str = "bf16", channel_len: int = 0,
               channel_scales=None):
    """anszp_dequant_zp on a uint8 device tensor of symbols."""
    torch = _torch()
    n = symbols.numel()
    dev = symbols.device
    out = torch.empty(max(n, 8), dtype=getattr(torch, _TORCH_OUT[out_dtype]), device=dev)
    lay = np.zeros(1, dtype=LAYER_DTYPE)
    lay[0] = (scale, zero_point, 8, channel_len, 0, 0)
    n_sc = 0 if channel_scales is None else channel_scales.numel()
    with torch.cuda.device(dev):
        _check(lib().anszp_dequant_zp(symbols.data_ptr(), n, lay.ctypes.data,
                                      channel_scales.data_ptr() if channel_scales is not None else None, n_sc,
                                      out.data_ptr(), OUT_CODES[out_dtype], _stream_ptr(torch, dev)),
               "anszp_dequant_zp")
    return out[:n]


def bits_of(t) -> np.ndarray:
    """Raw bit patterns of an output tensor as numpy (u8 / u32 / u16)."""
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).cpu().numpy().view(np.uint32)
    return t.cpu().numpy()


# --------------------------------------------------------------------------- fused decode + convolution
CONV_ROWS = 16          # anszp_conv_fused works on panels of 16, 32 or 64 output channels
CONV_MAX_K = 4608


def conv_rows_per_chunk(k: int) -> int:
    """Output channels per chunk for a layer with reduction length k = kh*kw*cin: the largest power of
    two (at most 16) that keeps a chunk at 4096 symbols or fewer, so that the wavefronts of a
    workgroup have a chunk each to decode where the rows are long."""
    r = 1
    while r < CONV_ROWS and 2 * r * k <= 4096:
        r *= 2
    return r


def pack_conv_layers(layer_symbols: Sequence[np.ndarray], shapes: Sequence[tuple], table_log: int, n_streams: int,
                     zero_points: Sequence[int], scales: Sequence[float], bitwidths: Optional[Sequence[int]] = None):
    """Compress conv layers for anszp_conv_fused.  layer_symbols[i] holds the symbols of layer i in the order
    [cout][kh][kw][cin]; shapes[i] = (cout, cin, kh, kw).  Returns the container, each layer's first chunk
    and its output channels per chunk."""
    rows = [conv_rows_per_chunk(cin * kh * kw) for (_, cin, kh, kw) in shapes]
    sizes = [r * cin * kh * kw for r, (_, cin, kh, kw) in zip(rows, shapes)]
    for sym, (cout, cin, kh, kw) in zip(layer_symbols, shapes):
        if len(sym) != cout * cin * kh * kw or cout % CONV_ROWS or cin * kh * kw > CONV_MAX_K:
            raise ValueError(f"layer shape {(cout, cin, kh, kw)} does not fit anszp_conv_fused")
    h = pack_layers(layer_symbols, table_log, n_streams, max(sizes), zero_points, scales, bitwidths, chunk_sizes=sizes)
    first = np.concatenate([[0], np.cumsum([cout // r for r, (cout, _, _, _) in zip(rows, shapes)])])[:-1]
    return h, [int(f) for f in first], rows


ACT_NHWC, ACT_C8 = 0, 1
ACT_CODES = {"nhwc": ACT_NHWC, "c8": ACT_C8}


def to_c8(t):
    """[batch][h][w][channels] -> [batch][channels / 8][h][w][8] (blocks of 8 channels), a copy."""
    b, h, w, c = t.shape
    return t.view(b, h, w, c // 8, 8).permute(0, 3, 1, 2, 4).contiguous()


def from_c8(t):
    """[batch][channels / 8][h][w][8] -> [batch][h][w][channels], a copy."""
    b, cb, h, w, _ = t.shape
    return t.permute(0, 2, 3, 1, 4).contiguous().view(b, h, w, cb * 8)


def _act_dims(t, layout: str):
    if layout == "c8":
        b, cb, h, w, e = t.shape
        if e != 8:
            raise ValueError("a c8 tensor is [batch][channels / 8][h][w][8]")
        return b, h, w, cb * 8
    b, h, w, c = t.shape
    return b, h, w, c


def conv_out_shape(batch: int, out_h: int, out_w: int, cout: int, layout: str):
    return (batch, cout // 8, out_h, out_w, 8) if layout == "c8" else (batch, out_h, out_w, cout)


def conv_args(d: DeviceContainer, layer: int, first_chunk: int, rows_per_chunk: int, x, shape: tuple, stride: int,
              pad: int, y, x_layout: str = "nhwc", y_layout: str = "nhwc") -> ConvArgs:
    """The argument struct of anszp_conv_fused for one layer: x a bf16 tensor in x_layout, y an fp32 or bf16
    tensor in y_layout ("nhwc": [batch][h][w][channels]; "c8": [batch][channels / 8][h][w][8]),
    shape = (cout, cin, kh, kw)."""
    torch = _torch()
    h = d.host
    cout, cin, kh, kw = shape
    B, H, W, cin_x = _act_dims(x, x_layout)
    ho, wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    if x.dtype != torch.bfloat16 or not x.is_contiguous() or cin_x != cin:
        raise ValueError("x must be a contiguous bf16 tensor with the layer's input channels")
    if y.dtype not in (torch.float32, torch.bfloat16) or not y.is_contiguous() or \
            tuple(y.shape) != conv_out_shape(B, ho, wo, cout, y_layout):
        raise ValueError("y must be a contiguous fp32 or bf16 tensor of the output's shape in y_layout")
    a = ConvArgs()
    a.tables = d.tables.data_ptr(); a.n_tables = len(h.freqs); a.table_log = h.table_log
    a.n_streams = h.n_streams; a.layer_id = layer
    a.chunks = d.chunks.data_ptr() + first_chunk * CHUNK_DTYPE.itemsize; a.n_chunks = len(h.chunks) - first_chunk
    a.stream_hdr = d.stream_hdr.data_ptr(); a.n_stream_hdr = len(h.stream_hdr)
    a.payload = d.payload.data_ptr(); a.payload_words = len(h.payload)
    a.layers = d.layers.data_ptr(); a.scales = d.scales.data_ptr(); a.n_scales = len(h.scales)
    a.rows_per_chunk = rows_per_chunk
    a.batch, a.in_h, a.in_w, a.cin, a.cout, a.kh, a.kw, a.stride, a.pad = B, H, W, cin, cout, kh, kw, stride, pad
    a.x = x.data_ptr(); a.y = y.data_ptr(); a.status = d.status.data_ptr()
    a.y_dtype = OUT_F32 if y.dtype == torch.float32 else OUT_BF16
    a.x_layout = ACT_CODES[x_layout]; a.y_layout = ACT_CODES[y_layout]
    return a


def conv_fused_raw(args: ConvArgs, device="cuda:0"):
    """anszp_conv_fused on torch's current stream of `device`."""
    torch = _torch()
    with torch.cuda.device(device):
        _check(lib().anszp_conv_fused(C.byref(args), _stream_ptr(torch, device)), "anszp_conv_fused")


def conv_fused(d: DeviceContainer, layer: int, first_chunk: int, rows_per_chunk: int, x, shape: tuple, stride: int,
               pad: int, y=None, y_dtype: str = "f32", x_layout: str = "nhwc", y_layout: str = "nhwc"):
    """anszp_conv_fused on torch's current stream: x is a bf16 tensor in x_layout, shape = (cout, cin, kh, kw);
    returns y in y_layout, fp32 or bf16 (y_dtype, or the dtype of the y passed in)."""
    torch = _torch()
    cout, cin, kh, kw = shape
    B, H, W, _ = _act_dims(x, x_layout)
    ho, wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    if ho < 1 or wo < 1:
        raise AnszpError(-2, "anszp_conv_fused")
    if y is None:
        if y_layout == "c8" and cout % 8:
            raise AnszpError(-2, "anszp_conv_fused")
        y = torch.empty(conv_out_shape(B, ho, wo, cout, y_layout), dtype=getattr(torch, _TORCH_OUT[y_dtype]), device=x.device)
    conv_fused_raw(conv_args(d, layer, first_chunk, rows_per_chunk, x, shape, stride, pad, y, x_layout, y_layout), x.device)
    return y


# --------------------------------------------------------------------------- packing on the GPU
def pack_layer_device(symbols_dev, freqs_dev, table_log: int, n_streams: int, chunk_size: int, layer_id: int = 0,
                      out_offset: int = 0, payload_word_offset: int = 0, stream_offset: int = 0,
                      payload_cap_words: Optional[int] = None):
    """anszp_pack_layer_device on torch's current stream: symbols_dev a uint8 tensor, freqs_dev an int32 tensor of
    256 frequencies, both on the GPU.  Returns (chunks, stream_hdr, payload, used, status) as device tensors
    (chunks as raw bytes of anszp_chunk_t; used: one int64; status: two int32)."""
    torch = _torch()
    dev = symbols_dev.device
    n = symbols_dev.numel()
    nc = C.c_uint64(); bound = C.c_uint64()
    _check(lib().anszp_pack_bound(n, table_log, n_streams, chunk_size, C.byref(nc), C.byref(bound)), "anszp_pack_bound")
    cap = bound.value if payload_cap_words is None else payload_cap_words
    chunks = torch.zeros(max(nc.value, 1) * CHUNK_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    hdr = torch.zeros(max(nc.value * n_streams, 4), dtype=torch.int32, device=dev)
    payload = torch.full((max(cap, 4),), -1, dtype=torch.int32, device=dev)
    used = torch.zeros(1, dtype=torch.int64, device=dev)
    status = torch.zeros(2, dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        _check(lib().anszp_pack_layer_device(symbols_dev.data_ptr(), n, freqs_dev.data_ptr(), table_log, n_streams, chunk_size,
                                             layer_id, out_offset, payload_word_offset, stream_offset, chunks.data_ptr(),
                                             hdr.data_ptr(), payload.data_ptr(), cap, used.data_ptr(), status.data_ptr(),
                                             _stream_ptr(torch, dev)), "anszp_pack_layer_device")
    return chunks, hdr, payload, used, status


def pack_jobs(layer_sizes: Sequence[int], chunk_sizes: Sequence[int]) -> np.ndarray:
    """The anszp_pack_job_t array of a set of layers stored one after the other."""
    jobs = np.zeros(len(layer_sizes), dtype=JOB_DTYPE)
    first = chunk = 0
    for i, (n, cs) in enumerate(zip(layer_sizes, chunk_sizes)):
        jobs[i] = (first, n, cs, chunk, (0, 0))
        first += n
        chunk += (n + cs - 1) // cs
    return jobs


def pack_layers_device(symbols_dev, layer_sizes: Sequence[int], freqs_dev, table_log: int, n_streams: int, chunk_size,
                       payload_cap_words: Optional[int] = None, out=None):
    """anszp_pack_layers_device on torch's current stream: symbols_dev a uint8 tensor holding the layers one after the
    other, freqs_dev an int32 tensor [n_layers, 256], both on the GPU; chunk_size: one for all layers or one per layer.
    Returns (chunks, stream_hdr, payload, used, status) as device tensors (out: the same five, to be reused)."""
    torch = _torch()
    dev = symbols_dev.device
    sizes = [int(n) for n in layer_sizes]
    css = [int(chunk_size)] * len(sizes) if np.isscalar(chunk_size) else [int(c) for c in chunk_size]
    jobs = pack_jobs(sizes, css)
    n_chunks = int(sum((n + c - 1) // c for n, c in zip(sizes, css)))
    bound = 0
    for n, c in zip(sizes, css):
        nc, b = C.c_uint64(), C.c_uint64()
        _check(lib().anszp_pack_bound(n, table_log, n_streams, c, C.byref(nc), C.byref(b)), "anszp_pack_bound")
        bound += b.value
    cap = bound if payload_cap_words is None else payload_cap_words
    jobs_dev = torch.from_numpy(jobs.view(np.uint8).copy()).to(dev)
    if out is None:
        chunks = torch.zeros(max(n_chunks, 1) * CHUNK_DTYPE.itemsize, dtype=torch.uint8, device=dev)
        hdr = torch.zeros(max(n_chunks * n_streams, 4), dtype=torch.int32, device=dev)
        payload = torch.full((max(cap, 4),), -1, dtype=torch.int32, device=dev)
        used = torch.zeros(1, dtype=torch.int64, device=dev)
        status = torch.zeros(2, dtype=torch.int32, device=dev)
    else:
        chunks, hdr, payload, used, status = out
    with torch.cuda.device(dev):
        _check(lib().anszp_pack_layers_device(symbols_dev.data_ptr(), jobs_dev.data_ptr(), len(sizes), n_chunks, freqs_dev.data_ptr(),
                                              table_log, n_streams, chunks.data_ptr(), hdr.data_ptr(), payload.data_ptr(), cap,
                                              used.data_ptr(), status.data_ptr(), _stream_ptr(torch, dev)), "anszp_pack_layers_device")
        torch.cuda.current_stream(dev).synchronize()      # (jobs_dev must outlive the launches)
    return chunks, hdr, payload, used, status
