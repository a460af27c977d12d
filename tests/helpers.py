"""Glue used by the GPU parity tests: turn the oracle's container (plain arrays) into the
ABI's structures, and compute the oracle's expected output for a workload."""
import numpy as np

from paper_2406_06237_amd import binding as B


def host_from_oracle(c, workload) -> B.HostContainer:
    """Wrap bytes produced by the oracle's encoder in the library's structures (no re-encoding)."""
    L = workload.layers
    chunks = np.zeros(c.n_chunks, dtype=B.CHUNK_DTYPE)
    chunks["layer_id"] = c.chunk_layer
    chunks["n_symbols"] = c.chunk_nsym
    chunks["out_offset"] = c.chunk_out_off
    chunks["payload_offset"] = c.chunk_payload_off
    chunks["payload_words"] = c.chunk_payload_words
    chunks["stream_offset"] = c.chunk_stream_off
    layers = np.zeros(len(L), dtype=B.LAYER_DTYPE)
    sc, n_sc = [], 0
    for i, l in enumerate(L):
        layers[i] = (l.scale, l.zero_point, l.bitwidth, l.channel_len, n_sc, int(c.layer_out_base[i]))
        if l.channel_len:
            sc.append(np.asarray(l.channel_scales, dtype=np.float32))
            n_sc += len(l.channel_scales)
    return B.HostContainer(c.R, c.N, c.chunk_size, workload.out_dtype, c.freqs.copy(), layers, chunks,
                           c.stream_hdr.copy(), c.payload.copy(),
                           np.concatenate(sc) if sc else np.zeros(0, np.float32), c.numel)


def oracle_encode(orc, workload):
    sizes = getattr(workload, "chunk_sizes", None)
    return orc.encode_layers(workload.symbols(), workload.table_log, workload.n_streams, sizes if sizes is not None else workload.chunk_size)


def oracle_expected(orc, c, workload, out_dtype=None, n_threads=8):
    """(symbols, weights-as-bit-patterns) from the oracle's decoder + dequantiser."""
    L = workload.layers
    dt = out_dtype or workload.out_dtype
    sym, wts, rc = orc.decode_dequant(c, [l.zero_point for l in L], [l.scale for l in L],
                                      [l.channel_len for l in L], [l.channel_scales for l in L],
                                      out_dtype=dt, n_threads=n_threads)
    assert rc == 0
    if dt == "u8":
        return sym, sym
    return sym, (wts.view(np.uint32) if dt == "f32" else wts)
