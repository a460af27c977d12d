#!/usr/bin/env python3
"""Benchmark of the hot path: tANS decode + zero-point dequantisation of a whole synthetic weight
set on one MI355X.  One "step" decodes every layer of the set once (one anszp_decode call).

Prints ONE JSON line: decoded Gsymbols/s (value), the HBM roofline of the decode kernel measured
live with events on the launch stream, and the CPU oracle timed on the host cores beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def load_traffic(name: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if a summary
    for this workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{name}.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                pass
    if "fetch_bytes_per_launch" in vals and "write_bytes_per_launch" in vals:
        return vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"]
    return None


def cpu_baseline(workload, repeats: int = 3):
    """The oracle as it stands (decode + dequant of the same weight set) on the host cores."""
    import numpy as np
    import oracle
    c = oracle.encode_layers(workload.symbols(), workload.table_log, workload.n_streams, workload.chunk_size)
    L = workload.layers
    tables = oracle.tables_for(c)
    cores = min(os.cpu_count() or 1, 16)
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = max(1, min(cores, int(env)))
    best = float("inf")
    for _ in range(repeats):
        t0 = time.perf_counter()
        sym, wts, rc = oracle.decode_dequant(c, [l.zero_point for l in L], [l.scale for l in L],
                                             [l.channel_len for l in L], [l.channel_scales for l in L],
                                             out_dtype=workload.out_dtype, n_threads=cores, tables=tables)
        best = min(best, time.perf_counter() - t0)
        assert rc == 0
    return {"value": workload.numel / best / 1e9, "unit": "Gsymbols/s", "cores": cores, "kind": "oracle",
            "sample": f"whole {workload.name} set ({workload.numel} symbols), decode+dequant, best of {repeats}, "
                      f"{best * 1e3:.1f} ms"}, wts


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4])
    ap.add_argument("--blocks", type=int, default=32, help="config 4 only: number of blocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB five times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build decodes on ONE GPU (chunks are independent: each GPU would decode the chunks "
              "of its own layers, no collective involved). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2406_06237_amd import binding as B
    from paper_2406_06237_amd import workloads as W

    w = {1: W.config1, 2: W.config2, 3: W.config3}.get(args.config, lambda: W.config4(args.blocks))()
    h = B.pack_workload(w)                      # library's own host packer
    dev = "cuda:0"
    d = B.to_device(h, dev)
    out = B.alloc_out(d)
    a = B.decode_args(d, out)
    stream = torch.cuda.current_stream(dev)

    for _ in range(args.warmup):
        B.decode_raw(a, dev)
    torch.cuda.synchronize(dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        B.decode_raw(a, dev)
    ev1.record(stream)
    torch.cuda.synchronize(dev)
    wall = time.perf_counter() - t0
    status = d.read_status()
    if status != (0, 0):
        print(f"bench.py: device status {status}", file=sys.stderr)
        sys.exit(1)
    kernel_ms = ev0.elapsed_time(ev1) / args.steps
    if args.calib_copy:
        src = torch.full((args.calib_copy << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize(dev)
    ms_per_step = wall * 1e3 / args.steps

    elem_bytes = {"u8": 1, "f32": 4, "bf16": 2}[w.out_dtype]
    algo_bytes = h.compressed_bytes() + w.numel * elem_bytes
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "decoded Gsymbols/s (tANS decode + zero-point dequant, whole weight set per step)",
        "value": w.numel / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gsymbols/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"config{args.config}:{w.name}", "symbols": w.numel, "layers": len(w.layers),
                   "chunks": int(len(h.chunks)), "streams_per_chunk": w.n_streams, "chunk_size": w.chunk_size,
                   "table_log": w.table_log, "out_dtype": w.out_dtype,
                   "compressed_bytes": h.compressed_bytes(),
                   "bits_per_symbol": 8.0 * h.compressed_bytes() / w.numel,
                   "source_entropy_bits": w.model_entropy_bits()},
        "effective_GBps": algo_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": load_traffic(f"config{args.config}"),
                     "kernel_ms": kernel_ms, "algorithmic_bytes": algo_bytes},
    }
    if not args.no_cpu_baseline:
        base, wts = cpu_baseline(w)
        result["cpu_baseline"] = base
        got = B.bits_of(out)[:w.numel]
        want = wts.view(np.uint32) if w.out_dtype == "f32" else wts
        result["matches_oracle"] = bool(np.array_equal(got, want))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
