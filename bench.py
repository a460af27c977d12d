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


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix rate


def bench_fused_conv(args):
    """Config 5: every conv layer of the ResNet-50-shaped set, weights decoded inside the convolution kernel
    (anszp_conv_fused), batch 64 at 224 x 224 geometry, synthetic N(0,1) bf16 activations.  One step = the 53
    launches, one per layer.  Prints one JSON line: TFLOP/s against the dense bf16 MFMA peak."""
    import numpy as np
    import torch
    from paper_2406_06237_amd import binding as B
    from paper_2406_06237_amd import workloads as W

    dev = "cuda:0"
    batch = args.batch
    w = W.config3()
    geo = W.resnet50_conv_geometry()
    shapes = [g[1] for g in geo]
    syms = w.symbols()                                     # per layer, read as [cout][kh][kw][cin]
    L = w.layers
    h, first, rows = B.pack_conv_layers(syms, shapes, w.table_log, w.n_streams, [l.zero_point for l in L],
                                        [l.scale for l in L], [l.bitwidth for l in L])
    d = B.to_device(h, dev)
    n_x = max(batch * g[4] * g[4] * g[1][1] for g in geo)
    codes, values = W.bf16_activations(n_x, 5)
    xbuf = torch.from_numpy(codes.view(np.int16)).to(dev).view(torch.bfloat16)
    out_hw = [(g[4] + 2 * g[3] - g[1][2]) // g[2] + 1 for g in geo]
    ybuf = torch.empty(max(batch * o * o * g[1][0] for o, g in zip(out_hw, geo)),
                       dtype=torch.float32 if args.y_dtype == "f32" else torch.bfloat16, device=dev)
    macs = [g[1][0] * g[1][1] * g[1][2] * g[1][3] * o * o * batch for o, g in zip(out_hw, geo)]

    # activations and outputs in blocks of 8 channels ("c8"), except an input whose channels are no multiple of 8
    # (the image the first layer reads), which is NHWC
    def x_layout(i):
        return args.layout if geo[i][1][1] % 8 == 0 else "nhwc"

    def views(i):
        (cout, cin, kh, kw), stride, pad, size = geo[i][1], geo[i][2], geo[i][3], geo[i][4]
        x = xbuf[:batch * size * size * cin]
        x = x.view(batch, cin // 8, size, size, 8) if x_layout(i) == "c8" else x.view(batch, size, size, cin)
        y = ybuf[:batch * out_hw[i] * out_hw[i] * cout].view(B.conv_out_shape(batch, out_hw[i], out_hw[i], cout, args.layout))
        return x, y, stride, pad

    calls = []
    for i in range(len(geo)):
        x, y, stride, pad = views(i)
        calls.append(B.conv_args(d, i, first[i], rows[i], x, shapes[i], stride, pad, y, x_layout(i), args.layout))

    def step():
        for a in calls:
            B.conv_fused_raw(a, dev)

    stream = torch.cuda.current_stream(dev)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize(dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize(dev)
    wall = time.perf_counter() - t0
    if d.read_status() != (0, 0):
        print(f"bench.py: device status {d.read_status()}", file=sys.stderr)
        sys.exit(1)
    kernel_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    flops = 2.0 * sum(macs)

    per_layer = []
    if args.per_layer:
        for i in range(len(geo)):
            x, y, stride, pad = views(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(3):
                B.conv_fused_raw(calls[i], dev)
            e1.record(stream)
            torch.cuda.synchronize(dev)
            ms = e0.elapsed_time(e1) / 3
            per_layer.append({"layer": geo[i][0], "shape": list(shapes[i]), "in": geo[i][4], "stride": geo[i][2],
                              "ms": ms, "TFLOPs": 2.0 * macs[i] / (ms * 1e-3) / 1e12})

    achieved = flops / (kernel_ms * 1e-3) / 1e12
    result = {
        "metric": "fused decode + conv TFLOP/s (ResNet-50 conv layers, weights decoded inside the kernel)",
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config5:resnet50_fused_conv", "batch": batch, "layers": len(geo), "image": 224,
                   "y_dtype": args.y_dtype, "activation_layout": args.layout,
                   "macs_per_step": int(sum(macs)), "symbols": w.numel, "compressed_bytes": h.compressed_bytes(),
                   "bits_per_symbol": 8.0 * h.compressed_bytes() / w.numel, "chunks": int(len(h.chunks))},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel_ms": kernel_ms},
    }
    if per_layer:
        result["per_layer"] = per_layer
    if not args.no_cpu_baseline:
        import oracle
        from oracle import conv_oracle as CO
        # sampled outputs of every layer against the oracle, one dot product each
        rng = np.random.default_rng(7)
        worst = 0.0
        for i in range(len(geo)):
            x, y, stride, pad = views(i)
            B.conv_fused_raw(calls[i], dev)
            torch.cuda.synchronize(dev)
            cout, cin, kh, kw = shapes[i]
            where = np.stack([rng.integers(0, n, 24) for n in (batch, out_hw[i], out_hw[i], cout)], axis=1)
            wb, wh, ww, wo_ = (torch.from_numpy(where[:, k]).to(dev) for k in range(4))
            got = (y[wb, wo_ // 8, wh, ww, wo_ % 8] if args.layout == "c8" else y[wb, wh, ww, wo_]).float().cpu().numpy().astype(np.float64)
            size = geo[i][4]
            xh = values[:batch * size * size * cin]
            xh = (xh.reshape(batch, cin // 8, size, size, 8).transpose(0, 2, 3, 1, 4).reshape(batch, size, size, cin)
                  if x_layout(i) == "c8" else xh.reshape(batch, size, size, cin))
            wts = CO.dequantized_weights(syms[i], L[i].zero_point, L[i].scale, (cout, kh, kw, cin))
            want = CO.conv2d_nhwc_samples(xh, wts, stride, pad, where)
            rms = float(np.sqrt(np.mean(want ** 2))) + 1e-30          # relative error, outputs below the rms measured against it
            worst = max(worst, float(np.max(np.abs(got - want) / np.maximum(np.abs(want), rms))))
        result["max_relative_error_sampled"] = worst
        result["matches_oracle"] = bool(worst <= 1e-2)
        # the oracle itself on the host: decode one layer's weights and convolve in fp64
        i = [g[0] for g in geo].index("layer3.1.conv2")
        cout, cin, kh, kw = shapes[i]
        size = geo[i][4]
        xh = values[:batch * size * size * cin].reshape(batch, size, size, cin)   # any N(0,1) values will do for a timing
        c = oracle.encode_layers([syms[i]], w.table_log, w.n_streams, rows[i] * cin * kh * kw)
        cores = min(os.cpu_count() or 1, 16)
        t0 = time.perf_counter()
        sym, _, rc = oracle.decode_dequant(c, [L[i].zero_point], [L[i].scale], [0], [None], out_dtype="f32", n_threads=cores)
        wts = CO.dequantized_weights(sym, L[i].zero_point, L[i].scale, (cout, kh, kw, cin))
        CO.conv2d_nhwc(xh, wts, geo[i][2], geo[i][3])
        dt = time.perf_counter() - t0
        assert rc == 0
        result["cpu_baseline"] = {"value": 2.0 * macs[i] / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                                  "sample": f"layer3.1.conv2 ({cout}x{cin}x{kh}x{kw}, {size}x{size}, batch {batch}): oracle "
                                            f"decode + fp64 convolution, {dt:.2f} s"}
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=64, help="config 5 only: images per step")
    ap.add_argument("--per-layer", action="store_true", help="config 5 only: also time every layer on its own")
    ap.add_argument("--y-dtype", default="bf16", choices=["bf16", "f32"], help="config 5 only: output element type")
    ap.add_argument("--layout", default="c8", choices=["c8", "nhwc"],
                    help="config 5 only: activations and outputs in blocks of 8 channels, or NHWC")
    ap.add_argument("--blocks", type=int, default=32, help="config 4 only: number of blocks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB five times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build decodes on ONE GPU (chunks are independent: each GPU would decode the chunks "
              "of its own layers, no collective involved). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.config == 5:
        return bench_fused_conv(args)

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
