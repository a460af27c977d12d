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
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE).  The counters cannot be
    read from inside this run; the figure is the one in the summary committed under profiles/ for this
    workload, and the second value returned says which file and which state of the kernel it belongs to."""
    rel = os.path.join("profiles", f"hbm_traffic_{name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    vals, commit = {}, None
    for line in open(path):
        if line.startswith("kernel_source_commit:"):
            commit = line.split(":", 1)[1].strip()
        elif ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                pass
    if "fetch_bytes_per_launch" in vals and "write_bytes_per_launch" in vals:
        return (vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"],
                f"{rel} (rocprofv3 --pmc, not measured in this run; kernel sources as of commit {commit})")
    return None, None


def lookups_per_stream(h):
    """Table look-ups the look-ahead kernel makes for every stream of a container (Sec. II-A steps merged into
    entries, see anszp.h): the automaton of the library's own tables walked on the host for all streams at
    once.  A stream's look-ups are a dependent chain, one lane each, whatever the bandwidth."""
    import numpy as np
    from paper_2406_06237_amd import binding as B
    t = B.split_table(B.build_tables_host(h.freqs, h.table_log))
    E = 2 << h.table_log                                                  # entries per table
    bits, count, base = (t[k].reshape(-1).astype(np.int64) for k in ("la_bits", "la_count", "la_base"))
    N = h.n_streams
    n_sym = (np.maximum(h.chunks["n_symbols"].astype(np.int64)[:, None] - np.arange(N)[None, :] + N - 1, 0) // N).reshape(-1)
    hdr = h.stream_hdr.astype(np.int64)
    words = (hdr >> 16).reshape(-1, N)
    first = (h.chunks["payload_offset"].astype(np.int64)[:, None] + np.cumsum(words, axis=1) - words).reshape(-1)
    table0 = np.repeat(h.chunks["layer_id"].astype(np.int64) * E, N)
    payload = np.concatenate([h.payload, np.zeros(4, np.uint32)]).astype(np.uint64)
    rev13 = np.array([int(f"{v:013b}"[::-1], 2) for v in range(1 << 13)], dtype=np.int64)

    def peek(pos, k):                                                     # next k <= 13 stream bits, first bit on top
        w = first + (pos >> 5)
        two = payload[w] | (payload[w + 1] << np.uint64(32))
        return rev13[((two >> (pos & 31).astype(np.uint64)) & np.uint64(0x1FFF)).astype(np.int64)] >> (13 - k)

    pos = np.zeros(len(hdr), np.int64)
    idx = 2 * (hdr & ((1 << h.table_log) - 1)) + peek(pos, np.ones(len(hdr), np.int64))
    left, lookups = n_sym.copy(), np.zeros(len(hdr), np.int64)
    while True:
        live = left > 0
        if not live.any():
            break
        e = table0 + np.where(live, idx, 0)
        idx = np.where(live, base[e] + peek(pos, bits[e] + 1), idx)
        pos = np.where(live, pos + bits[e], pos)
        left = left - np.where(live, count[e], 0)
        lookups += live
    return lookups.reshape(-1, N)


def time_launches(B, torch, args, dev, steps, warmup):
    """Average duration of one anszp_decode launch, events on the launch stream."""
    stream = torch.cuda.current_stream(dev)
    for _ in range(warmup):
        B.decode_raw(args, dev)
    torch.cuda.synchronize(dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        B.decode_raw(args, dev)
    e1.record(stream)
    torch.cuda.synchronize(dev)
    return e0.elapsed_time(e1) / steps


def chain_bound(w, h, steps):
    """The second bound beside the HBM roofline: look-ups of the slowest stream x the time of one look-up.
    The time of a look-up is measured in this run as a slope: the slowest chunk's layer decoded alone, as one
    chunk of full size and as one chunk of half size (one workgroup each, so launch and staging cancel)."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2406_06237_amd import binding as B
    from paper_2406_06237_amd import workloads as W
    per_stream = lookups_per_stream(h)
    slowest = int(np.argmax(per_stream.max(axis=1)))
    layer = w.layers[int(h.chunks["layer_id"][slowest])]
    full = min(w.chunk_size, layer.numel)
    points = []
    for n in (full, full // 2):
        one = W.Workload(f"{layer.name}[:{n}]", [dataclasses.replace(layer, shape=(n,))], w.table_log, w.n_streams,
                         w.chunk_size, w.out_dtype)
        hh = B.pack_workload(one)
        d = B.to_device(hh, "cuda:0")
        out = B.alloc_out(d)
        ms = time_launches(B, torch, B.decode_args(d, out), "cuda:0", steps, 10)      # (n_chunks == 1: nothing to plan)
        assert d.read_status() == (0, 0)
        points.append((int(lookups_per_stream(hh).max()), ms * 1e3))
    (s1, t1), (s0, t0) = points
    ns = 1e3 * (t1 - t0) / max(1, s1 - s0)
    s = int(per_stream.max())
    return {"us": s * ns * 1e-3, "lookups_slowest_stream": s, "ns_per_lookup": ns,
            "symbols_slowest_stream": int(-(-int(h.chunks["n_symbols"][slowest]) // w.n_streams)),
            "how": f"slope of two one-chunk launches of layer {layer.name}: {s1} look-ups in {t1:.2f} us, {s0} in {t0:.2f} us "
                   "(events on the launch stream); launch, staging and the wait for the last stores are not in it"}


def replicate(h, k):
    """k copies of a container side by side (own tables, words, headers and outputs), for one launch."""
    import dataclasses
    import numpy as np
    chunks, layers = [], []
    for r in range(k):
        c, l = h.chunks.copy(), h.layers.copy()
        c["layer_id"] += r * len(h.layers)
        c["out_offset"] += r * h.numel
        c["payload_offset"] += r * len(h.payload)
        c["stream_offset"] += r * len(h.stream_hdr)
        l["out_base"] += r * h.numel
        l["scales_offset"] += r * len(h.scales)
        chunks.append(c)
        layers.append(l)
    assert len(h.payload) % 4 == 0
    return dataclasses.replace(h, freqs=np.tile(h.freqs, (k, 1)), layers=np.concatenate(layers), chunks=np.concatenate(chunks),
                               stream_hdr=np.tile(h.stream_hdr, k), payload=np.tile(h.payload, k), scales=np.tile(h.scales, k),
                               numel=h.numel * k)


def steady_state(w, h, k, steps, elem_bytes):
    """k replicas of the set decoded by ONE launch: what the kernel sustains once the chip is full.  Never the
    headline: the headline decodes the set once per launch."""
    import torch
    from paper_2406_06237_amd import binding as B
    d = B.to_device(replicate(h, k), "cuda:0")
    out = B.alloc_out(d)
    a = B.decode_args(d, out)
    plan = B.plan_decode(a, "cuda:0")
    stream = torch.cuda.current_stream("cuda:0")
    for _ in range(5):
        B.decode_planned_raw(a, plan, "cuda:0")
    torch.cuda.synchronize("cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        B.decode_planned_raw(a, plan, "cuda:0")
    e1.record(stream)
    torch.cuda.synchronize("cuda:0")
    ms = e0.elapsed_time(e1) / steps
    assert d.read_status() == (0, 0)
    same = bool(torch.equal(out[:h.numel].view(torch.int16), out[(k - 1) * h.numel:k * h.numel].view(torch.int16))) \
        if w.out_dtype == "bf16" else None
    nbytes = k * (h.compressed_bytes() + w.numel * elem_bytes)
    return {"label": f"{k} replicas of the set in one launch (not the headline)", "replicas": k, "kernel_ms": ms,
            "Gsymbols_per_s": k * w.numel / (ms * 1e-3) / 1e9, "GBps": nbytes / (ms * 1e-3) / 1e9,
            "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "first_and_last_replica_equal": same}


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

    def timed(n_threads):
        best, wts = float("inf"), None
        for _ in range(repeats):
            t0 = time.perf_counter()
            sym, wts, rc = oracle.decode_dequant(c, [l.zero_point for l in L], [l.scale for l in L],
                                                 [l.channel_len for l in L], [l.channel_scales for l in L],
                                                 out_dtype=workload.out_dtype, n_threads=n_threads, tables=tables)
            best = min(best, time.perf_counter() - t0)
            assert rc == 0
        return best, wts

    best, wts = timed(cores)
    single, _ = timed(1)
    return {"value": workload.numel / best / 1e9, "unit": "Gsymbols/s", "cores": cores, "kind": "oracle",
            "sample": f"whole {workload.name} set ({workload.numel} symbols), decode+dequant, best of {repeats}, "
                      f"{best * 1e3:.1f} ms",
            "single_thread": {"value": workload.numel / single / 1e9, "unit": "Gsymbols/s", "cores": 1,
                              "sample": f"the same set on one thread, best of {repeats}, {single * 1e3:.1f} ms"}}, wts


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix rate


def bench_fused_conv(args):
    """Config 5: every conv layer of the ResNet-50-shaped set, weights decoded inside the convolution kernel
    (anszp_conv_fused), batch 64 at 224 x 224 geometry, synthetic N(0,1) bf16 activations.  One step = the 53
    launches, one per layer.  Returns the result (TFLOP/s against the dense bf16 MFMA peak): `--config 5` prints it as
    the JSON line, the default run carries it as a secondary result beside the headline."""
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
    return result


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
    ap.add_argument("--no-secondary", action="store_true", help="config 3 only: leave out the ResNet-18-shaped set")
    ap.add_argument("--no-plan", action="store_true", help="time anszp_decode instead of anszp_decode_planned")
    ap.add_argument("--no-extras", action="store_true", help="leave out the chain bound and the steady-state launch")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB five times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build decodes on ONE GPU (chunks are independent: each GPU would decode the chunks "
              "of its own layers, no collective involved). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.config == 5:
        print(json.dumps(bench_fused_conv(args)))
        return

    result = bench_decode(args, args.config, headline=True)
    if args.config == 3 and not args.no_secondary:
        # the ResNet-18-shaped set beside the headline, same measurement (bench.py --config 4 runs the large
        # stack: minutes, not part of the default run)
        sec = bench_decode(args, 2, headline=False)
        result["secondary"] = [{k: sec[k] for k in ("config", "value", "unit", "ms_per_step", "roofline", "without_plan", "chain_bound",
                                                    "cpu_baseline", "matches_oracle") if k in sec}]
        # the fused decode + convolution over the same weight set (config 5), one step = its 53 launches
        conv = bench_fused_conv(args)
        result["secondary"].append({k: conv[k] for k in ("metric", "config", "value", "unit", "steps", "ms_per_step", "roofline",
                                                         "max_relative_error_sampled", "matches_oracle", "cpu_baseline") if k in conv})
    print(json.dumps(result))


def bench_decode(args, config, headline):
    """One decode configuration: K launches timed on the wall clock and with events, the roofline of the
    launch, the chain bound, and the oracle on the host cores with a bit-for-bit comparison."""
    import numpy as np
    import torch
    from paper_2406_06237_amd import binding as B
    from paper_2406_06237_amd import workloads as W

    w = {1: W.config1, 2: W.config2, 3: W.config3}.get(config, lambda: W.config4(args.blocks))()
    h = B.pack_workload(w)                      # library's own host packer
    dev = "cuda:0"
    d = B.to_device(h, dev)
    out = B.alloc_out(d)
    a = B.decode_args(d, out)
    stream = torch.cuda.current_stream(dev)
    # The work assignment of the launch is prepared once, like the tables (the arrays of a network do not change
    # between inferences): anszp_plan_decode before the timed region, anszp_decode_planned inside it.  The launch
    # without a plan (anszp_decode) is timed beside it.
    plan = None if args.no_plan else B.plan_decode(a, dev)

    def step():
        if plan is None:
            B.decode_raw(a, dev)
        else:
            B.decode_planned_raw(a, plan, dev)

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
    status = d.read_status()
    if status != (0, 0):
        print(f"bench.py: device status {status}", file=sys.stderr)
        sys.exit(1)
    kernel_ms = ev0.elapsed_time(ev1) / args.steps
    if headline and args.calib_copy:
        src = torch.full((args.calib_copy << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize(dev)
    ms_per_step = wall * 1e3 / args.steps

    elem_bytes = {"u8": 1, "f32": 4, "bf16": 2}[w.out_dtype]
    algo_bytes = h.compressed_bytes() + w.numel * elem_bytes
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    traffic, traffic_source = load_traffic(f"config{config}")
    result = {
        "metric": "decoded Gsymbols/s (tANS decode + zero-point dequant, whole weight set per step)",
        "value": w.numel / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gsymbols/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"config{config}:{w.name}", "symbols": w.numel, "layers": len(w.layers),
                   "chunks": int(len(h.chunks)), "streams_per_chunk": w.n_streams, "chunk_size": w.chunk_size,
                   "table_log": w.table_log, "out_dtype": w.out_dtype,
                   "entry_point": "anszp_decode" if plan is None else "anszp_decode_planned (plan written once by anszp_plan_decode, before the timed region)",
                   "compressed_bytes": h.compressed_bytes(),
                   "bits_per_symbol": 8.0 * h.compressed_bytes() / w.numel,
                   "source_entropy_bits": w.model_entropy_bits()},
        "effective_GBps": algo_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms": kernel_ms, "algorithmic_bytes": algo_bytes,
                     "timer": "events on the launch stream around the K launches / K"},
    }
    if plan is not None and not args.no_extras and config != 4:
        result["without_plan"] = {"entry_point": "anszp_decode", "kernel_ms": time_launches(B, torch, a, dev, args.steps, args.warmup)}
        result["without_plan"]["hbm_frac"] = algo_bytes / (result["without_plan"]["kernel_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS
    if config in (2, 3) and not args.no_extras:
        result["chain_bound"] = chain_bound(w, h, max(20, args.steps // 4))
        if headline:
            result["steady_state"] = steady_state(w, h, 8, max(10, args.steps // 10), elem_bytes)
    if not args.no_cpu_baseline:
        base, wts = cpu_baseline(w)
        result["cpu_baseline"] = base
        got = B.bits_of(out)[:w.numel]
        want = wts.view(np.uint32) if w.out_dtype == "f32" else wts
        result["matches_oracle"] = bool(np.array_equal(got, want))
    return result


if __name__ == "__main__":
    main()
