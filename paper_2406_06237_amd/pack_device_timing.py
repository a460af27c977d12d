"""Times the packer on the GPU (anszp_pack_layer_device) on the layers of the ResNet-50-shaped set
(config 3): `python -m paper_2406_06237_amd.pack_device_timing`.  One call per layer, symbols and
frequencies resident in device memory; prints symbols/s over the whole set and the host packer's rate
on one layer beside it."""
from __future__ import annotations

import time

import numpy as np


def main():
    import torch
    from . import binding as B
    from . import workloads as W

    dev = "cuda:0"
    w = W.config3()
    syms = w.symbols()
    freqs = [B.normalize_freqs(np.bincount(s, minlength=256), w.table_log) for s in syms]
    s_dev = [torch.from_numpy(s).to(dev) for s in syms]
    f_dev = [torch.from_numpy(f.astype(np.uint32).view(np.int32)).to(dev) for f in freqs]

    def step():
        for s, f in zip(s_dev, f_dev):
            B.pack_layer_device(s, f, w.table_log, w.n_streams, w.chunk_size)

    step()
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    reps = 5
    for _ in range(reps):
        step()
    torch.cuda.synchronize(dev)
    gpu = (time.perf_counter() - t0) / reps
    i = int(np.argmax([len(s) for s in syms]))
    t0 = time.perf_counter()
    B.pack_layer(syms[i], freqs[i], w.table_log, w.n_streams, w.chunk_size, 0, 0, 0, 0)
    host = time.perf_counter() - t0
    print(f"GPU packer: {w.numel} symbols in {len(syms)} calls, {gpu * 1e3:.2f} ms per set "
          f"({w.numel / gpu / 1e9:.2f} Gsymbols/s, allocations of the outputs included)")
    print(f"host packer: layer {w.layers[i].name} ({len(syms[i])} symbols) in {host * 1e3:.1f} ms "
          f"({len(syms[i]) / host / 1e9:.3f} Gsymbols/s, one thread)")


if __name__ == "__main__":
    main()
