"""Table-size study on synthetic weights (the analogue of the paper's Sec. III-B table: compressed size of
a ResNet-50 for l = 64, 128, 256 states, one stream per layer against parallel streams).

The paper's trained network is not available; `workloads.resnet50_odd_bins()` stands in for it (same layer
shapes, odd bin counts 13..31 with the zero-point in the middle, below one bit per weight on average), so
only the trend is comparable: how the gap to the entropy bound grows as the table shrinks, and what
parallel streams cost.  Everything here runs on the host through the library's own packer.

    python -m paper_2406_06237_amd.table_size_study [--states 64 128 256 4096] [--layers K]
"""
import argparse

import numpy as np

from . import binding as B
from . import workloads as W


def study(states=(64, 128, 256), max_layers=None):
    """Rows of (states, geometry, container bytes, bytes with the paper's per-stream cost, streams)."""
    w = W.resnet50_odd_bins()
    layers = w.layers if max_layers is None else w.layers[:max_layers]
    syms = [l.symbols() for l in layers]
    numel = sum(len(s) for s in syms)
    # empirical entropy bound of the set: each layer with its own symbol statistics (Sec. III-A: one coder per layer)
    bound_bits = 0.0
    for s in syms:
        cnt = np.bincount(s, minlength=256).astype(np.float64)
        p = cnt[cnt > 0] / cnt.sum()
        bound_bits += -(p * np.log2(p)).sum() * len(s)
    rows = []
    for st in states:
        R = int(st).bit_length() - 1
        assert 1 << R == st
        for geometry in ("single stream per layer", "64 streams, channel-sized", "64 streams per 65,536 (benchmark)"):
            total = streams = 0
            for l, s in zip(layers, syms):
                if geometry.startswith("single"):
                    n_streams, chunk = 1, max(len(s), 1)
                elif "channel" in geometry:        # a stream as long as one input channel's weights: Cout * kh * kw
                    per_stream = len(s) // l.shape[1] if len(l.shape) == 4 else len(s)
                    n_streams, chunk = 64, 64 * max(per_stream, 1)
                else:
                    n_streams, chunk = 64, 65536
                f = B.normalize_freqs(np.bincount(s, minlength=256), R)
                chunks, hdr, payload = B.pack_layer(s, f, R, n_streams, chunk)
                used = int(np.count_nonzero(hdr >> 16)) if n_streams > 1 else 1
                total += 4 * int(chunks["payload_words"].astype(np.uint64).sum()) + 4 * len(hdr)
                streams += max(used, 1)
            # the paper counts only the final state (log2 l bits) per stream; this container spends a 32-bit
            # header and, on average, half a word of padding
            paper_like = total - streams * 6 + streams * R / 8.0
            rows.append((st, geometry, total, paper_like, streams))
    return rows, bound_bits / 8.0, numel


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--states", type=int, nargs="+", default=[64, 128, 256, 4096])
    ap.add_argument("--layers", type=int, default=None, help="only the first K layers")
    a = ap.parse_args()
    rows, bound, numel = study(a.states, a.layers)
    print(f"{numel} weights, entropy bound {bound / 1e6:.3f} MB ({8 * bound / numel:.3f} bit/weight)")
    print(f"{'states':>6}  {'geometry':<36} {'container MB':>12} {'gap':>7}   {'paper accounting MB':>19} {'gap':>7}  streams")
    for st, g, total, paper_like, streams in rows:
        print(f"{st:>6}  {g:<36} {total / 1e6:>12.3f} {100 * (total / bound - 1):>6.2f}%   {paper_like / 1e6:>19.3f} "
              f"{100 * (paper_like / bound - 1):>6.2f}%  {streams}")


if __name__ == "__main__":
    main()
