"""Seeded synthetic weight sets that stand in for the paper's trained networks.

This module only makes INPUTS: layer shapes, per-layer quantizer parameters and
quantized symbols drawn from stated distributions.  It contains no part of the
codec (no table construction, no encoding, decoding or dequantisation), so that
the CPU oracle and the GPU library can both be fed from it without sharing any
of the method's arithmetic.

The paper (Sec. III-A) evaluates ImageNet-trained ResNet-18/50 whose quantized
weights concentrate on the zero-point (Sec. II-B) and reach about 0.85 bit per
weight in the feature extractor (Sec. III-C).  Those weights are not available;
the sets below keep the public layer shapes and the stated value distributions.

Random numbers come from a counter-based SplitMix64 generator written out
below, so a (seed, index) pair always gives the same symbol.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
BASE_SEED = 0x240606237000


def splitmix64(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """n 64-bit outputs of SplitMix64 for counters offset+1 .. offset+n."""
    idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & _MASK64) + idx * np.uint64(_GOLDEN))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _uniform01(seed: int, n: int, offset: int = 0) -> np.ndarray:
    return (splitmix64(seed, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def sample_symbols(pmf: np.ndarray, n: int, seed: int) -> np.ndarray:
    """n i.i.d. symbols from pmf by inverse CDF on 32-bit thresholds."""
    pmf = np.asarray(pmf, dtype=np.float64)
    cdf = np.cumsum(pmf / pmf.sum())
    thr = np.minimum(np.floor(cdf * 4294967296.0), 4294967295.0).astype(np.uint64)
    thr[-1] = np.uint64(4294967296)  # last symbol takes the rest
    out = np.empty(n, dtype=np.uint8)
    step = 1 << 22
    for start in range(0, n, step):
        m = min(step, n - start)
        r = splitmix64(seed, m, start) >> np.uint64(32)
        out[start:start + m] = np.searchsorted(thr, r, side="right").astype(np.uint8)
    return out


def entropy_bits(pmf: np.ndarray) -> float:
    p = np.asarray(pmf, dtype=np.float64)
    p = p[p > 0]
    return float(-(p * np.log2(p)).sum())


def laplace_pmf(alphabet: int, z: int, beta: float) -> np.ndarray:
    q = np.arange(alphabet, dtype=np.float64)
    p = np.exp(-np.abs(q - z) / beta)
    return p / p.sum()


def laplace_beta_for_entropy(alphabet: int, z: int, target_bits: float) -> float:
    lo, hi = 1e-3, 1e3
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        if entropy_bits(laplace_pmf(alphabet, z, mid)) < target_bits:
            lo = mid
        else:
            hi = mid
    return math.sqrt(lo * hi)


def peaked_geometric_pmf(alphabet: int, z: int, p0: float, rho: float = 0.5) -> np.ndarray:
    """P(z) = p0; the rest is a two-sided geometric rho^|q-z| cut to [0, alphabet)."""
    q = np.arange(alphabet, dtype=np.float64)
    w = rho ** np.abs(q - z)
    w[z] = 0.0
    if w.sum() == 0.0:
        p = np.zeros(alphabet)
        p[z] = 1.0
        return p
    p = (1.0 - p0) * w / w.sum()
    p[z] = p0
    return p


@dataclass
class Layer:
    name: str
    shape: tuple
    bitwidth: int
    zero_point: int
    scale: float
    pmf: np.ndarray
    seed: int
    channel_len: int = 0                      # 0: one scale per layer
    channel_scales: Optional[np.ndarray] = None

    @property
    def numel(self) -> int:
        return int(np.prod(self.shape))

    def symbols(self) -> np.ndarray:
        return sample_symbols(self.pmf, self.numel, self.seed)


CHANNEL_GROUP = 64        # input channels per group = streams per chunk when streams follow the input channels


def to_channel_groups(tensor: np.ndarray) -> np.ndarray:
    """A conv weight tensor [cout][cin][kh][kw] (cin a multiple of 64) in the order [cin / 64][cout][kh][kw][64]:
    with 64 streams per chunk and chunks that start on multiples of 64, stream k of every chunk holds weights of
    input channel 64 g + k only, and a wavefront-step still writes 64 consecutive elements."""
    cout, cin, kh, kw = tensor.shape
    assert cin % CHANNEL_GROUP == 0
    t = tensor.reshape(cout, cin // CHANNEL_GROUP, CHANNEL_GROUP, kh, kw)
    return np.ascontiguousarray(t.transpose(1, 0, 3, 4, 2)).reshape(-1)


def from_channel_groups(flat: np.ndarray, shape) -> np.ndarray:
    """Inverse of to_channel_groups."""
    cout, cin, kh, kw = shape
    t = np.asarray(flat).reshape(cin // CHANNEL_GROUP, cout, kh, kw, CHANNEL_GROUP)
    return np.ascontiguousarray(t.transpose(1, 0, 4, 2, 3)).reshape(cout, cin, kh, kw)


@dataclass
class ChannelLayer(Layer):
    """A conv layer whose weights follow their INPUT channel (Sec. III-B: the streams of a layer are its input
    channels): channel c has its own P(zero-point), spread evenly over [p0_low, p0_high] in a seeded random
    order, so streams differ in compressibility and the storage order matters.  symbols() returns the layer in
    storage order [cin / 64][cout][kh][kw][64]; tensor() the same weights as [cout][cin][kh][kw]."""
    p0_low: float = 0.6
    p0_high: float = 0.95

    def tensor(self) -> np.ndarray:
        cout, cin, kh, kw = self.shape
        alphabet = 1 << self.bitwidth
        order = np.argsort(splitmix64(self.seed, cin))
        p0 = self.p0_low + (self.p0_high - self.p0_low) * (order.astype(np.float64) + 0.5) / cin
        t = np.empty((cout, cin, kh, kw), dtype=np.uint8)
        for c in range(cin):
            pmf = peaked_geometric_pmf(alphabet, self.zero_point, float(p0[c]))
            t[:, c] = sample_symbols(pmf, cout * kh * kw, self.seed + 1 + c).reshape(cout, kh, kw)
        return t

    def symbols(self) -> np.ndarray:
        return to_channel_groups(self.tensor())

    @property
    def group_symbols(self) -> int:
        """Symbols of one group of 64 input channels: the chunk size that makes a stream a whole channel."""
        cout, cin, kh, kw = self.shape
        return cout * kh * kw * CHANNEL_GROUP


def channel_grouped(shapes=((128, 128, 3, 3), (512, 64, 3, 3), (256, 256, 1, 1), (64, 64, 1, 1)), table_log: int = 12,
                    seed: int = 77) -> "Workload":
    """Conv layers coded with one stream per input channel.  The layer's pmf (mixture over its channels) is only
    informational: tables come from the symbols' histogram.  chunk_sizes holds one chunk size per layer."""
    layers = []
    for i, shape in enumerate(shapes):
        b = 3 + (i % 3) * 2
        z = 1 << (b - 1)
        layers.append(ChannelLayer(f"grouped{i}", tuple(shape), b, z, 0.01 * (i + 1), peaked_geometric_pmf(1 << b, z, 0.8),
                                   BASE_SEED + 7000 * (i + 1) + seed))
    w = Workload("channel_grouped", layers, table_log, CHANNEL_GROUP, 65536, "bf16",
                 notes="streams follow the input channels; storage order [cin/64][cout][kh][kw][64]")
    w.chunk_sizes = [l.group_symbols for l in layers]
    return w


@dataclass
class Workload:
    name: str
    layers: List[Layer]
    table_log: int
    n_streams: int
    chunk_size: int
    out_dtype: str                            # "f32" | "bf16"
    notes: str = ""
    chunk_sizes: Optional[List[int]] = None   # one chunk size per layer instead of chunk_size for all
    _cache: dict = field(default_factory=dict, repr=False)

    @property
    def numel(self) -> int:
        return sum(l.numel for l in self.layers)

    def symbols(self) -> List[np.ndarray]:
        if "sym" not in self._cache:
            self._cache["sym"] = [l.symbols() for l in self.layers]
        return self._cache["sym"]

    def model_entropy_bits(self) -> float:
        """Parameter-weighted entropy of the generating distributions."""
        return sum(l.numel * entropy_bits(l.pmf) for l in self.layers) / self.numel


def resnet18_conv_shapes():
    shapes = [("conv1", (64, 3, 7, 7))]
    cin = 64
    for stage, cout in enumerate((64, 128, 256, 512), start=1):
        for block in range(2):
            c_in_block = cin if block == 0 else cout
            shapes.append((f"layer{stage}.{block}.conv1", (cout, c_in_block, 3, 3)))
            shapes.append((f"layer{stage}.{block}.conv2", (cout, cout, 3, 3)))
            if block == 0 and c_in_block != cout:
                shapes.append((f"layer{stage}.{block}.downsample", (cout, c_in_block, 1, 1)))
        cin = cout
    return shapes


def resnet50_conv_shapes():
    shapes = [("conv1", (64, 3, 7, 7))]
    cin = 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        cout = width * 4
        for block in range(blocks):
            c_in_block = cin if block == 0 else cout
            shapes.append((f"layer{stage}.{block}.conv1", (width, c_in_block, 1, 1)))
            shapes.append((f"layer{stage}.{block}.conv2", (width, width, 3, 3)))
            shapes.append((f"layer{stage}.{block}.conv3", (cout, width, 1, 1)))
            if block == 0:
                shapes.append((f"layer{stage}.{block}.downsample", (cout, c_in_block, 1, 1)))
        cin = cout
    return shapes


def resnet50_conv_geometry():
    """(name, (cout, cin, kh, kw), stride, pad, input height = width) of every conv layer of a ResNet-50 fed
    with 224 x 224 images (stride on the 3x3 convolution of a stage's first block, as in torchvision)."""
    out = [("conv1", (64, 3, 7, 7), 2, 3, 224)]
    size, cin = 56, 64                                   # after the 3x3 stride-2 max pooling
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        cout = width * 4
        for block in range(blocks):
            c_in_block = cin if block == 0 else cout
            stride = 2 if (block == 0 and stage > 1) else 1
            out.append((f"layer{stage}.{block}.conv1", (width, c_in_block, 1, 1), 1, 0, size))
            out.append((f"layer{stage}.{block}.conv2", (width, width, 3, 3), stride, 1, size))
            out.append((f"layer{stage}.{block}.conv3", (cout, width, 1, 1), 1, 0, size // stride))
            if block == 0:
                out.append((f"layer{stage}.{block}.downsample", (cout, c_in_block, 1, 1), stride, 0, size))
            size //= stride
        cin = cout
    return out


def bf16_activations(n: int, seed: int):
    """n standard normal values rounded to bfloat16 (nearest even): their 16-bit codes and their values."""
    v = np.random.default_rng(seed).standard_normal(n).astype(np.float32)
    bits = v.view(np.uint32)
    codes = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)
    return codes, (codes.astype(np.uint32) << 16).view(np.float32)


def _seed(config: int, layer: int) -> int:
    return (BASE_SEED + (config << 20) + layer) & _MASK64


def config1() -> Workload:
    """One 64x64x3x3 conv tensor, 4-bit symbols, Laplace at ~1.2 bit, one stream, fp32."""
    beta = laplace_beta_for_entropy(16, 8, 1.2)
    lay = Layer("conv", (64, 64, 3, 3), 4, 8, 0.02, laplace_pmf(16, 8, beta), _seed(1, 0))
    return Workload("single_conv_64x64x3x3", [lay], 10, 1, 36864, "f32",
                    notes=f"Laplace beta={beta:.4f}")


def config2() -> Workload:
    """ResNet-18-shaped conv stack, bitwidth U{2..6}, Laplace at 0.6-2.0 bit, 32 streams / 16384."""
    shapes = resnet18_conv_shapes()
    u = _uniform01(_seed(2, 1 << 16), 3 * len(shapes))
    layers = []
    for i, (name, shape) in enumerate(shapes):
        b = 2 + int(u[3 * i] * 5)
        z = 1 << (b - 1)
        hmax = min(2.0, 0.9 * b)
        target = 0.6 + u[3 * i + 1] * (hmax - 0.6)
        beta = laplace_beta_for_entropy(1 << b, z, target)
        scale = float(np.float32(0.005 + u[3 * i + 2] * 0.045))
        layers.append(Layer(name, shape, b, z, scale, laplace_pmf(1 << b, z, beta), _seed(2, i)))
    return Workload("resnet18_convs", layers, 11, 32, 16384, "bf16")


def config3() -> Workload:
    """ResNet-50-shaped conv stack, 1-8 bit, P(zero-point) in [0.7, 0.95] (largest layer
    gets the largest), two-sided geometric tails, 64 streams / 65536, table 2^12, bf16."""
    shapes = resnet50_conv_shapes()
    n = len(shapes)
    u = _uniform01(_seed(3, 1 << 16), 3 * n)
    p0_draws = np.sort(0.7 + 0.25 * u[0:n])
    order = np.argsort([int(np.prod(s)) for _, s in shapes], kind="stable")
    p0 = np.empty(n)
    p0[order] = p0_draws                       # rank-matched: biggest layer, biggest p0
    layers = []
    for i, (name, shape) in enumerate(shapes):
        b = 1 + int(u[n + i] * 8)
        z = 1 << (b - 1)
        scale = float(np.float32(0.005 + u[2 * n + i] * 0.045))
        layers.append(Layer(name, shape, b, z, scale,
                            peaked_geometric_pmf(1 << b, z, float(p0[i])), _seed(3, i)))
    return Workload("resnet50_convs", layers, 12, 64, 65536, "bf16")


def resnet50_odd_bins() -> Workload:
    """ResNet-50-shaped conv stack with the alphabets the paper describes (Sec. II-B, III-C): an odd
    number of bins with the zero-point in the middle, 31 bins for the smaller half of the layers down
    to 13 bins for the largest ones, mass concentrated on the zero-point so that the set averages
    below one bit per weight.  Used by the table-size study; any table of 64 states or more can code it."""
    shapes = resnet50_conv_shapes()
    n = len(shapes)
    u = _uniform01(_seed(6, 1 << 16), 2 * n)
    sizes = np.array([int(np.prod(s)) for _, s in shapes])
    rank = np.empty(n, dtype=int)
    rank[np.argsort(sizes, kind="stable")] = np.arange(n)
    p0_draws = np.sort(0.72 + 0.22 * u[0:n])
    layers = []
    for i, (name, shape) in enumerate(shapes):
        frac = rank[i] / max(n - 1, 1)                       # 0 smallest layer .. 1 largest
        bins = 31 if frac < 0.5 else int(31 - 18 * (frac - 0.5) / 0.5) | 1   # odd, 31 .. 13
        z = (bins - 1) // 2
        scale = float(np.float32(0.005 + u[n + i] * 0.045))
        layers.append(Layer(name, shape, 5, z, scale,
                            peaked_geometric_pmf(bins, z, float(p0_draws[rank[i]])), _seed(6, i)))
    return Workload("resnet50_odd_bins", layers, 8, 64, 65536, "bf16")


def config4(n_blocks: int = 32, d_model: int = 4096, d_ff: int = 11008) -> Workload:
    """Transformer-sized linear stack: per block 4 of d x d and 3 of d x d_ff, 4-bit,
    Laplace at ~2.5 bit, per-output-channel fp32 scales, 64 streams / 262144."""
    beta = laplace_beta_for_entropy(16, 8, 2.5)
    pmf = laplace_pmf(16, 8, beta)
    layers = []
    i = 0
    for blk in range(n_blocks):
        for j in range(7):
            rows, cols = (d_model, d_model) if j < 4 else (d_model, d_ff)
            su = _uniform01(_seed(4, (1 << 16) + i), rows)
            scales = (0.005 + 0.045 * su).astype(np.float32)
            layers.append(Layer(f"block{blk}.w{j}", (rows, cols), 4, 8, float(scales[0]), pmf,
                                _seed(4, i), channel_len=cols, channel_scales=scales))
            i += 1
    return Workload(f"linear_stack_{n_blocks}x", layers, 12, 64, 262144, "bf16",
                    notes=f"Laplace beta={beta:.4f}")


def tiny(seed: int = 7, n: int = 5000, bitwidth: int = 4, n_streams: int = 64,
         chunk_size: int = 2048, table_log: int = 10, p0: float = 0.8,
         out_dtype: str = "bf16") -> Workload:
    """Small ragged case for quick checks."""
    z = 1 << (bitwidth - 1)
    lay = Layer("tiny", (n,), bitwidth, z, 0.0125,
                peaked_geometric_pmf(1 << bitwidth, z, p0), _seed(15, seed))
    return Workload("tiny", [lay], table_log, n_streams, chunk_size, out_dtype)
