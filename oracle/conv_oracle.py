"""CPU oracle of the fused decode + convolution stretch (numpy, fp64).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg; the GPU library never imports it.

What the fused path must deliver is an ordinary 2-D convolution (cross-correlation, as in every
deep-learning framework) of an activation tensor with the weights the decoder reconstructs,
w = scale * (q - z) (Sec. II-B).  The oracle is that definition written out in fp64:

    y[b, ho, wo, o] = sum_{r, s, c} x[b, ho*stride - pad + r, wo*stride - pad + s, c] * w[o, r, s, c]

with x taken as zero outside the image.  Layouts: activations and outputs are NHWC, weights are
[Cout][kh][kw][Cin] (the order in which a layer's symbols are entropy-coded for this path).
"""
from __future__ import annotations

import numpy as np


def out_size(n: int, k: int, stride: int, pad: int) -> int:
    return (n + 2 * pad - k) // stride + 1


def dequantized_weights(symbols: np.ndarray, zero_point: int, scale: float, shape) -> np.ndarray:
    """Sec. II-B: w = scale * (q - z), the scale being the layer's float32 value, in fp64."""
    q = symbols.astype(np.int64) - int(zero_point)
    return (float(np.float32(scale)) * q.astype(np.float64)).reshape(shape)


def conv2d_nhwc(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Whole output tensor.  One matrix product per kernel tap (r, s), added up in fp64."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, H, W, Cin = x.shape
    Cout, kh, kw, Cin2 = w.shape
    assert Cin == Cin2
    Ho, Wo = out_size(H, kh, stride, pad), out_size(W, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.zeros((B, Ho, Wo, Cout), dtype=np.float64)
    for r in range(kh):
        for s in range(kw):
            patch = xp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :]
            y += patch.reshape(-1, Cin).dot(w[:, r, s, :].T).reshape(B, Ho, Wo, Cout)
    return y


def conv2d_nhwc_samples(x: np.ndarray, w: np.ndarray, stride: int, pad: int, where: np.ndarray) -> np.ndarray:
    """Single outputs y[b, ho, wo, o] for the rows (b, ho, wo, o) of `where`, one dot product each."""
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    out = np.zeros(len(where), dtype=np.float64)
    for i, (b, ho, wo, o) in enumerate(np.asarray(where, dtype=np.int64)):
        acc = 0.0
        for r in range(kh):
            h = ho * stride - pad + r
            if h < 0 or h >= H:
                continue
            for s in range(kw):
                v = wo * stride - pad + s
                if v < 0 or v >= W:
                    continue
                acc += float(np.dot(x[b, h, v, :].astype(np.float64), w[o, r, s, :].astype(np.float64)))
        out[i] = acc
    return out
