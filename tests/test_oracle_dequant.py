"""Pins for the oracle's dequantiser (Sec. II-B: uniform quantizer with a zero-point).

w = scale * (q - z) with a single binary32 rounding; bf16 is round-to-nearest-even of w.
Checked against an fp64 evaluation (the product of an fp32 and a 9-bit integer is exact in
fp64, so rounding it once to fp32 is the IEEE result), against torch's bf16 conversion, and
on hand-built tie cases.
"""
import numpy as np
import pytest
import torch


def _bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("z,scale", [(8, 0.02), (128, 0.0123456), (1, 0.05), (0, 3.0e-3), (255, 0.7),
                                      (8, float(np.float32(1e-40))), (77, float(np.float32(3.1e38 / 255)))])
def test_dequant_matches_fp64_then_single_rounding(orc, z, scale):
    q = np.arange(256, dtype=np.uint8)
    s32 = np.float32(scale)
    expect32 = (np.float64(s32) * (q.astype(np.float64) - z)).astype(np.float32)
    got32 = orc.dequant(q, z, float(s32), "f32")
    assert np.array_equal(_bits(got32), _bits(expect32))
    got16 = orc.dequant(q, z, float(s32), "bf16")
    t = torch.from_numpy(expect32.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got16, t)


def test_zero_point_maps_to_positive_zero(orc):
    for z in (0, 1, 8, 128, 255):
        q = np.array([z], dtype=np.uint8)
        assert _bits(orc.dequant(q, z, 0.02, "f32"))[0] == 0
        assert orc.dequant(q, z, 0.02, "bf16")[0] == 0


def test_bf16_ties_round_to_even(orc):
    q = np.array([1, 2], dtype=np.uint8)           # q - z = +1, +2 with z = 0
    for pattern, expect in ((0x3F808000, 0x3F80), (0x3F818000, 0x3F82), (0x3F808001, 0x3F81),
                            (0x3F807FFF, 0x3F80), (0x3F81FFFF, 0x3F82)):
        scale = float(np.array([pattern], dtype=np.uint32).view(np.float32)[0])
        got = orc.dequant(q, 0, scale, "bf16")
        assert got[0] == expect
        assert got[1] == expect + 0x0080          # times two: exponent + 1, same mantissa
    neg = orc.dequant(np.array([0], dtype=np.uint8), 1, float(np.array([0x3F818000], np.uint32).view(np.float32)[0]), "bf16")
    assert neg[0] == 0xBF82


def test_per_channel_scales(orc):
    rng = np.random.default_rng(3)
    q = rng.integers(0, 16, size=6 * 50, dtype=np.uint8)
    scales = rng.uniform(0.005, 0.05, size=6).astype(np.float32)
    got = orc.dequant(q, 8, 0.0, "f32", channel_len=50, channel_scales=scales)
    expect = (np.repeat(scales.astype(np.float64), 50) * (q.astype(np.float64) - 8)).astype(np.float32)
    assert np.array_equal(_bits(got), _bits(expect))
