"""Pins of the convolution oracle (fused decode + conv stretch): it must agree with things it does
not contain — a library convolution, a matrix product, a hand-checkable shift, plain loops."""
import numpy as np
import pytest

from oracle import conv_oracle as CO


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("B,H,W,Cin,Cout,k,stride,pad", [
    (2, 9, 7, 5, 4, 3, 1, 1), (1, 10, 10, 3, 6, 7, 2, 3), (2, 8, 8, 8, 16, 1, 1, 0),
    (1, 9, 9, 4, 4, 1, 2, 0), (1, 11, 6, 2, 3, 3, 2, 1), (1, 5, 5, 1, 1, 5, 1, 0),
])
def test_against_the_library_convolution(B, H, W, Cin, Cout, k, stride, pad):
    torch = pytest.importorskip("torch")
    x = _rand((B, H, W, Cin), 1)
    w = _rand((Cout, k, k, Cin), 2)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2),
                                      stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
    got = CO.conv2d_nhwc(x, w, stride, pad)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_pointwise_convolution_is_a_matrix_product():
    x = _rand((3, 4, 5, 7), 3)
    w = _rand((6, 1, 1, 7), 4)
    want = x.reshape(-1, 7) @ w.reshape(6, 7).T
    np.testing.assert_allclose(CO.conv2d_nhwc(x, w, 1, 0).reshape(-1, 6), want, rtol=1e-13, atol=1e-13)


def test_one_hot_tap_shifts_the_image():
    # a 3x3 kernel that is 1 at tap (r, s) = (0, 2) for channel pair (o, c) = (1, 0): with pad 1 the
    # output pixel (h, w) of channel 1 is input pixel (h - 1, w + 1) of channel 0, zero outside
    x = _rand((1, 6, 6, 2), 5)
    w = np.zeros((2, 3, 3, 2))
    w[1, 0, 2, 0] = 1.0
    y = CO.conv2d_nhwc(x, w, 1, 1)
    assert np.all(y[..., 0] == 0)
    want = np.zeros((6, 6))
    want[1:, :5] = x[0, :5, 1:, 0]
    np.testing.assert_array_equal(y[0, :, :, 1], want)


def test_plain_loops_on_a_tiny_case():
    B, H, W, Cin, Cout, k, stride, pad = 1, 5, 4, 2, 3, 3, 2, 1
    x = _rand((B, H, W, Cin), 6)
    w = _rand((Cout, k, k, Cin), 7)
    Ho, Wo = CO.out_size(H, k, stride, pad), CO.out_size(W, k, stride, pad)
    assert (Ho, Wo) == (3, 2)
    want = np.zeros((B, Ho, Wo, Cout))
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for o in range(Cout):
                    for r in range(k):
                        for s in range(k):
                            h, v = ho * stride - pad + r, wo * stride - pad + s
                            if 0 <= h < H and 0 <= v < W:
                                for c in range(Cin):
                                    want[b, ho, wo, o] += x[b, h, v, c] * w[o, r, s, c]
    np.testing.assert_allclose(CO.conv2d_nhwc(x, w, stride, pad), want, rtol=1e-13, atol=1e-13)


def test_samples_equal_the_whole_tensor():
    x = _rand((2, 7, 8, 3), 8)
    w = _rand((5, 3, 3, 3), 9)
    y = CO.conv2d_nhwc(x, w, 2, 1)
    rng = np.random.default_rng(10)
    where = np.stack([rng.integers(0, d, 40) for d in y.shape], axis=1)
    got = CO.conv2d_nhwc_samples(x, w, 2, 1, where)
    np.testing.assert_allclose(got, y[tuple(where.T)], rtol=1e-12, atol=1e-12)


def test_dequantized_weights_follow_the_zero_point_rule():
    q = np.array([0, 3, 4, 7], dtype=np.uint8)
    w = CO.dequantized_weights(q, 4, 0.25, (4,))
    np.testing.assert_array_equal(w, [-1.0, -0.25, 0.0, 0.75])      # exact: 0.25 is a power of two
    assert CO.dequantized_weights(q, 4, 0.1, (4,))[2] == 0.0        # the zero-point decodes to zero (Sec. II-B)
