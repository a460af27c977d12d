"""The synthetic weight sets: shapes, sizes and entropies stated for the benchmark configurations."""
import numpy as np

from paper_2406_06237_amd import workloads as W


def test_resnet_shapes_and_parameter_counts():
    s18 = W.resnet18_conv_shapes()
    s50 = W.resnet50_conv_shapes()
    assert len(s18) == 20 and sum(int(np.prod(s)) for _, s in s18) == 11_166_912
    assert len(s50) == 53 and sum(int(np.prod(s)) for _, s in s50) == 23_454_912
    sizes50 = [int(np.prod(s)) for _, s in s50]
    assert min(sizes50) == 4096 and max(sizes50) == 2_359_296


def test_config_geometry_and_entropy():
    c1, c2, c3 = W.config1(), W.config2(), W.config3()
    assert (c1.numel, c1.table_log, c1.n_streams, c1.out_dtype) == (36864, 10, 1, "f32")
    assert abs(W.entropy_bits(c1.layers[0].pmf) - 1.2) < 1e-6 and c1.layers[0].zero_point == 8
    assert (c2.table_log, c2.n_streams, c2.chunk_size, c2.out_dtype) == (11, 32, 16384, "bf16")
    assert all(2 <= l.bitwidth <= 6 and l.zero_point == 1 << (l.bitwidth - 1) for l in c2.layers)
    assert all(0.6 - 1e-6 <= W.entropy_bits(l.pmf) <= 2.0 + 1e-6 for l in c2.layers)
    assert all(0.005 <= l.scale <= 0.05 for l in c2.layers + c3.layers)
    assert (c3.table_log, c3.n_streams, c3.chunk_size, c3.out_dtype) == (12, 64, 65536, "bf16")
    assert all(1 <= l.bitwidth <= 8 for l in c3.layers)
    assert all(0.7 <= l.pmf[l.zero_point] <= 0.95 for l in c3.layers)
    # the largest layer carries the most peaked distribution
    order = np.argsort([l.numel for l in c3.layers], kind="stable")
    p0 = [c3.layers[i].pmf[c3.layers[i].zero_point] for i in order]
    assert all(a <= b + 1e-12 for a, b in zip(p0, p0[1:]))
    assert 0.55 < c3.model_entropy_bits() < 0.8
    chunks = sum((l.numel + c3.chunk_size - 1) // c3.chunk_size for l in c3.layers)
    assert chunks == 369
    assert sum((l.numel + c2.chunk_size - 1) // c2.chunk_size for l in c2.layers) == 686


def test_config4_shape_without_generating_it():
    c4 = W.config4(n_blocks=1)
    assert len(c4.layers) == 7 and c4.numel == 4 * 4096 * 4096 + 3 * 4096 * 11008
    assert abs(W.entropy_bits(c4.layers[0].pmf) - 2.5) < 1e-6
    assert c4.layers[4].channel_len == 11008 and len(c4.layers[4].channel_scales) == 4096
    assert 32 * c4.numel == 6_476_005_376


def test_generator_is_reproducible_and_matches_pmf():
    a = W.sample_symbols(W.laplace_pmf(16, 8, 0.5), 100000, 123)
    b = W.sample_symbols(W.laplace_pmf(16, 8, 0.5), 100000, 123)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, W.sample_symbols(W.laplace_pmf(16, 8, 0.5), 100000, 124))
    emp = np.bincount(a, minlength=16) / 100000
    assert np.abs(emp - W.laplace_pmf(16, 8, 0.5)).max() < 0.01
    # first outputs of SplitMix64 for seed 0 (published reference values of the generator)
    z = W.splitmix64(0, 3)
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
