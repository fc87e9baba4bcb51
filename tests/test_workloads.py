"""The seeded generators: published SplitMix64 outputs, distribution moments, determinism."""
import numpy as np

from workloads import configs, rng


def test_splitmix64_reference_outputs():
    # first three outputs of the SplitMix64 generator seeded with 0 (Steele, Lea, Flood 2014;
    # the values printed by the public-domain reference implementation)
    assert [int(v) for v in rng.splitmix64(0, 3)] == [
        0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert int(rng.splitmix64(0, 1, offset=2)[0]) == 0x06C45D188009454F


def test_moments_and_ranges():
    u = rng.uniform(1, (1 << 18,), -1.0, 1.0)
    assert -1.0 <= u.min() and u.max() <= 1.0 and abs(u.mean()) < 5e-3 and abs(u.var() - 1 / 3) < 5e-3
    z = rng.normal(2, (1 << 18,), 1.0, 3.0)
    assert abs(z.mean() - 1.0) < 1e-2 and abs(z.var() - 3.0) < 3e-2
    # kurtosis of a normal is 3: catches a broken Box-Muller pairing
    zc = (z - z.mean()) / z.std()
    assert abs((zc ** 4).mean() - 3.0) < 0.05


def test_configs_are_deterministic_and_sets_differ():
    a = configs.SoftmaxWorkload(rows=4, cols=64).make()["x"]
    b = configs.SoftmaxWorkload(rows=4, cols=64).make()["x"]
    c = configs.SoftmaxWorkload(rows=4, cols=64).make(set_index=1)["x"]
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    d = configs.ConvWorkload(N=1, H=8, W=8, C=64, K=4).make()
    w = rng.bf16_bits_to_f32(d["w_bf16"])
    assert abs(w.var() - 2.0 / 576) < 4e-4


def test_bf16_roundtrip():
    f = np.array([1.0, -0.5, 3.140625, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8], dtype=np.float32)
    back = rng.bf16_bits_to_f32(rng.f32_to_bf16_bits(f))
    assert np.array_equal(back, np.array([1.0, -0.5, 3.140625, 1.0, 1 + 2.0 ** -6], dtype=np.float32))
