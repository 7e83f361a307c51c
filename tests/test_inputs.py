"""The seeded generators: determinism, ranges, moments, and bf16 rounding."""
import numpy as np

from paper_2505_02146_amd import inputs


def test_splitmix64_known_values():
    # First outputs of SplitMix64 from state 0, as published with the reference generator
    # (Vigna, xoshiro/splitmix64.c test vectors): the finaliser applied to 1*golden, 2*golden, ...
    got = inputs._splitmix64(np.array([0], dtype=np.uint64))[0]
    assert int(got) == 0xE220A8397B1DCDAF


def test_deterministic_and_chunk_independent():
    a = inputs.normal((1000,), 5, 1)
    b = inputs.normal((10, 100), 5, 1).reshape(-1)
    assert np.array_equal(a, b)
    big = inputs.uniform_pm1(((1 << 22) + 5,), 1, 2)
    assert np.array_equal(big[:100], inputs.uniform_pm1((100,), 1, 2))
    assert not np.array_equal(inputs.normal((100,), 5, 1), inputs.normal((100,), 5, 2))
    assert not np.array_equal(inputs.normal((100,), 5, 1), inputs.normal((100,), 6, 1))


def test_moments_and_ranges():
    u = inputs.uniform_pm1((200000,), 0, 1).astype(np.float64)
    assert u.min() >= -1.0 and u.max() < 1.0
    assert abs(u.mean()) < 0.01 and abs(u.var() - 1 / 3) < 0.01
    z = inputs.normal((200000,), 0, 1, 0.125).astype(np.float64)
    assert abs(z.mean()) < 0.002 and abs(z.std() - 0.125) < 0.002
    assert abs(np.mean(z ** 4) / z.var() ** 2 - 3.0) < 0.1
    i = inputs.int8_uniform((200000,), 0, 1)
    assert i.min() == -128 and i.max() == 127 and abs(i.astype(np.float64).mean() + 0.5) < 0.6
    s = inputs.small_integers((10000,), 0, 1)
    assert s.min() == -8 and s.max() == 8 and np.array_equal(s, np.round(s))


def test_bf16_round_to_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0], np.float32)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even): goes up
    want = np.array([0x3F80, 0x3F80, 0x3F81, 0x3F82, 0xC020, 0x0000], np.uint16)
    assert np.array_equal(inputs.to_bf16_bits(f), want)
    back = inputs.bf16_bits_to_f32(want)
    assert np.array_equal(back, np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0], np.float32))
    x = inputs.normal((5000,), 1, 1)
    r = inputs.bf16_bits_to_f32(inputs.to_bf16_bits(x))
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_workload_shapes():
    w = inputs.workload("gemm_f32_256")
    assert w["A"].shape == (256, 256) and w["A"].dtype == np.float32
    w = inputs.workload("bgemm_bf16_qk")
    assert w["A"].shape == (96, 512, 64) and w["B"].shape == (96, 512, 64) and w["A"].dtype == np.uint16
