"""The seeded input generator: determinism, slice consistency, distribution, bf16 rounding."""
import numpy as np

from synth import (CONFIGS, K_ID, Q_ID, V_ID, bf16_bits_to_f32, f32_to_bf16_bits, gen_qkv, gen_tensor)


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.140625, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    # 1+2^-8 is a tie between 1.0 (even) and 1+2^-7; 1+3*2^-8 a tie between 1+2^-7 (odd) and 1+2^-6 (even)
    want = np.array([0x3F80, 0x3F80, 0x3F82, 0xBF80, 0x4049, 0x3F81], dtype=np.uint16)
    assert np.array_equal(f32_to_bf16_bits(x), want)
    assert np.array_equal(f32_to_bf16_bits(bf16_bits_to_f32(want)), want)


def test_deterministic_and_slices_carry_the_same_bits():
    full = gen_tensor(5, K_ID, (1, 3, 300, 64), unit_rms=True)
    again = gen_tensor(5, K_ID, (1, 3, 300, 64), unit_rms=True, chunk_rows=37)
    assert np.array_equal(full, again)
    part = gen_tensor(5, K_ID, (1, 3, 300, 64), unit_rms=True, heads=(1, 3), rows=(10, 211))
    assert np.array_equal(part, full[:, 1:3, 10:211])


def test_tensors_and_seeds_differ():
    a = gen_tensor(5, Q_ID, (1, 1, 64, 64), unit_rms=False)
    assert not np.array_equal(a, gen_tensor(5, K_ID, (1, 1, 64, 64), unit_rms=False))
    assert not np.array_equal(a, gen_tensor(6, Q_ID, (1, 1, 64, 64), unit_rms=False))
    assert not np.array_equal(gen_tensor(5, V_ID, (1, 1, 64, 64), unit_rms=False),
                              gen_tensor(5, K_ID, (1, 1, 64, 64), unit_rms=False))


def test_standard_normal_moments():
    x = bf16_bits_to_f32(gen_tensor(11, V_ID, (1, 2, 8192, 64), unit_rms=False)).astype(np.float64)
    n = x.size
    assert abs(x.mean()) < 5 / np.sqrt(n)
    assert abs(x.var() - 1.0) < 0.01
    assert abs((x ** 4).mean() - 3.0) < 0.05
    assert abs(np.corrcoef(x.ravel()[:-1], x.ravel()[1:])[0, 1]) < 5 / np.sqrt(n)


def test_unit_rms_rows():
    x = bf16_bits_to_f32(gen_tensor(12, Q_ID, (1, 2, 512, 128), unit_rms=True)).astype(np.float64)
    rms = np.sqrt((x * x).mean(axis=-1))
    assert np.abs(rms - 1.0).max() < 4e-3          # bf16 rounding of a unit-RMS fp32 row


def test_config_shapes():
    assert CONFIGS[1].Sq == 4 * 16 * 16 and CONFIGS[2].Sq == 8 * 30 * 40
    assert CONFIGS[3].Skv == 33 * 34 * 60 + 256 == 67576 and CONFIGS[3].kv_valid_len == 67476
    assert CONFIGS[4].Sq == 33 * 45 * 80 + 256 == 119056 and CONFIGS[4].heads_per_group == 3
    c5 = CONFIGS[5]
    assert c5.query_ranges == ((0, 47622), (47622, 41669), (89291, 29765))
    assert sum(n for _, n in c5.query_ranges) == c5.Sq
    assert c5.key_chunks == tuple((i * 29764, 29764) for i in range(4))
    assert CONFIGS[4].flops == 4 * 119056 ** 2 * 128 * 24
    q, k, v = gen_qkv(CONFIGS[1].seed, 1, 2, 16, 32, 64, unit_rms=False)
    assert q.shape == (1, 2, 16, 64) and k.shape == v.shape == (1, 2, 32, 64) and q.dtype == np.uint16
