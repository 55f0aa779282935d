"""Pins of the pack oracle."""
import numpy as np

from oracle import pack as K
from synth.inputs import bf16_bits_to_f32, f32_to_bf16_bits


def test_rounding_matches_bit_level_routine():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * np.float32(s) for s in (1e-3, 1.0, 300.0)])
    # exact ties: values half way between two bf16 neighbours
    base = bf16_bits_to_f32(rng.integers(0x3000, 0x4800, 5000).astype(np.uint16))
    ties = (base.view(np.uint32) | np.uint32(0x8000)).view(np.float32)
    x = np.concatenate([x, ties, -ties])
    want = bf16_bits_to_f32(f32_to_bf16_bits(x)).astype(np.float64)
    assert np.array_equal(K.round_to_bf16(x), want)


def test_placement():
    B, S, H, d = 2, 5, 3, 4
    b, s, h, c = np.meshgrid(np.arange(B), np.arange(S), np.arange(H), np.arange(d), indexing="ij")
    x = (b * 64 + s * 8 + h * 2 + (c == 0)).astype(np.float64)     # small integers: exact in bf16
    y = K.pack_heads(x, unit_rms=False)
    assert y.shape == (B, H, S, d)
    for bb in range(B):
        for hh in range(H):
            for ss in range(S):
                assert np.array_equal(y[bb, hh, ss], x[bb, ss, hh])


def test_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 64, 4, 128)) * rng.uniform(0.01, 50, (1, 64, 4, 1))
    y = K.pack_heads(x, unit_rms=True)
    rms = np.sqrt(np.mean(y * y, axis=-1))
    assert np.all(np.abs(rms - 1) < 2e-3)                           # bf16 rounding, averaged over 128 values
    assert np.array_equal(K.pack_heads(x * 8.0, True), y)           # power of two: exact
    assert np.array_equal(K.pack_heads(x * 0.25, True), y)
    assert np.array_equal(K.pack_heads(-x, True), -y)
    # direction is kept: y is x/|x| * sqrt(d) up to rounding
    ref = x / np.linalg.norm(x, axis=-1, keepdims=True) * np.sqrt(128)
    assert np.max(np.abs(y.transpose(0, 2, 1, 3) - ref) / np.maximum(np.abs(ref), 2.0 ** -6)) <= 2.0 ** -8


def test_zero_vector_stays_zero():
    x = np.zeros((1, 2, 2, 8))
    x[0, 1, 1] = 3.0
    y = K.pack_heads(x, True)
    assert np.all(y[0, :, 0] == 0) and np.all(y[0, 0, 1] == 0) and np.all(y[0, 1, 1] == 1.0)


def test_premul_is_applied_before_the_single_rounding():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((1, 16, 2, 64))
    c = 0.1275174
    y = K.pack_heads(x, True, premul=c)
    exact = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) * c
    assert np.array_equal(y, K.round_to_bf16(exact.transpose(0, 2, 1, 3)))
    assert np.array_equal(K.pack_heads(x, False, premul=0.5), 0.5 * K.pack_heads(x, False))     # power of two: exact
    # not the same as rounding first and scaling afterwards
    assert not np.array_equal(y, K.round_to_bf16(K.pack_heads(x, True) * c))
