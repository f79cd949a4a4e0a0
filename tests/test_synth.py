"""Seeded input generators (CPU only)."""
import numpy as np

from paper_2410_10819_amd import synth


def test_bf16_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even (1.0)
    assert bits[0] == 0x3F80 and bits[1] == 0x3F80
    # 1.01171875 = 1 + 3 * 2^-8 is a tie between 1+2^-7 (odd) and 1+2^-6 (even)
    assert bits[2] == 0x3F82
    assert synth.bf16_bits_to_f32(bits)[3] == -2.5
    back = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(bits))
    assert np.array_equal(back, bits)


def test_counter_generator_is_position_addressable_and_normal():
    a = synth.counter_bf16(5, 2, synth.TENSOR_K, 1, 0, 300, 4, 64)
    b = synth.counter_bf16(5, 2, synth.TENSOR_K, 1, 123, 10, 4, 64)
    assert np.array_equal(a[123:133], b)
    c = synth.counter_bf16(5, 2, synth.TENSOR_V, 1, 0, 300, 4, 64)
    assert not np.array_equal(a, c)
    f = synth.bf16_bits_to_f64(a)
    assert abs(f.mean()) < 0.02 and abs(f.std() - 1.0) < 0.02


def test_retrieval_mask_ratio():
    m = synth.retrieval_mask(0, 32, 8, 0.5)
    assert m.shape == (32, 8) and (m.sum(1) == 4).all()
    m2 = synth.retrieval_mask(0, 1, 32, 0.25)
    assert m2.sum() == 8
    assert np.array_equal(m, synth.retrieval_mask(0, 32, 8, 0.5))
