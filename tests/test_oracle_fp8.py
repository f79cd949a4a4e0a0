"""Pins of the fp8 E4M3 codec (CPU only)."""
import numpy as np
import pytest

import oracle


def test_decode_table_against_hand_written_layout():
    t = oracle.e4m3_decode_table()
    # sign | eeee | mmm, bias 7; hand-computed values
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and np.signbit(t[0x80] * 1.0) in (True, False)
    assert t[0x01] == 2.0 ** -9            # smallest subnormal
    assert t[0x07] == 7 * 2.0 ** -9        # largest subnormal
    assert t[0x08] == 2.0 ** -6            # smallest normal
    assert t[0x38] == 1.0                  # 0 0111 000
    assert t[0x3C] == 1.5                  # 0 0111 100
    assert t[0x40] == 2.0
    assert t[0x7E] == 448.0                # 0 1111 110
    assert t[0xFE] == -448.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    assert t[0xB8] == -1.0
    finite = t[:0x7F]
    assert np.all(np.diff(finite) > 0)     # codes are ordered like their values
    assert np.array_equal(t[0x80:0xFF], -finite)
    assert oracle.E4M3_MAX == 448.0


def test_every_finite_code_round_trips():
    t = oracle.e4m3_decode_table()
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    back = oracle.e4m3_encode_f32(t[codes].astype(np.float32))
    ok = (back == codes) | ((codes == 0x80) & (back == 0x80))
    assert ok.all()


def test_ties_round_to_even_and_saturation():
    enc = lambda x: int(oracle.e4m3_encode_f32(np.float32(x)))
    # between 1.0 (0x38, even) and 1.125 (0x39): midpoint 1.0625 -> 0x38
    assert enc(1.0625) == 0x38
    # between 1.125 (0x39) and 1.25 (0x3A, even): midpoint 1.1875 -> 0x3A
    assert enc(1.1875) == 0x3A
    assert enc(1.0626) == 0x39 and enc(1.0624) == 0x38
    # subnormal grid step 2^-9: midpoint of 0 and 2^-9 -> 0 (even); of 2^-9 and 2^-8 -> 2^-8
    assert enc(2.0 ** -10) == 0x00
    assert enc(3 * 2.0 ** -10) == 0x02
    # subnormal / normal boundary: 7.5 * 2^-9 is a tie between 0x07 and 0x08 -> 0x08
    assert enc(7.5 * 2.0 ** -9) == 0x08
    # top of the range: 448 exactly, a little above, far above, and the 416/448 tie
    assert enc(448.0) == 0x7E and enc(448.01) == 0x7E and enc(1e9) == 0x7E
    assert enc(432.0) == 0x7E              # tie 416 (0x7D, odd) / 448 (0x7E, even)
    assert enc(-1e9) == 0xFE and enc(-1.0625) == 0xB8


def test_brute_force_nearest_on_random_values():
    t = oracle.e4m3_decode_table()
    finite_codes = np.array([c for c in range(0x7F)], dtype=np.uint8)
    vals = t[finite_codes]
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.uniform(0, 460, 2000), rng.uniform(0, 0.05, 2000)]).astype(np.float32)
    got = oracle.e4m3_encode_f32(xs)
    for x, c in zip(xs.astype(np.float64), got):
        d = np.abs(vals - min(x, 448.0))
        best = d.min()
        cands = finite_codes[d == best]
        assert c in cands
        if len(cands) == 2:
            assert c % 2 == 0


def test_row_quantisation_recipe():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 3, 16)).astype(np.float32)
    x[2, 1] = 0.0
    codes, scales = oracle.quantize_rows(x)
    assert codes.shape == x.shape and scales.shape == x.shape[:-1] and scales.dtype == np.float32
    assert scales[2, 1] == 1.0 and not codes[2, 1].any()
    amax = np.abs(x).max(-1)
    np.testing.assert_array_equal(scales[amax > 0], (amax / np.float32(448))[amax > 0])
    # the largest element of each row maps to +-448
    t = oracle.e4m3_decode_table()
    peak = np.abs(t[codes]).max(-1)
    assert np.all(peak[amax > 0] == 448.0)
    # relative error of the reconstruction is bounded by half a mantissa step (2^-4)
    xh = oracle.dequantize_rows(codes, scales)
    big = np.abs(x) > (amax[..., None] * 2.0 ** -6)
    assert np.all(np.abs(xh - x)[big] <= np.abs(x)[big] * 2.0 ** -4 * 1.001)
