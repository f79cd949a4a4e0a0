"""The oracle's 4-bit KV codec against values worked out by hand and its invariants."""
import numpy as np

import oracle


def test_hand_computed_rows():
    # lo = 0, hi = 15 -> scale 1: integers are their own codes; halves round to even
    x = np.array([[0.0, 15.0, 1.0, 2.5, 3.5, 7.49, 7.51, 14.5]], dtype=np.float32)
    code, scale, lo = oracle.quantize_rows_int4(x)
    assert scale[0] == 1.0 and lo[0] == 0.0
    assert code[0].tolist() == [0, 15, 1, 2, 4, 7, 8, 14]
    # lo = -3, hi = 4.5 -> scale 0.5: code = (x + 3) / 0.5
    y = np.array([[-3.0, 4.5, -2.75, -2.25, 0.0, 1.0]], dtype=np.float32)
    code, scale, lo = oracle.quantize_rows_int4(y)
    assert scale[0] == 0.5 and lo[0] == -3.0
    assert code[0].tolist() == [0, 15, 0, 2, 6, 8]          # 0.5 -> 0 (even), 1.5 -> 2 (even)
    deq = oracle.dequantize_rows_int4(code, scale, lo)
    assert deq[0].tolist() == [-3.0, 4.5, -3.0, -2.0, 0.0, 1.0]


def test_constant_and_zero_rows():
    x = np.full((2, 8), 1.25, dtype=np.float32)
    x[1] = 0.0
    code, scale, lo = oracle.quantize_rows_int4(x)
    assert (code == 0).all() and (scale == 1.0).all() and lo.tolist() == [1.25, 0.0]
    assert np.array_equal(oracle.dequantize_rows_int4(code, scale, lo), x.astype(np.float64))


def test_extremes_error_bound_and_monotonicity():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((500, 128)).astype(np.float32)
    code, scale, lo = oracle.quantize_rows_int4(x)
    assert code.min() == 0 and code.max() == 15
    rows = np.arange(500)
    assert (code[rows, x.argmin(1)] == 0).all() and (code[rows, x.argmax(1)] == 15).all()
    err = np.abs(oracle.dequantize_rows_int4(code, scale, lo) - x.astype(np.float64))
    assert (err <= scale[:, None].astype(np.float64) * 0.5 * (1 + 1e-5)).all()
    order = np.argsort(x, axis=1)
    assert (np.diff(np.take_along_axis(code.astype(int), order, axis=1), axis=1) >= 0).all()


def test_packing_layout():
    codes = np.array([[1, 2, 3, 4, 15, 0, 9, 10]], dtype=np.uint8)
    packed = oracle.pack_int4(codes)
    assert packed[0].tolist() == [0x21, 0x43, 0x0F, 0xA9]
    assert np.array_equal(oracle.unpack_int4(packed), codes)


def test_int8_hand_computed_rows_and_invariants():
    # lo = 0, hi = 255 -> scale 1: integers are their own codes; halves round to even
    x = np.array([[0.0, 255.0, 1.0, 2.5, 3.5, 127.49, 127.51, 254.5]], dtype=np.float32)
    code, scale, lo = oracle.quantize_rows_int8(x)
    assert scale[0] == 1.0 and lo[0] == 0.0
    assert code[0].tolist() == [0, 255, 1, 2, 4, 127, 128, 254]
    # lo = -1, hi = 126.5 -> scale 0.5
    y = np.array([[-1.0, 126.5, -0.75, -0.25, 0.0, 63.0]], dtype=np.float32)
    code, scale, lo = oracle.quantize_rows_int8(y)
    assert scale[0] == 0.5 and lo[0] == -1.0
    assert code[0].tolist() == [0, 255, 0, 2, 2, 128]
    assert oracle.dequantize_rows_int8(code, scale, lo)[0].tolist() == [-1.0, 126.5, -1.0, 0.0, 0.0, 63.0]
    const = np.full((1, 8), -2.5, dtype=np.float32)
    code, scale, lo = oracle.quantize_rows_int8(const)
    assert (code == 0).all() and scale[0] == 1.0 and lo[0] == -2.5
    rng = np.random.default_rng(1)
    z = rng.standard_normal((300, 128)).astype(np.float32)
    code, scale, lo = oracle.quantize_rows_int8(z)
    rows = np.arange(300)
    assert (code[rows, z.argmin(1)] == 0).all() and (code[rows, z.argmax(1)] == 255).all()
    err = np.abs(oracle.dequantize_rows_int8(code, scale, lo) - z.astype(np.float64))
    assert (err <= scale[:, None].astype(np.float64) * 0.5 * (1 + 1e-4)).all()
