"""fp8 (OCP E4M3, finite-only "fn" flavour) KV codec of the oracle (test infrastructure).

The paper's capacity experiment quantises the KV cache to 4 bits with another
system's kernels (Section 3.4, combination with quantization); the benchmark
configuration this build follows replaces that by fp8 E4M3 codes with one fp32
scale per (token, KV head), separately for K and for V.  Nothing here comes
from the paper except the idea of a quantised KV cache.

Codec (all arithmetic in IEEE fp32, emulated with numpy.float32):
    amax  = max |x| over the head_dim values of the row
    scale = amax / 448            (scale = 1 when amax == 0)
    code  = round-to-nearest-even of x / scale onto the E4M3 grid, saturating at 448
    x_hat = value(code) * scale

E4M3 bit layout (OCP 8-bit floating point specification): 1 sign bit, 4 exponent
bits with bias 7, 3 mantissa bits; exponent field 0 = subnormal (mantissa * 2^-9);
S.1111.111 is NaN, there is no infinity, the largest finite value is
S.1111.110 = 448.

Pins (tests/test_oracle_fp8.py): the decode table against the layout written
out by hand, round trip of every finite code, hand-picked ties, saturation.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table() -> np.ndarray:
    """float64 value of each of the 256 codes (NaN for 0x7F and 0xFF)."""
    table = np.zeros(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        exp = (code >> 3) & 0xF
        man = code & 0x7
        if exp == 0xF and man == 0x7:
            table[code] = np.nan
        elif exp == 0:
            table[code] = sign * man * 2.0 ** (-9)
        else:
            table[code] = sign * (1.0 + man / 8.0) * 2.0 ** (exp - 7)
    return table


_POS_CODES = np.arange(0, 0x7F, dtype=np.uint8)            # 0x00 .. 0x7E, ascending values
_POS_VALUES = e4m3_decode_table()[:0x7F]


def e4m3_encode_f32(x) -> np.ndarray:
    """Round fp32 values to the nearest E4M3 code, ties to the even code,
    magnitudes above the largest finite value saturate to it.  x must be finite."""
    x = np.asarray(x, dtype=np.float32)
    mag = np.abs(x).astype(np.float64)
    hi = np.searchsorted(_POS_VALUES, mag, side="left")       # first grid value >= mag
    hi = np.minimum(hi, len(_POS_VALUES) - 1)
    lo = np.maximum(hi - 1, 0)
    d_hi = np.abs(_POS_VALUES[hi] - mag)
    d_lo = np.abs(mag - _POS_VALUES[lo])
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & ((_POS_CODES[lo] & 1) == 0))
    code = np.where(pick_lo, _POS_CODES[lo], _POS_CODES[hi]).astype(np.uint8)
    code = np.where(mag >= E4M3_MAX, np.uint8(0x7E), code)
    sign = (np.signbit(x)).astype(np.uint8) << 7
    return (code | sign).astype(np.uint8)


def quantize_rows(x):
    """x [..., D] (fp32-representable) -> (codes uint8 [..., D], scales fp32 [...])."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.max(np.abs(x), axis=-1).astype(np.float32)
    scale = np.where(amax == 0, np.float32(1.0), amax / np.float32(448.0)).astype(np.float32)
    ratio = (x / scale[..., None]).astype(np.float32)
    return e4m3_encode_f32(ratio), scale


def dequantize_rows(codes, scales) -> np.ndarray:
    """float64 values code * scale (exact product of an fp32 scale and an E4M3 value)."""
    table = e4m3_decode_table()
    return table[np.asarray(codes, dtype=np.uint8)] * np.asarray(scales, dtype=np.float64)[..., None]
