"""4-bit KV codec of the oracle (test infrastructure).

The paper's capacity experiment stores the KV cache in 4 bits with another system's kernels
(Section 3.4, combination with quantization) and gives no codec details; "parity unpinned" with
respect to the paper.  The codec built here is the usual asymmetric per-row one: for every
(token, KV head), K and V separately, in IEEE fp32 arithmetic (emulated with numpy.float32):

    lo    = min x, hi = max x over the head_dim values of the row
    scale = (hi - lo) / 15                  (scale = 1 when hi == lo)
    code  = clamp(round-to-nearest-even((x - lo) / scale), 0, 15)
    x_hat = code * scale + lo               (evaluated exactly on the fp32 parameters)

Codes are packed two per byte, element 2i in the low nibble and element 2i + 1 in the high one.

The 8-bit form of the same codec (codes 0..255, scale = (hi - lo) / 255, one code per byte) is
quantize_rows_int8 / dequantize_rows_int8.

Pins (tests/test_oracle_int4.py): hand-computed rows, extremes map to 0 and 15 (255), ties go to the
even code, constant rows, error bound scale / 2, packing layout.
"""
from __future__ import annotations

import numpy as np


def _quantize_rows(x, top):
    x = np.asarray(x, dtype=np.float32)
    lo = np.min(x, axis=-1).astype(np.float32)
    hi = np.max(x, axis=-1).astype(np.float32)
    span = (hi - lo).astype(np.float32)
    scale = np.where(span == 0, np.float32(1.0), span / np.float32(top)).astype(np.float32)
    t = (x - lo[..., None]).astype(np.float32)
    r = (t / scale[..., None]).astype(np.float32)
    code = np.clip(np.rint(r), 0, top).astype(np.uint8)     # numpy rint rounds half to even
    return code, scale, lo


def quantize_rows_int4(x):
    """x [..., D] (fp32-representable) -> (codes uint8 [..., D] in 0..15, scale fp32 [...], lo fp32 [...])."""
    return _quantize_rows(x, 15)


def quantize_rows_int8(x):
    """The 8-bit form: codes 0..255, scale = (hi - lo) / 255."""
    return _quantize_rows(x, 255)


def dequantize_rows_int4(codes, scale, lo) -> np.ndarray:
    """float64 values code * scale + lo."""
    return (np.asarray(codes, dtype=np.float64) * np.asarray(scale, dtype=np.float64)[..., None]
            + np.asarray(lo, dtype=np.float64)[..., None])


dequantize_rows_int8 = dequantize_rows_int4     # the same expression: code * scale + lo


def pack_int4(codes) -> np.ndarray:
    """codes uint8 [..., D] -> bytes uint8 [..., D/2]: element 2i low nibble, 2i+1 high nibble."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_int4(packed) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out
