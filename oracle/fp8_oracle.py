"""CPU oracle for the 8-bit KV-cache option: the E4M3 number format and a cache held in it.

TEST INFRASTRUCTURE ONLY (see stage_oracle.py): imported by tests, the smoke check and the
benchmark's CPU-baseline leg, never by the product path; shares no code with the HIP kernels.

The paper stores the KV cache in the model's 16-bit type (Sec. 4.1, Table 2) and shows that the
decode phase is bound by reading that cache (Sec. 2.1); holding it in 8 bits halves those bytes.
The format is the public OCP 8-bit floating-point E4M3 encoding: bit 7 sign, bits 6..3 exponent
with bias 7, bits 2..0 mantissa; exponent field 0 is subnormal (2^-6 * m/8); there are no
infinities; S.1111.111 is NaN, so the largest finite magnitude is 2^8 * 1.75 = 448.

Conversion to E4M3 as used for the cache: x / scale is formed in `precision` (the kernel divides in
fp32; both sides take the rounding decision on the same number), then rounded to the nearest
representable value, ties to the code with an even mantissa; magnitudes that round beyond 448, and
infinities, saturate to +-448; NaN stays NaN.  The cache then *is* the decoded values times scale.

Pinned by tests/test_fp8_pins.py: the decode table against values that follow from the format by
hand and against an independent library implementation of the format, the encoder against brute
force over the table, ties, saturation, monotonicity and the half-step error bound.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
E4M3_MAX = 448.0
E4M3_NAN = 0x7F


def e4m3_decode_table() -> np.ndarray:
    """value[c] for the 256 codes, float64 (NaN for 0x7f and 0xff), straight from the format."""
    out = np.empty(256, F64)
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = 2.0 ** -6 * (m / 8.0)
        else:
            v = 2.0 ** (e - 7) * (1.0 + m / 8.0)
        out[c] = -v if s else v
    return out


_TABLE = e4m3_decode_table()
_POS = _TABLE[:0x7F]                      # codes 0x00..0x7e: 0 .. 448, strictly increasing
_MID = (_POS[:-1] + _POS[1:]) / 2.0       # midpoint between code c and c + 1


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return _TABLE[np.asarray(codes, np.uint8)]


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of every element of x (float64 taken as exact): round to nearest, ties to
    the even code, saturating; NaN -> 0x7f | sign."""
    x = np.asarray(x, F64)
    mag = np.abs(x)
    # number of midpoints strictly below |x|: code c such that mid[c-1] < |x| <= mid[c]
    c = np.searchsorted(_MID, mag, side="left").astype(np.int64)
    # exactly on a midpoint: searchsorted('left') gave the lower code; the tie goes to the even one
    c_hi = np.minimum(c + 1, 0x7E)
    on_mid = (c < len(_MID)) & (mag == _MID[np.minimum(c, len(_MID) - 1)])
    c = np.where(on_mid & (c % 2 == 1), c_hi, c)
    c = np.minimum(c, 0x7E)               # beyond the last midpoint: saturate (covers +-inf)
    c = np.where(np.isnan(x), E4M3_NAN, c)
    return (c | (np.signbit(x).astype(np.int64) << 7)).astype(np.uint8)


def kv_quantize(x: np.ndarray, scale: float, precision=np.float32) -> np.ndarray:
    """Codes stored for values x at cache scale `scale`: encode(x / scale), the quotient formed in
    `precision` (inputs are rounded to it first)."""
    q = np.asarray(x).astype(precision) / precision(scale)
    return e4m3_encode(q.astype(F64))


def kv_dequantize(codes: np.ndarray, scale: float) -> np.ndarray:
    """What attention reads back: decoded value times scale, float64."""
    return e4m3_decode(codes) * F64(scale)


def kv_roundtrip(x: np.ndarray, scale: float, precision=np.float32) -> np.ndarray:
    return kv_dequantize(kv_quantize(x, scale, precision), scale)
