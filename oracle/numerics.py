"""Oracle: bf16 and fp8-e4m3 rounding.  TEST INFRASTRUCTURE ONLY.

The paper measures in FP8 (Sec. 1, Sec. 6) without naming the flavour; this
build reads it as OCP e4m3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
bits, largest finite value 448, no infinities, code 0x7F / 0xFF = NaN).
bf16 is the upper 16 bits of IEEE binary32.  Rounding is to nearest, ties to
the neighbour whose last mantissa bit is 0; fp8 conversion saturates at +-448.
Both are written as "pick the nearest table entry", not as bit tricks.
"""
import numpy as np


def e4m3_decode_table():
    """float64[256]: value of every e4m3 code (NaN for 0x7F and 0xFF)."""
    vals = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            vals[code] = np.nan
        elif e == 0:
            vals[code] = sign * (m / 8.0) * 2.0 ** (-6)
        else:
            vals[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return vals


def e4m3_encode(x):
    """uint8 codes: nearest e4m3 value, ties to even code, saturating at 448."""
    x = np.asarray(x, dtype=np.float64)
    table = e4m3_decode_table()
    pos = table[:0x7F]                      # codes 0x00..0x7E ascend from 0 to 448
    a = np.minimum(np.abs(x), 448.0)
    hi = np.searchsorted(pos, a, side="left")      # first code with value >= a
    hi = np.clip(hi, 0, 0x7E)
    lo = np.clip(hi - 1, 0, 0x7E)
    d_lo = np.abs(a - pos[lo])
    d_hi = np.abs(pos[hi] - a)
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    code = np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)
    return code


def e4m3_decode(code):
    return e4m3_decode_table()[np.asarray(code, dtype=np.uint8)]


def e4m3_quantise(x):
    """(codes, scale): per-tensor scale = max|x| / 448, codes = encode(x / scale)."""
    x = np.asarray(x, dtype=np.float64)
    amax = float(np.max(np.abs(x))) if x.size else 0.0
    scale = amax / 448.0 if amax > 0 else 1.0
    scale = float(np.float32(scale))        # the scale crosses the boundary as a float
    return e4m3_encode(x / scale), scale


def bf16_round(x):
    """float32 array whose values are the bf16 neighbours of x (nearest, ties to even)."""
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    down = u & 0xFFFF0000                    # truncate toward zero (sign-magnitude)
    up = down + 0x10000
    rem = u & 0xFFFF
    take_up = (rem > 0x8000) | ((rem == 0x8000) & (((down >> 16) & 1) == 1))
    r = np.where(take_up, up, down).astype(np.uint32)
    out = r.view(np.float32).copy()
    nan = np.isnan(x)
    out[nan] = np.nan
    return out.reshape(x.shape)
