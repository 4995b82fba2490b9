"""Number formats of the per-group quantizers -- CPU oracle (test infrastructure only).

This package is the slow, plain reference the GPU library is checked against.  Only
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the product
never does, and this package imports nothing from the product.

Formats:
  * symmetric INT-b: integers in [-Q, Q], Q = 2^(b-1) - 1, the largest representable
    integer (Sec. 3.1, Eq. 1-2).
  * NVFP4: the paper only names it (Sec. 4.4, Fig. 1).  Reading used here: E2M1
    element codes (OCP microscaling FP4 value set), one E4M3 scale per 16 consecutive
    channels, one fp32 scale per tensor.
  * bf16 inputs arrive as uint16 bit patterns and are widened exactly.

`fl32(v)` rounds an fp64 value once to binary32 (round-to-nearest-even).  For one
+, -, * or / of binary32 operands evaluated in fp64 and then rounded by fl32 the result
equals the IEEE binary32 operation (53 >= 2*24+2, so the double rounding is innocuous).
"""
from __future__ import annotations

import numpy as np

# magnitudes of the eight E2M1 codes, index = (exponent<<1 | mantissa)
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)
E2M1_MAX = 6.0
E4M3_MAX = 448.0
NVFP4_BLOCK = 16

FMT_NVFP4 = 0
FMT_INT4 = 1
FMT_INT3 = 2


def qmax(fmt: int) -> int:
    """Q of Eq. 1: largest representable integer of the symmetric b-bit grid."""
    if fmt == FMT_INT4:
        return 7
    if fmt == FMT_INT3:
        return 3
    raise ValueError("qmax is defined for the INT formats only")


def fl32(v):
    """One rounding to binary32, returned as float64 (so later ops stay in fp64)."""
    with np.errstate(over="ignore", invalid="ignore"):
        return np.asarray(v, dtype=np.float64).astype(np.float32).astype(np.float64)


def is_normal32(v) -> np.ndarray:
    """True where a (non-negative, binary32-representable) value is a normal number."""
    v = np.asarray(v, dtype=np.float64)
    return np.isfinite(v) & (np.abs(v) >= 2.0 ** -126)


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 data must be given as uint16 bit patterns")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits_rne(v) -> np.ndarray:
    """Round fp64 values to bf16, round-to-nearest-even, one rounding -> uint16 bits."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    flat_v = v.reshape(-1)
    flat_o = out.reshape(-1)
    a = np.abs(flat_v)
    # bracket |v| by the two neighbouring bf16 magnitudes: truncate the fp32 image and
    # step one bf16 ulp to either side as needed, then choose in fp64.
    f = a.astype(np.float32)
    t = f.view(np.uint32) & np.uint32(0xFFFF0000)
    t_f = t.view(np.float32).astype(np.float64)
    above = t_f > a                    # the fp32 rounding went past a bf16 value
    t = np.where(above, t - np.uint32(0x10000), t)
    lo = t
    hi = t + np.uint32(0x10000)
    lo_f = lo.view(np.float32).astype(np.float64)
    hi_f = hi.view(np.float32).astype(np.float64)
    d_lo = a - lo_f
    d_hi = hi_f - a
    lo_even = ((lo >> np.uint32(16)) & np.uint32(1)) == 0
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~lo_even)
    mag = (np.where(take_hi, hi, lo) >> np.uint32(16)).astype(np.uint16)
    sign = np.where(np.signbit(flat_v), np.uint16(0x8000), np.uint16(0))
    flat_o[:] = mag | sign
    return out


# ----------------------------------------------------------------------------- E2M1

def e2m1_rne_sat(a) -> np.ndarray:
    """Index (0..7) of the E2M1 magnitude nearest to a >= 0.

    Ties go to the code with an even index (even mantissa bit), values above the
    largest magnitude saturate to it.  Written as "how many decision boundaries does
    a pass": the boundary between codes j and j+1 is their midpoint; a value exactly
    on it stays at j when j is even and moves to j+1 when j is odd.
    """
    a = np.asarray(a, dtype=np.float64)
    idx = np.zeros(a.shape, dtype=np.int64)
    for j in range(7):
        mid = 0.5 * (E2M1_VALUES[j] + E2M1_VALUES[j + 1])
        if j % 2 == 0:
            idx += (a > mid)
        else:
            idx += (a >= mid)
    return idx


def e2m1_decode(idx) -> np.ndarray:
    return E2M1_VALUES[np.asarray(idx, dtype=np.int64)]


# ----------------------------------------------------------------------------- E4M3

def e4m3_decode(code) -> np.ndarray:
    """Value of a non-negative E4M3 ("fn": bias 7, no infinities) byte, codes 0..126."""
    c = np.asarray(code, dtype=np.int64)
    e = (c >> 3) & 0xF
    m = c & 0x7
    sub = m.astype(np.float64) * 2.0 ** -9
    nor = np.ldexp(1.0 + m.astype(np.float64) / 8.0, e - 7)
    return np.where(e == 0, sub, nor)


_E4M3_TABLE = e4m3_decode(np.arange(127))          # strictly increasing, 0 .. 448


def e4m3_rne_sat(t) -> np.ndarray:
    """Code (0..126) of the E4M3 value nearest to t >= 0.

    Round-to-nearest, ties to the even code, everything above 448 (infinity included)
    saturates to 448 (code 0x7E).
    """
    t = np.asarray(t, dtype=np.float64)
    tt = np.minimum(t, E4M3_MAX)                      # inf and > 448 -> 448
    hi = np.searchsorted(_E4M3_TABLE, tt, side="left")   # first code with value >= tt
    hi = np.clip(hi, 0, 126)
    lo = np.maximum(hi - 1, 0)
    d_lo = tt - _E4M3_TABLE[lo]
    d_hi = _E4M3_TABLE[hi] - tt
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    take_hi |= (hi == lo)
    return np.where(take_hi, hi, lo).astype(np.int64)


# ----------------------------------------------------------------------------- nibbles

def pack_nibbles(codes) -> np.ndarray:
    """[rows, K] 4-bit codes (0..15) -> [rows, K/2] bytes, even k in the low nibble."""
    c = np.asarray(codes, dtype=np.uint8)
    if c.shape[-1] % 2:
        raise ValueError("K must be even")
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def int_to_nibble(z) -> np.ndarray:
    """Signed integer codes -> 4-bit two's complement containers."""
    return (np.asarray(z, dtype=np.int64) & 0xF).astype(np.uint8)


def nibble_to_int(n) -> np.ndarray:
    n = np.asarray(n, dtype=np.int64)
    return np.where(n >= 8, n - 16, n)
