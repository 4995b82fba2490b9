"""Per-group quantizers -- CPU oracle (test infrastructure only; see formats.py).

Sec. 3.1: a token row (or a weight row) of K channels is cut into K/g contiguous groups;
every group shares one scale s = max|x| / Q (Eq. 1) and each element becomes
z = clip(round(x / s), -Q, Q), dequantized as s*z (Eq. 2).  The paper does not fix the
precision of the scale arithmetic, the tie rule of "round", nor what happens for an
all-zero group.  The reading used throughout (each step is one binary32 operation,
written fl32):

  INT-b, per group
      amax = max|x|                       (exact, inputs are bf16)
      s    = fl32(amax / Q)               (the stored scale)
      inv  = fl32(1 / s) if s is a normal number else 0
      z    = clip(rint_half_even(fl32(x * inv)), -Q, Q)
      xhat = s * z                        (exact real product)

  NVFP4, per tensor
      T    = fl32(absmax / 2688)          (2688 = 448 * 6; absmax = max|W| for weights,
                                           the calibration-set max|X| for activations)
      encT = fl32(1 / T) if T is normal else 0
  NVFP4, per block of 16
      t    = fl32(fl32(amax * encT) / 6)
      s_b  = E4M3_rne_sat(t)              (the stored byte)
      d    = fl32(value(s_b) * T)
      inv  = fl32(1 / d) if d is normal else 0
      code = sign(x) << 3 | E2M1_rne_sat(|fl32(x * inv)|)
      xhat = +-E2M1[idx] * value(s_b) * T (exact real product)

Because the inputs are bf16, x/s sits at least 2^-14 (relative) away from any rounding
boundary unless it is exactly on it, and the pinned sequence is accurate to ~2^-22, so
for INT the pinned sequence agrees with the exact-real Eq. 2 except on exact ties
(`quantize_int_exact` reports them).
"""
from __future__ import annotations

from typing import NamedTuple

import numpy as np

from . import formats as F


class IntQuant(NamedTuple):
    z: np.ndarray        # [rows, K] int8 codes in [-Q, Q]
    scale: np.ndarray    # [rows, K/g] float32 stored scales


class Nvfp4Quant(NamedTuple):
    code: np.ndarray     # [rows, K] uint8 nibbles: sign<<3 | E2M1 index
    scale: np.ndarray    # [rows, K/16] uint8 E4M3 bytes
    tensor_scale: np.float32


def _grouped(x: np.ndarray, g: int) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError("x must be [rows, K]")
    rows, K = x.shape
    if g <= 0 or K % g:
        raise ValueError("group size must divide K")
    return x.reshape(rows, K // g, g)


# ----------------------------------------------------------------------------- INT

def quantize_int(x, g: int, fmt: int) -> IntQuant:
    """Eq. 1-2 with the pinned binary32 sequence above. x: [rows, K] float64 (bf16 values)."""
    Q = float(F.qmax(fmt))
    xg = _grouped(x, g)
    amax = np.max(np.abs(xg), axis=2)
    s = F.fl32(amax / Q)
    with np.errstate(divide="ignore"):
        inv = np.where(F.is_normal32(s), F.fl32(1.0 / np.where(s == 0, 1.0, s)), 0.0)
    v = F.fl32(xg * inv[:, :, None])
    z = np.clip(np.rint(v), -Q, Q)
    rows, G, _ = xg.shape
    return IntQuant(z.reshape(rows, G * g).astype(np.int8), s.astype(np.float32))


def dequantize_int(q: IntQuant, g: int) -> np.ndarray:
    """xhat = s * z, exact in fp64 (24-bit scale times a 3-bit integer)."""
    rows, K = q.z.shape
    zz = q.z.astype(np.float64).reshape(rows, K // g, g)
    return (zz * q.scale.astype(np.float64)[:, :, None]).reshape(rows, K)


def quantize_int_exact(x, g: int, fmt: int):
    """Eq. 2 evaluated without the binary32 steps: z = round(Q*x/amax).

    Q*|x| is exact in fp64 (3 + 8 bits); the quotient by the 8-bit amax is either exactly
    a half-integer (a tie, exactly representable) or at least 2^-9 away from one, so the
    correctly rounded fp64 quotient decides every non-tie correctly.
    Returns (z_half_even, tie_mask).
    """
    Q = float(F.qmax(fmt))
    xg = _grouped(x, g)
    amax = np.max(np.abs(xg), axis=2, keepdims=True)
    safe = np.where(amax == 0, 1.0, amax)
    q = (Q * xg) / safe
    q = np.where(amax == 0, 0.0, q)
    tie = (np.abs(q) - np.floor(np.abs(q))) == 0.5
    z = np.clip(np.rint(q), -Q, Q)
    rows, G, _ = xg.shape
    return z.reshape(rows, G * g).astype(np.int8), tie.reshape(rows, G * g)


# ----------------------------------------------------------------------------- NVFP4

def nvfp4_tensor_scale(absmax) -> np.float32:
    """T = fl32(absmax / (448*6)): maps the largest block scale onto the E4M3 maximum."""
    return np.float32(F.fl32(np.float64(absmax) / (F.E4M3_MAX * F.E2M1_MAX)))


def quantize_nvfp4(x, tensor_scale) -> Nvfp4Quant:
    """Two-level NVFP4 quantizer with the pinned binary32 sequence above."""
    g = F.NVFP4_BLOCK
    T = np.float64(np.float32(tensor_scale))
    encT = F.fl32(1.0 / T) if F.is_normal32(T) else np.float64(0.0)
    xg = _grouped(x, g)
    amax = np.max(np.abs(xg), axis=2)
    t = F.fl32(F.fl32(amax * encT) / 6.0)
    sb = F.e4m3_rne_sat(t)
    d = F.fl32(F.e4m3_decode(sb) * T)
    with np.errstate(divide="ignore"):
        inv = np.where(F.is_normal32(d), F.fl32(1.0 / np.where(d == 0, 1.0, d)), 0.0)
    v = F.fl32(xg * inv[:, :, None])
    idx = F.e2m1_rne_sat(np.abs(v))
    sign = np.signbit(xg).astype(np.int64)
    code = (sign << 3) | idx
    rows, G, _ = xg.shape
    return Nvfp4Quant(code.reshape(rows, G * g).astype(np.uint8), sb.astype(np.uint8),
                      np.float32(tensor_scale))


def dequantize_nvfp4(q: Nvfp4Quant) -> np.ndarray:
    """xhat = +-E2M1[idx] * E4M3(s_b) * T; exact in fp64 (2 + 4 + 24 significant bits)."""
    g = F.NVFP4_BLOCK
    rows, K = q.code.shape
    c = q.code.astype(np.int64)
    mag = F.e2m1_decode(c & 7)
    sgn = np.where((c >> 3) & 1, -1.0, 1.0)
    sc = F.e4m3_decode(q.scale).astype(np.float64) * np.float64(q.tensor_scale)
    return ((sgn * mag).reshape(rows, K // g, g) * sc[:, :, None]).reshape(rows, K)


# ----------------------------------------------------------------------------- uniform front

def quantize(fmt: int, g: int, x, tensor_scale=None):
    """Quantize [rows, K] values in the given channel order; returns the format's tuple."""
    if fmt == F.FMT_NVFP4:
        if g != F.NVFP4_BLOCK:
            raise ValueError("NVFP4 uses blocks of 16")
        if tensor_scale is None:
            raise ValueError("NVFP4 needs the per-tensor scale")
        return quantize_nvfp4(x, tensor_scale)
    return quantize_int(x, g, fmt)


def dequantize(fmt: int, g: int, q) -> np.ndarray:
    if fmt == F.FMT_NVFP4:
        return dequantize_nvfp4(q)
    return dequantize_int(q, g)


def packed_codes(fmt: int, q) -> np.ndarray:
    """The byte layout the library stores: two 4-bit containers per byte, even k low."""
    if fmt == F.FMT_NVFP4:
        return F.pack_nibbles(q.code)
    return F.pack_nibbles(F.int_to_nibble(q.z))
