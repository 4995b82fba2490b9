"""Dequantized reference product -- CPU oracle (test infrastructure only; see formats.py).

Eq. 8: Y = X W ~ Q(X P) Q(P^T W).  With W stored [N, K] (out x in) the reordered layer is
        Y[m, n] = sum_k xhat[m, k] * what[n, k]
where xhat, what are the dequantized values of the two quantized operands, both in the
same (permuted) channel order.  Everything is fp64; the matmul is the library routine.
"""
from __future__ import annotations

import numpy as np

from . import formats as F
from . import quantize as Qz


def dequant_product(fmt: int, g: int, qa, qw, rows=None) -> np.ndarray:
    """fp64 product of the dequantized operands; optional subset of activation rows."""
    a = Qz.dequantize(fmt, g, qa)
    w = Qz.dequantize(fmt, g, qw)
    if rows is not None:
        a = a[np.asarray(rows)]
    return a @ w.T


def dequant_product_from_packed(fmt: int, g: int, a_codes, a_scales, a_tensor_scale,
                                w_codes, w_scales, w_tensor_scale, rows=None) -> np.ndarray:
    """Same product starting from the stored byte layout (codes packed two per byte)."""
    def build(codes, scales, ts):
        nib = F.unpack_nibbles(codes)
        if fmt == F.FMT_NVFP4:
            return Qz.Nvfp4Quant(nib, np.asarray(scales, dtype=np.uint8), np.float32(ts))
        return Qz.IntQuant(F.nibble_to_int(nib).astype(np.int8),
                           np.asarray(scales, dtype=np.float32))
    return dequant_product(fmt, g, build(a_codes, a_scales, a_tensor_scale),
                           build(w_codes, w_scales, w_tensor_scale), rows)


def add_bias(y, bias) -> np.ndarray:
    """The linear layer's bias, one value per output column: y[m, n] + b[n] (fp64)."""
    return np.asarray(y, dtype=np.float64) + np.asarray(bias, dtype=np.float64)[None, :]


def plain_product(x, w) -> np.ndarray:
    """Unquantized Y = X W^T in fp64 (left side of Eq. 8)."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def bf16_round(y) -> np.ndarray:
    """bf16 (RNE) image of fp64 values, as uint16 bits."""
    return F.f64_to_bf16_bits_rne(y)
