"""Normalisation followed by the channel reorder -- CPU oracle (test infrastructure only;
see formats.py).

App. C ("absorbing the permutation into normalisation layers").  The layer in front of a
quantized linear layer is RMSNorm, LayerNorm, or LayerNorm with an adaptive scale and shift;
the method needs its output in the reordered channel order, y_P[j] = y[pi(j)].  This module
writes that down in the plain two-step form (normalise in the original order, then gather);
the GPU library computes the fused form (indexed load, statistics, gathered vectors), which
App. C's equivariance identities say is the same function:

    RMSNorm(x; gamma) = x / sqrt(mean_i x_i^2 + eps) * gamma
    LN(x)             = (x - mu) / sqrt(sigma^2 + eps),  mu = mean_i x_i,
                        sigma^2 = mean_i (x_i - mu)^2
    AdaLN(x; s, b)    = (1 + s) * LN(x) + b            (modulation vectors per sample)

Everything in fp64; the output is rounded once to bf16 where a caller asks for bits.

Readings where the paper is silent:
  * eps is added to the mean square / variance under the root (as printed);
  * the variance is the biased one (1/d), as printed;
  * a plain affine LayerNorm gamma * LN(x) + beta is AdaLN with s = gamma - 1, b = beta and one
    modulation row shared by all tokens;
  * modulation vectors are given per sample: token row m uses modulation row m // rows_per_mod;
  * the normalised tensor handed to the quantizer is a bf16 tensor (the dtype of the
    activations), so quantization acts on the bf16-rounded output.
"""
from __future__ import annotations

import numpy as np

from . import formats as F


def rmsnorm(x, gamma, eps: float) -> np.ndarray:
    """App. C, RMSNorm: rows of x [M, d] scaled by 1 / sqrt(mean square + eps), times gamma [d]."""
    x = np.asarray(x, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    mean_sq = np.sum(x * x, axis=1, keepdims=True) / x.shape[1]
    return x / np.sqrt(mean_sq + eps) * gamma[None, :]


def layernorm(x, eps: float) -> np.ndarray:
    """App. C, LayerNorm without affine part: (x - mu) / sqrt(sigma^2 + eps) per row."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[1]
    mu = np.sum(x, axis=1, keepdims=True) / d
    var = np.sum((x - mu) ** 2, axis=1, keepdims=True) / d
    return (x - mu) / np.sqrt(var + eps)


def adaln(x, scale, shift, rows_per_mod: int, eps: float) -> np.ndarray:
    """App. C, LayerNorm followed by modulation: (1 + s) * LN(x) + b.

    scale, shift: [n_mod, d]; token row m takes modulation row m // rows_per_mod."""
    x = np.asarray(x, dtype=np.float64)
    scale = np.asarray(scale, dtype=np.float64)
    shift = np.asarray(shift, dtype=np.float64)
    which = np.arange(x.shape[0]) // int(rows_per_mod)
    return (1.0 + scale[which]) * layernorm(x, eps) + shift[which]


def reorder(y, perm) -> np.ndarray:
    """y_P[:, j] = y[:, pi(j)]  (App. C: the output in the reordered channel order)."""
    y = np.asarray(y)
    return y if perm is None else y[:, np.asarray(perm, dtype=np.int64)]


def rmsnorm_reordered(x, gamma, eps, perm) -> np.ndarray:
    """Normalise in the original order, then reorder (the two-step form of App. C)."""
    return reorder(rmsnorm(x, gamma, eps), perm)


def adaln_reordered(x, scale, shift, rows_per_mod, eps, perm) -> np.ndarray:
    return reorder(adaln(x, scale, shift, rows_per_mod, eps), perm)


def to_bf16_bits(y) -> np.ndarray:
    """One rounding (nearest even) of the fp64 result to bf16 bit patterns."""
    return F.f64_to_bf16_bits_rne(y)
