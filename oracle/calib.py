"""Calibration statistics and permutation selection -- CPU oracle (test infrastructure
only; see formats.py).

Sec. 3.2-3.3.  Per input channel i the method keeps the second moment of the activations
over the calibration tokens and of the weights that multiply that channel (Assumption 1,
Eq. 9).  Channels are ordered by the joint score
        v_i = (mu_a,i^2)^alpha * (mu_w,i^2)^(1-alpha)          (Eq. 9)
in descending order (Prop. 1), alpha is searched over a uniform grid and the candidate
with the smallest quantization error on the calibration data wins (Sec. 3.3, App.
"Implementation Details"); the winner replaces the original order only if
        (E_orig - E_reorder) / E_orig > tau                     (acceptance rule).

Readings where the paper is silent:
  * a common factor does not change a sort, so sums of squares stand in for the means;
  * the sort key is the logarithm of v_i (same order), a term with weight zero is left out
    (so 0 * log 0 never appears; matches 0^0 = 1), a zero sum sorts last;
  * ties keep ascending channel index; alpha ties go to the smallest alpha;
  * E is the sum of the two tensors' relative squared quantization errors,
        E(pi) = ||X - Xhat_pi||^2 / ||X||^2 + ||W - What_pi||^2 / ||W||^2,
    over all calibration tokens, each side quantized in the order pi;
  * perm[j] = original channel placed at position j  (x_j <- x[pi(j)], App. C).
"""
from __future__ import annotations

from typing import List, NamedTuple, Sequence

import numpy as np

from . import formats as F
from . import quantize as Qz

DEFAULT_ALPHAS = (0.0, 0.2, 0.4, 0.6, 0.8, 1.0)


def column_sumsq(x) -> np.ndarray:
    """S[i] = sum over rows of x[r, i]^2, fp64, plain loop over rows (Sec. 3.2, mu_i^2)."""
    x = np.asarray(x, dtype=np.float64)
    acc = np.zeros(x.shape[1], dtype=np.float64)
    for r in range(x.shape[0]):
        acc += x[r] * x[r]
    return acc


def absmax(x) -> float:
    return float(np.max(np.abs(np.asarray(x, dtype=np.float64)))) if np.size(x) else 0.0


def joint_key(sa, sw, alpha: float) -> np.ndarray:
    """log of Eq. 9's score; the term whose exponent is zero is omitted."""
    sa = np.asarray(sa, dtype=np.float64)
    sw = np.asarray(sw, dtype=np.float64)
    key = np.zeros(sa.shape, dtype=np.float64)
    with np.errstate(divide="ignore"):
        if alpha != 0.0:
            key = key + alpha * np.log(sa)
        if alpha != 1.0:
            key = key + (1.0 - alpha) * np.log(sw)
    return key


def sort_descending(key) -> np.ndarray:
    """Prop. 1: channels in descending key order; equal keys keep ascending index."""
    key = np.asarray(key, dtype=np.float64)
    return np.argsort(-key, kind="stable").astype(np.int32)


def min_relative_key_gap(key, perm) -> float:
    """Smallest gap between neighbouring sorted keys relative to their magnitude (a
    diagnostic: a case is well-posed for bit-exact comparison only if this is not tiny)."""
    k = np.asarray(key, dtype=np.float64)[np.asarray(perm)]
    k = k[np.isfinite(k)]
    if k.size < 2:
        return np.inf
    gap = k[:-1] - k[1:]
    den = np.maximum(np.maximum(np.abs(k[:-1]), np.abs(k[1:])), 1e-300)
    return float(np.min(gap / den))


def squared_error(fmt: int, g: int, x, perm=None, tensor_scale=None) -> float:
    """||x_pi - Q(x_pi)||^2 summed over all entries, fp64 (Eq. 3 on a finite sample)."""
    x = np.asarray(x, dtype=np.float64)
    xp = x if perm is None else x[:, np.asarray(perm)]
    q = Qz.quantize(fmt, g, xp, tensor_scale)
    d = xp - Qz.dequantize(fmt, g, q)
    return float(np.sum(d * d))


class SelectResult(NamedTuple):
    perm: np.ndarray            # [K] int32, identity when rejected
    accepted: bool
    alpha_index: int            # index of the best candidate in the alpha grid
    e_orig: float
    e_best: float
    e_cand: List[float]         # E for every alpha
    cand_perms: List[np.ndarray]
    min_key_gap: float


def calibration_error(fmt: int, g: int, x_batches: Sequence[np.ndarray], w, perm,
                      act_tensor_scale=None, w_tensor_scale=None,
                      sum_x2: float | None = None, sum_w2: float | None = None) -> float:
    """E(pi) of the module docstring."""
    if sum_x2 is None:
        sum_x2 = float(sum(np.sum(np.asarray(xb, dtype=np.float64) ** 2) for xb in x_batches))
    if sum_w2 is None:
        sum_w2 = float(np.sum(np.asarray(w, dtype=np.float64) ** 2))
    ex = 0.0
    for xb in x_batches:
        ex += squared_error(fmt, g, xb, perm, act_tensor_scale)
    ew = squared_error(fmt, g, w, perm, w_tensor_scale)
    return ex / sum_x2 + ew / sum_w2


def output_error(fmt: int, g: int, x_batches: Sequence[np.ndarray], w, perm,
                 act_tensor_scale=None, w_tensor_scale=None) -> float:
    """The other reading of "quantization error on the calibration data" (Sec. 3.3): the relative
    error of the layer's output,
        E_out(pi) = sum_b ||X_b W^T - Q(X_b P) Q(P^T W)^T||^2 / sum_b ||X_b W^T||^2      (Eq. 8),
    both operands quantized in the order pi; the unquantized product does not depend on pi."""
    w = np.asarray(w, dtype=np.float64)
    wp = w if perm is None else w[:, np.asarray(perm)]
    w_hat = Qz.dequantize(fmt, g, Qz.quantize(fmt, g, wp, w_tensor_scale))
    num = den = 0.0
    for xb in x_batches:
        xb = np.asarray(xb, dtype=np.float64)
        xp = xb if perm is None else xb[:, np.asarray(perm)]
        x_hat = Qz.dequantize(fmt, g, Qz.quantize(fmt, g, xp, act_tensor_scale))
        y = xb @ w.T
        d = y - x_hat @ w_hat.T
        num += float(np.sum(d * d))
        den += float(np.sum(y * y))
    return num / den


def select_permutation(fmt: int, g: int, x_batches: Sequence[np.ndarray], w,
                       alphas: Sequence[float] = DEFAULT_ALPHAS, tau: float = 0.0,
                       act_tensor_scale=None, metric: str = "tensor") -> SelectResult:
    """Joint second-moment reordering with calibration-based acceptance (Sec. 3.3).

    x_batches: calibration activations, each [M, K] fp64 (bf16 values); w: [N, K].
    metric: "tensor" -- E of the module docstring (the two tensors' relative errors);
            "output" -- output_error above (the layer-output reading).
    """
    w = np.asarray(w, dtype=np.float64)
    K = w.shape[1]
    sa = np.zeros(K)
    for xb in x_batches:
        sa += column_sumsq(xb)
    sw = column_sumsq(w)
    w_ts = None
    if fmt == F.FMT_NVFP4:
        w_ts = Qz.nvfp4_tensor_scale(absmax(w))
        if act_tensor_scale is None:
            act_tensor_scale = Qz.nvfp4_tensor_scale(max(absmax(xb) for xb in x_batches))
    sum_x2 = float(np.sum(sa))
    sum_w2 = float(np.sum(sw))

    if metric == "tensor":
        def err(p):
            return calibration_error(fmt, g, x_batches, w, p, act_tensor_scale, w_ts, sum_x2, sum_w2)
    elif metric == "output":
        def err(p):
            return output_error(fmt, g, x_batches, w, p, act_tensor_scale, w_ts)
    else:
        raise ValueError("metric must be 'tensor' or 'output'")

    ident = np.arange(K, dtype=np.int32)
    e_orig = err(None)
    cands, errs, gaps = [], [], []
    for a in alphas:
        key = joint_key(sa, sw, float(a))
        p = sort_descending(key)
        cands.append(p)
        gaps.append(min_relative_key_gap(key, p))
        errs.append(err(p))
    j = int(np.argmin(np.asarray(errs)))          # first minimum = smallest alpha
    best = cands[j]
    accepted = (not np.array_equal(best, ident)) and e_orig > 0.0 and \
        ((e_orig - errs[j]) / e_orig > tau)
    return SelectResult(best.copy() if accepted else ident, bool(accepted), j, e_orig, errs[j],
                        list(errs), cands, float(min(gaps)))


def partition_objective(a, perm, g: int) -> float:
    """sum_k max_{i in G_k} a_i for the contiguous groups induced by perm (Eq. 6 / Prop. 1)."""
    a = np.asarray(a, dtype=np.float64)[np.asarray(perm)]
    return float(np.sum(np.max(a.reshape(-1, g), axis=1)))
