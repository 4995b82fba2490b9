"""Alternative reorder criteria of the ablation (Tab. 2a) -- CPU oracle (test infrastructure only;
see formats.py).

The method sorts channels by the joint second moment (Eq. 9).  The ablation compares that with
variance, absmax, round-robin and random orderings.  The paper names them without formulas; the
readings taken here:
  * a criterion supplies one non-negative statistic per channel and side, which enters the joint
    score of Eq. 9 in place of the second moment (the score is a product of powers, so any fixed
    power of the statistic gives the same order as long as both sides use the same one):
        second moment  sum_r x[r, i]^2
        variance       sum_r (x[r, i] - mean_i)^2
        absmax         (max_r |x[r, i]|)^2
  * round-robin: channels sorted by the joint second moment are dealt out one by one to the K / g
    groups in turn (rank r goes to group r mod (K / g), slot r div (K / g)), which spreads the
    large channels evenly over the groups -- the opposite of clustering them;
  * random: a seeded permutation; both sides sort the channels by the 53 high bits of a
    counter-based 64-bit hash of (seed + channel), ascending, equal hashes in ascending channel order.
"""
from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1


def column_sum(x) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    acc = np.zeros(x.shape[1], dtype=np.float64)
    for r in range(x.shape[0]):
        acc += x[r]
    return acc


def column_absmax(x) -> np.ndarray:
    return np.max(np.abs(np.asarray(x, dtype=np.float64)), axis=0)


def column_variance_sum(x) -> np.ndarray:
    """sum_r (x[r, i] - mean_i)^2: n times the (biased) variance of channel i, two passes."""
    x = np.asarray(x, dtype=np.float64)
    mean = column_sum(x) / x.shape[0]
    d = x - mean[None, :]
    return np.sum(d * d, axis=0)


def round_robin(order, g: int) -> np.ndarray:
    """Deal the channels of `order` (best first) to the K / g groups in turn."""
    order = np.asarray(order)
    K = order.shape[0]
    if K % g:
        raise ValueError("group size must divide K")
    n_groups = K // g
    perm = np.empty(K, dtype=np.int32)
    for r in range(K):
        perm[(r % n_groups) * g + r // n_groups] = order[r]
    return perm


def splitmix64(v: int) -> int:
    """The splitmix64 output function applied to the counter v (mod 2^64)."""
    z = (v + 0x9E3779B97F4A7C15) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def random_order(seed: int, K: int) -> np.ndarray:
    keys = np.array([splitmix64((seed + i) & MASK64) >> 11 for i in range(K)], dtype=np.uint64)
    return np.argsort(keys, kind="stable").astype(np.int32)
