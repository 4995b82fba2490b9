"""Hadamard rotation followed by the channel reorder -- CPU oracle (test infrastructure only;
see formats.py).

App. D (PermuQuant-H): the per-group quantizer acts on the Hadamard-transformed representation,
and the reorder is applied after the transform, x H P, so that the permutation decides which
transformed channels share a scale.  Here H is written out as a dense orthogonal matrix and
applied with the library matmul in fp64; the GPU library runs a fast transform and writes its
output in the order pi.

Readings where the paper is silent:
  * H is normalised, H H^T = I (entries +-1 / sqrt(d)), so that (x H)(W H)^T = x W^T and the
    rotated layer computes the same function;
  * for d = 2^k the Sylvester matrix in natural order, S[i, j] = (-1)^popcount(i & j);
  * for d = 2^k * m with m in {12, 20} the Kronecker product S_{2^k} (x) P_m, where P_m is the
    Paley (type I) Hadamard matrix of order m = q + 1, q = 11 or 19: with chi the quadratic
    character mod q and Q[i, j] = chi(i - j),  P = I + [[0, 1^T], [-1, Q]].  Channel i = a * m + b
    carries index a in the Sylvester factor and b in the Paley factor.  Other widths are not offered;
  * the transformed tensor is a bf16 tensor (one rounding of the fp64 / fp32 result).
Which Hadamard matrix the authors used is not stated; any of them gives an orthogonal rotation,
so results agree with theirs in distribution only: parity with the authors' H is unpinned.
"""
from __future__ import annotations

import numpy as np

from . import formats as F

PALEY_ORDERS = (12, 20)


def sylvester(n: int) -> np.ndarray:
    """Unnormalised Sylvester-Hadamard matrix of order n = 2^k, natural order."""
    if n < 1 or n & (n - 1):
        raise ValueError("order must be a power of two")
    i = np.arange(n)
    bits = i[:, None] & i[None, :]
    pop = np.zeros_like(bits)
    while np.any(bits):
        pop += bits & 1
        bits = bits >> 1
    return np.where(pop % 2 == 0, 1.0, -1.0)


def paley(m: int) -> np.ndarray:
    """Unnormalised Paley type I Hadamard matrix of order m = q + 1, q prime, q = 3 (mod 4)."""
    q = m - 1
    if q < 3 or q % 4 != 3 or any(q % p == 0 for p in range(2, int(q ** 0.5) + 1)):
        raise ValueError("m - 1 must be a prime congruent to 3 modulo 4")
    squares = {(r * r) % q for r in range(1, q)}
    chi = np.array([0] + [1 if r in squares else -1 for r in range(1, q)], dtype=np.float64)
    idx = (np.arange(q)[:, None] - np.arange(q)[None, :]) % q
    s = np.zeros((m, m))
    s[0, 1:] = 1.0
    s[1:, 0] = -1.0
    s[1:, 1:] = chi[idx]
    return np.eye(m) + s


def factor(d: int):
    """d = 2^k * m with m in {1, 12, 20}: returns (2^k, m) for the smallest such m, or raises."""
    for m in (1,) + PALEY_ORDERS:
        if d % m == 0:
            p = d // m
            if p >= 1 and p & (p - 1) == 0:
                return p, m
    raise ValueError("no Hadamard construction offered for width %d" % d)


def hadamard_matrix(d: int) -> np.ndarray:
    """The normalised d x d matrix H of the module docstring."""
    p, m = factor(d)
    h = sylvester(p)
    if m > 1:
        h = np.kron(h, paley(m))
    return h / np.sqrt(float(d))


def rotate(x) -> np.ndarray:
    """x H, row by row (fp64)."""
    x = np.asarray(x, dtype=np.float64)
    return x @ hadamard_matrix(x.shape[1])


def rotate_reordered(x, perm) -> np.ndarray:
    """x H P: position j of the result holds transformed channel pi(j)  (App. D)."""
    y = rotate(x)
    return y if perm is None else y[:, np.asarray(perm, dtype=np.int64)]


def to_bf16_bits(y) -> np.ndarray:
    return F.f64_to_bf16_bits_rne(y)
