"""Pins for the oracle's normalisation layers and channel reorder (paper App. C).

The oracle's norm functions are checked against hand-worked values, closed forms, the
invariances App. C states, and torch's own layer_norm / rms_norm in fp64 -- none of which
re-use the oracle's formulas."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import formats as F
from oracle import norm as N

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "norm_worked_examples.txt")


def _num(tok: str) -> float:
    """'1.5', '-0.5/sqrt(1.25)'"""
    if "/sqrt(" in tok:
        p, q = tok.split("/sqrt(")
        return float(p) / math.sqrt(float(q.rstrip(")")))
    return float(tok)


def _examples():
    out = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, *fields = [f.strip() for f in line.split("|")]
            kind, eps = head.split()
            out.append((kind, float(eps), [[_num(t) for t in f.split()] for f in fields]))
    return out


@pytest.mark.parametrize("kind,eps,fields", _examples())
def test_worked_examples(kind, eps, fields):
    x = np.array([fields[0]])
    if kind == "rms":
        y = N.rmsnorm(x, np.array(fields[1]), eps)
    elif kind == "ln":
        y = N.layernorm(x, eps)
    else:
        y = N.adaln(x, np.array([fields[1]]), np.array([fields[2]]), 1, eps)
    np.testing.assert_allclose(y[0], fields[-1], rtol=1e-14, atol=1e-15)


def test_examples_cover_every_kind():
    kinds = {k for k, _, _ in _examples()}
    assert kinds == {"rms", "ln", "adaln"}


def test_constant_rows_closed_form():
    # a constant row c: mean square c^2, zero variance
    for c, eps in ((2.0, 0.0), (-3.0, 1e-6), (0.5, 0.25)):
        x = np.full((2, 16), c)
        gamma = np.linspace(-1, 2, 16)
        np.testing.assert_allclose(N.rmsnorm(x, gamma, eps), c / math.sqrt(c * c + eps) * gamma[None, :].repeat(2, 0),
                                   rtol=1e-15)
        assert np.all(N.layernorm(x, eps if eps > 0 else 1.0) == 0.0)


def test_unit_statistics_of_the_output():
    rng = np.random.default_rng(3)
    x = rng.normal(size=(5, 96)) * rng.uniform(0.1, 30, size=(5, 1)) + rng.normal(size=(5, 1))
    y = N.layernorm(x, 0.0)
    np.testing.assert_allclose(y.mean(axis=1), 0.0, atol=1e-14)
    np.testing.assert_allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)
    r = N.rmsnorm(x, np.ones(96), 0.0)
    np.testing.assert_allclose((r * r).mean(axis=1), 1.0, rtol=1e-13)
    # with eps the output mean square is ms / (ms + eps)
    eps = 0.7
    ms = (x * x).mean(axis=1)
    r = N.rmsnorm(x, np.ones(96), eps)
    np.testing.assert_allclose((r * r).mean(axis=1), ms / (ms + eps), rtol=1e-13)


def test_affine_invariance_of_layernorm():
    rng = np.random.default_rng(4)
    x = rng.normal(size=(4, 64))
    y = N.layernorm(x, 0.0)
    np.testing.assert_allclose(N.layernorm(3.5 * x + 11.0, 0.0), y, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(N.layernorm(-2.0 * x, 0.0), -y, rtol=1e-11, atol=1e-12)
    # RMSNorm is invariant to a positive scale only, not to a shift
    g = rng.normal(size=64)
    np.testing.assert_allclose(N.rmsnorm(7.0 * x, g, 0.0), N.rmsnorm(x, g, 0.0), rtol=1e-12)
    assert not np.allclose(N.rmsnorm(x + 1.0, g, 0.0), N.rmsnorm(x, g, 0.0))


def test_against_torch_library_norms():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(7, 80)) * 4.0 + 0.3
    g = rng.normal(size=80)
    b = rng.normal(size=80)
    eps = 1e-5
    xt = torch.from_numpy(x)
    ref_ln = torch.nn.functional.layer_norm(xt, (80,), None, None, eps).numpy()
    np.testing.assert_allclose(N.layernorm(x, eps), ref_ln, rtol=1e-12, atol=1e-13)
    ref_rms = torch.nn.functional.rms_norm(xt, (80,), torch.from_numpy(g), eps).numpy()
    np.testing.assert_allclose(N.rmsnorm(x, g, eps), ref_rms, rtol=1e-12, atol=1e-13)
    # affine LayerNorm = AdaLN with s = gamma - 1, b = beta, one modulation row for all tokens
    ref_aff = torch.nn.functional.layer_norm(xt, (80,), torch.from_numpy(g), torch.from_numpy(b), eps).numpy()
    np.testing.assert_allclose(N.adaln(x, (g - 1.0)[None, :], b[None, :], 7, eps), ref_aff, rtol=1e-12, atol=1e-12)


def test_modulation_rows_follow_the_sample():
    rng = np.random.default_rng(6)
    M, d, per = 10, 24, 4                     # samples of 4, 4 and a ragged last one of 2 tokens
    x = rng.normal(size=(M, d))
    s = rng.normal(size=(3, d))
    b = rng.normal(size=(3, d))
    y = N.adaln(x, s, b, per, 1e-6)
    for m in range(M):                        # row by row, straight from the printed formula
        mu = sum(x[m]) / d
        var = sum((v - mu) ** 2 for v in x[m]) / d
        for j in range(d):
            want = (1.0 + s[m // per][j]) * (x[m][j] - mu) / math.sqrt(var + 1e-6) + b[m // per][j]
            assert abs(y[m, j] - want) <= 1e-13 * max(1.0, abs(want))


def test_reorder_direction():
    # position j of the reordered tensor holds original channel pi(j)
    y = np.array([[10.0, 11.0, 12.0, 13.0]])
    assert N.reorder(y, [2, 0, 3, 1]).tolist() == [[12.0, 10.0, 13.0, 11.0]]
    assert N.reorder(y, None) is y or np.array_equal(N.reorder(y, None), y)


def test_equivariance_identities():
    # App. C: P RMSNorm(x; gamma) = RMSNorm(P x; P gamma);  P AdaLN(x; s, b) = AdaLN(P x; P s, P b)
    rng = np.random.default_rng(7)
    M, d = 6, 48
    x = rng.normal(size=(M, d)) * np.exp(rng.normal(size=d))      # channels of very different size
    g = rng.normal(size=d)
    s = rng.normal(size=(2, d))
    b = rng.normal(size=(2, d))
    perm = rng.permutation(d)
    lhs = N.rmsnorm_reordered(x, g, 1e-6, perm)
    rhs = N.rmsnorm(x[:, perm], g[perm], 1e-6)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-13, atol=1e-15)
    lhs = N.adaln_reordered(x, s, b, 3, 1e-6, perm)
    rhs = N.adaln(x[:, perm], s[:, perm], b[:, perm], 3, 1e-6)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-14)
    # a gather of gamma with the wrong direction (inverse permutation) is not the same function
    inv = np.argsort(perm)
    assert not np.allclose(lhs, N.adaln(x[:, perm], s[:, inv], b[:, inv], 3, 1e-6))


def test_bf16_output_is_one_rounding():
    y = np.array([[1.0 + 2.0 ** -9, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8 + 2.0 ** -30)]])
    bits = N.to_bf16_bits(y)
    back = F.bf16_bits_to_f64(bits)
    # below half an ulp -> down; ties -> even mantissa; just above a tie -> away
    assert back.tolist() == [[1.0, 1.0, 1.0 + 2.0 ** -6, -(1.0 + 2.0 ** -7)]]
