"""Pins for the oracle's Hadamard rotation (paper App. D): the defining properties of a Hadamard
matrix, small instances written out by hand, the textbook butterfly as a second algorithm, and
the index conventions of the Kronecker product and of the reorder."""
import numpy as np
import pytest

from oracle import hadamard as H


def test_small_sylvester_matrices_by_hand():
    assert H.sylvester(1).tolist() == [[1.0]]
    assert H.sylvester(2).tolist() == [[1, 1], [1, -1]]
    assert H.sylvester(4).tolist() == [[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]]
    with pytest.raises(ValueError):
        H.sylvester(12)


@pytest.mark.parametrize("m", [12, 20])
def test_paley_matrix_is_hadamard(m):
    p = H.paley(m)
    assert set(np.unique(p).tolist()) == {-1.0, 1.0}
    assert np.array_equal(p @ p.T, m * np.eye(m))
    assert np.all(p[0] == 1.0) and np.all(p[1:, 0] == -1.0)          # the bordering row and column
    s = p - np.eye(m)
    assert np.array_equal(s, -s.T)                                     # type I: identity plus a skew matrix
    with pytest.raises(ValueError):
        H.paley(16)                                                    # 15 is not prime


def test_paley_12_quadratic_residues():
    # the squares mod 11 are {1, 3, 4, 5, 9}: entry (i, j) of the core is +1 iff i - j is one of them
    p = H.paley(12)
    for i in range(11):
        for j in range(11):
            if i != j:
                assert p[1 + i, 1 + j] == (1.0 if (i - j) % 11 in (1, 3, 4, 5, 9) else -1.0)


@pytest.mark.parametrize("d", [1, 2, 16, 64, 12, 20, 48, 80, 96, 768])
def test_rotation_is_orthogonal_with_equal_magnitudes(d):
    h = H.hadamard_matrix(d)
    np.testing.assert_allclose(np.abs(h), 1.0 / np.sqrt(d), rtol=1e-15)
    np.testing.assert_allclose(h @ h.T, np.eye(d), atol=1e-13)


def test_factorisation_of_model_widths():
    assert H.factor(3072) == (256, 12) and H.factor(4096) == (4096, 1)
    assert H.factor(12288) == (1024, 12) and H.factor(2560) == (128, 20) and H.factor(1536) == (128, 12)
    for d in (1152, 60, 240, 3840):
        with pytest.raises(ValueError):
            H.factor(d)


def _butterfly(v):
    """Textbook in-place fast Walsh-Hadamard transform (natural order), unnormalised."""
    v = list(v)
    h = 1
    while h < len(v):
        for i in range(0, len(v), 2 * h):
            for j in range(i, i + h):
                v[j], v[j + h] = v[j] + v[j + h], v[j] - v[j + h]
        h *= 2
    return v


def test_power_of_two_rotation_equals_the_fast_transform():
    rng = np.random.default_rng(21)
    x = rng.normal(size=(3, 128))
    y = H.rotate(x)
    for r in range(3):
        np.testing.assert_allclose(y[r], np.array(_butterfly(x[r])) / np.sqrt(128.0), rtol=1e-12, atol=1e-13)


def test_kronecker_index_convention():
    # channel i = a * m + b: unit vector e_i is mapped to row i of H = S (x) P / sqrt(d)
    d, m = 24, 12
    s, p = H.sylvester(2), H.paley(12)
    for a, b in ((0, 0), (1, 0), (0, 5), (1, 7)):
        e = np.zeros((1, d))
        e[0, a * m + b] = 1.0
        y = H.rotate(e)[0]
        for a2 in range(2):
            for b2 in range(m):
                assert abs(y[a2 * m + b2] - s[a, a2] * p[b, b2] / np.sqrt(d)) < 1e-15


def test_rotated_layer_computes_the_same_product():
    rng = np.random.default_rng(22)
    x = rng.normal(size=(5, 96))
    w = rng.normal(size=(7, 96))
    np.testing.assert_allclose(H.rotate(x) @ H.rotate(w).T, x @ w.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.sum(H.rotate(x) ** 2, axis=1), np.sum(x ** 2, axis=1), rtol=1e-13)
    # an outlier channel is spread evenly: a one-hot row becomes a row of equal magnitudes
    e = np.zeros((1, 96))
    e[0, 17] = 8.0
    np.testing.assert_allclose(np.abs(H.rotate(e)), 8.0 / np.sqrt(96.0), rtol=1e-14)


def test_reorder_is_applied_after_the_rotation():
    rng = np.random.default_rng(23)
    x = rng.normal(size=(2, 48))
    perm = rng.permutation(48)
    y = H.rotate(x)
    got = H.rotate_reordered(x, perm)
    for j in range(48):
        assert np.array_equal(got[:, j], y[:, perm[j]])
    # not the same as permuting first (the transform mixes the channels again)
    assert not np.allclose(got, H.rotate(x[:, perm]))
    assert np.array_equal(H.rotate_reordered(x, None), y)
