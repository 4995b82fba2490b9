"""Pins of the dense 3-bit layout of INT3 codes (oracle/int3.py): hand-worked bytes, the size of a
row, brute force with whole-row integers, round trips and rejection of what does not fit."""
import os

import numpy as np
import pytest

from oracle import int3

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "int3_dense_worked_examples.txt")


def _examples():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            z, b = line.split("|")
            out.append(([int(t) for t in z.split()], [int(t, 16) for t in b.split()]))
    return out


@pytest.mark.parametrize("z,expect", _examples())
def test_hand_worked_bytes(z, expect):
    got = int3.pack_dense(np.array([z]))
    assert got.dtype == np.uint8
    assert got[0].tolist() == expect
    assert int3.unpack_dense(np.array([expect], dtype=np.uint8), len(z))[0].tolist() == z


def test_there_are_enough_examples():
    assert len(_examples()) >= 8


@pytest.mark.parametrize("rows,K", [(1, 8), (3, 32), (5, 96), (2, 3072)])
def test_row_size_and_whole_row_integer(rows, K):
    """A row read as one little-endian integer is sum_k (z_k mod 8) 8^k (Python integers)."""
    rng = np.random.default_rng(K + rows)
    z = rng.integers(-3, 4, size=(rows, K))
    p = int3.pack_dense(z)
    assert p.shape == (rows, 3 * K // 8)
    for r in range(rows):
        n = 0
        for k in range(K - 1, -1, -1):
            n = n * 8 + (int(z[r, k]) % 8)
        assert bytes(p[r].tolist()) == n.to_bytes(3 * K // 8, "little")


def test_round_trip_of_every_code_at_every_position():
    for pos in range(8):
        for v in range(-4, 4):
            z = np.zeros((1, 8), dtype=np.int64)
            z[0, pos] = v
            p = int3.pack_dense(z)
            assert int3.unpack_dense(p, 8).tolist() == z.tolist()
            # a single code touches only the bytes its three bits fall into
            touched = {(3 * pos + i) // 8 for i in range(3)}
            assert all(p[0, b] == 0 for b in range(3) if b not in touched)


def test_round_trip_random_bytes():
    """Every byte string is a valid row: unpack then pack is the identity."""
    rng = np.random.default_rng(7)
    p = rng.integers(0, 256, size=(6, 3 * 64 // 8), dtype=np.uint8)
    z = int3.unpack_dense(p, 64)
    assert z.min() >= -4 and z.max() <= 3
    assert np.array_equal(int3.pack_dense(z), p)


def test_rows_are_independent_and_unpadded():
    rng = np.random.default_rng(3)
    z = rng.integers(-3, 4, size=(4, 40))
    p = int3.pack_dense(z)
    for r in range(4):
        assert np.array_equal(p[r], int3.pack_dense(z[r:r + 1])[0])
    assert p.tobytes() == b"".join(int3.pack_dense(z[r:r + 1]).tobytes() for r in range(4))


def test_rejects_what_does_not_fit():
    with pytest.raises(ValueError):
        int3.pack_dense(np.array([[4, 0, 0, 0, 0, 0, 0, 0]]))
    with pytest.raises(ValueError):
        int3.pack_dense(np.array([[-5, 0, 0, 0, 0, 0, 0, 0]]))
    with pytest.raises(ValueError):
        int3.pack_dense(np.zeros((1, 12), dtype=np.int64))
    with pytest.raises(ValueError):
        int3.unpack_dense(np.zeros((1, 4), dtype=np.uint8), 8)
