"""Pins for the oracle's alternative reorder criteria (paper Tab. 2a)."""
import numpy as np
import pytest

from oracle import calib as C
from oracle import criteria as R


def test_statistics_by_hand():
    x = np.array([[1.0, -4.0, 2.0], [3.0, 2.0, 2.0], [-2.0, -1.0, 2.0]])
    assert R.column_sum(x).tolist() == [2.0, -3.0, 6.0]
    assert R.column_absmax(x).tolist() == [3.0, 4.0, 2.0]
    # means 2/3, -1, 2: deviations squared and summed
    np.testing.assert_allclose(R.column_variance_sum(x), [14.0 - 4.0 / 3.0, 21.0 - 3.0, 0.0], rtol=1e-15)
    # variance = second moment - n mean^2, and numpy's own variance
    np.testing.assert_allclose(R.column_variance_sum(x), C.column_sumsq(x) - R.column_sum(x) ** 2 / 3, rtol=1e-14)
    np.testing.assert_allclose(R.column_variance_sum(x) / 3, np.var(x, axis=0), rtol=1e-14, atol=1e-16)


def test_round_robin_deal():
    # 8 channels, groups of 2 -> 4 groups: ranks 0..3 open the groups, ranks 4..7 fill them
    order = np.array([7, 6, 5, 4, 3, 2, 1, 0])
    assert R.round_robin(order, 2).tolist() == [7, 3, 6, 2, 5, 1, 4, 0]
    assert R.round_robin(order, 8).tolist() == order.tolist()            # one group: the order itself
    assert R.round_robin(order, 1).tolist() == order.tolist()            # groups of one: also the order
    p = R.round_robin(np.random.default_rng(0).permutation(96), 16)
    assert sorted(p.tolist()) == list(range(96))
    with pytest.raises(ValueError):
        R.round_robin(order, 3)


def test_round_robin_spreads_the_largest_channels():
    rng = np.random.default_rng(1)
    a = np.sort(np.exp(2 * rng.normal(size=64)))[::-1]
    order = np.arange(64)                      # already sorted, largest first
    p = R.round_robin(order, 8)
    top = set(range(8))                        # the eight largest channels
    for grp in range(8):
        assert len(top & set(p[grp * 8:(grp + 1) * 8].tolist())) == 1     # one per group
    assert a[p[0]] == a[0]


def test_splitmix64_reference_values():
    # first outputs of the published generator seeded with 0 (state advanced by the golden-ratio
    # increment before each output: output k is the function applied to the counter k * increment)
    inc = 0x9E3779B97F4A7C15
    outs = [R.splitmix64((k * inc) & R.MASK64) for k in range(3)]
    assert outs == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_random_order_is_a_seeded_permutation():
    p = R.random_order(5, 300)
    assert sorted(p.tolist()) == list(range(300))
    assert np.array_equal(p, R.random_order(5, 300)) and not np.array_equal(p, R.random_order(6, 300))
    # sorted by hash: the hashes along the permutation ascend
    h = [R.splitmix64(5 + int(i)) >> 11 for i in p]
    assert all(h[i] <= h[i + 1] for i in range(299))
    # not close to the identity
    assert np.mean(p == np.arange(300)) < 0.05
