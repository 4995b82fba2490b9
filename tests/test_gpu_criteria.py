"""GPU parity of the alternative reorder criteria (paper Tab. 2a) through the C ABI against the
oracle: per-channel sums to 1e-12 (fp64 accumulation in another order), per-channel maxima and every
permutation bit-exact."""
import sys

import numpy as np
import pytest
import torch

from oracle import calib as OC
from oracle import criteria as OR
from oracle import formats as OF
from paper_2605_09503_amd import pq, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _bits(v):
    return synth.f64_to_bf16_bits(np.asarray(v, dtype=np.float64))


def _dev(bits):
    return pq.bf16_from_bits(bits, DEV)


@pytest.mark.parametrize("rows,K,pad", [(300, 520, 0), (37, 1032, 8), (1, 8, 0), (4608, 3072, 0)])
def test_channel_stats(rows, K, pad):
    _say("channel stats rows=%d K=%d ld=%d" % (rows, K, K + pad))
    rng = np.random.default_rng(9800 + rows + K)
    bits = _bits(rng.standard_normal((rows, K + pad)) * np.exp(rng.standard_normal(K + pad)) + 0.3)
    x = _dev(bits)[:, :K]
    total = torch.zeros(K, dtype=torch.float64, device=DEV)
    amax = torch.zeros(K, dtype=torch.float32, device=DEV)
    pq.pq_calib_channel_stats(x, total, amax, K=K)
    pq.pq_calib_channel_stats(x, total, amax, K=K)                  # two batches: sums add, maxima fold
    sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
    pq.pq_calib_moments(x, sumsq, None, rows=rows, K=K, ld=K + pad)
    pq.pq_calib_moments(x, sumsq, None, rows=rows, K=K, ld=K + pad)
    var = pq.pq_channel_statistic(pq.CRIT_VARIANCE, total, sumsq, None, 2 * rows, torch.empty(K, dtype=torch.float64, device=DEV))
    am2 = pq.pq_channel_statistic(pq.CRIT_ABSMAX, None, None, amax, 0, torch.empty(K, dtype=torch.float64, device=DEV))
    torch.cuda.synchronize()
    x64 = OF.bf16_bits_to_f64(bits[:, :K])
    ref_sum = 2.0 * OR.column_sum(x64)
    scale = 2.0 * np.sum(np.abs(x64), axis=0)
    assert np.all(np.abs(total.cpu().numpy() - ref_sum) <= 1e-12 * scale + 1e-300)
    assert np.array_equal(amax.cpu().numpy(), OR.column_absmax(x64).astype(np.float32))
    assert np.array_equal(am2.cpu().numpy(), OR.column_absmax(x64) ** 2)
    # variance of the doubled sample = 2 x the variance sum of one copy; the one-pass form loses
    # 2^-52 * sumsq / variance relative to the two-pass definition
    ref_var = 2.0 * OR.column_variance_sum(x64)
    ss = 2.0 * OC.column_sumsq(x64)
    assert np.all(np.abs(var.cpu().numpy() - ref_var) <= 1e-12 * ss + 1e-300)


def test_orders_match_the_oracle():
    K, g = 1280, 64
    rng = np.random.default_rng(9810)
    a = np.exp(2 * rng.standard_normal(K))
    w = np.exp(rng.standard_normal(K))
    a_d, w_d = torch.from_numpy(a).to(DEV), torch.from_numpy(w).to(DEV)
    order = torch.empty(K, dtype=torch.int32, device=DEV)
    for alpha in (0.0, 0.4, 1.0):
        pq.pq_order_by_score(a_d, w_d, alpha, order)
        torch.cuda.synchronize()
        assert np.array_equal(order.cpu().numpy(), OC.sort_descending(OC.joint_key(a, w, alpha)))
    rr = torch.empty(K, dtype=torch.int32, device=DEV)
    pq.pq_order_round_robin(order, g, rr)
    rnd = torch.empty(K, dtype=torch.int32, device=DEV)
    pq.pq_order_random(12345, rnd)
    rnd2 = torch.empty(K, dtype=torch.int32, device=DEV)
    pq.pq_order_random(2 ** 63 + 7, rnd2)                      # a seed that wraps modulo 2^64 on the way
    torch.cuda.synchronize()
    assert np.array_equal(rr.cpu().numpy(), OR.round_robin(order.cpu().numpy(), g))
    assert np.array_equal(rnd.cpu().numpy(), OR.random_order(12345, K))
    assert np.array_equal(rnd2.cpu().numpy(), OR.random_order(2 ** 63 + 7, K))


def test_criteria_rank_as_in_the_ablation_on_structured_channels():
    """A few outlier channels among many ordinary ones (the structure the method is built for):
    clustering by the second moment puts the outliers into one group and lowers the quantization error,
    a random order leaves it about where it was, and round-robin (outliers dealt to different groups)
    keeps every outlier's group coarse -- evaluated with pq_quant_error against the oracle's error."""
    rows, K, g, fmt = 96, 1024, 64, pq.FMT_INT4
    rng = np.random.default_rng(9820)
    chan = np.exp(0.3 * rng.standard_normal(K))
    chan[rng.choice(K, 16, replace=False)] *= 30.0
    bits = _bits(rng.standard_normal((rows, K)) * chan)
    x = _dev(bits)
    x64 = OF.bf16_bits_to_f64(bits)
    sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
    pq.pq_calib_moments(x, sumsq, None)
    ones = torch.ones(K, dtype=torch.float64, device=DEV)
    order = pq.pq_order_by_score(sumsq, ones, 1.0, torch.empty(K, dtype=torch.int32, device=DEV))
    rr = pq.pq_order_round_robin(order, g, torch.empty(K, dtype=torch.int32, device=DEV))
    rnd = pq.pq_order_random(1, torch.empty(K, dtype=torch.int32, device=DEV))
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    errs = {}
    for name, p in (("orig", None), ("second_moment", order), ("round_robin", rr), ("random", rnd)):
        pq.pq_quant_error(fmt, g, x, p, 1.0, out)
        torch.cuda.synchronize()
        errs[name] = out.item()
        ref = OC.squared_error(fmt, g, x64, None if p is None else p.cpu().numpy())
        np.testing.assert_allclose(errs[name], ref, rtol=1e-10)
    assert errs["second_moment"] < 0.8 * errs["orig"]
    assert errs["round_robin"] > errs["orig"] > errs["second_moment"]
    assert 0.8 * errs["orig"] < errs["random"] < 1.25 * errs["orig"]
