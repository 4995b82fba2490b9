"""pq_calib_moments_static -- the entry point that allocates nothing (its partial sums live in a device
array the library holds) -- against pq_calib_moments, through the C ABI: two calls in a row, the second
on a smaller input, so that the array still holds the first call's partial sums when the second runs.
Same kernels and summation order: the results must be bit-equal, and both agree with the oracle."""
import numpy as np
import pytest
import torch

from oracle import calib as OC
from oracle import formats as OF
from paper_2605_09503_amd import pq, synth

import pq_testlib as T

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(bits):
    x = pq.bf16_from_bits(bits, DEV)
    K = bits.shape[1]
    out = []
    for fn in (pq.pq_calib_moments_static, pq.pq_calib_moments):
        sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
        amax = torch.zeros(1, dtype=torch.float32, device=DEV)
        fn(x, sumsq, amax)
        fn(x, sumsq, amax)                     # in/out: a second batch (the same tensor) accumulates
        torch.cuda.synchronize()
        out.append((sumsq.cpu().numpy(), amax.item()))
    return out


def test_calib_moments_static_two_calls():
    rng = np.random.default_rng(7700)
    shapes = [(1000, 3072), (77, 520)]         # the second call is smaller and ragged in rows and columns
    for rows, K in shapes:
        print("pq_calib_moments_static rows=%d K=%d" % (rows, K), flush=True)
        bits = synth.f64_to_bf16_bits(rng.standard_normal((rows, K)) * np.exp(rng.standard_normal(K)))
        (s_static, m_static), (s_ws, m_ws) = _both(bits)
        np.testing.assert_array_equal(s_static, s_ws)
        assert m_static == m_ws
        x64 = OF.bf16_bits_to_f64(bits)
        ref = 2.0 * OC.column_sumsq(x64)
        assert np.all(np.abs(s_static - ref) <= T.MOMENTS_RTOL * ref)
        assert m_static == np.float32(OC.absmax(x64))


def test_calib_moments_static_refuses_what_does_not_fit():
    K = 524288
    x = torch.zeros((64, K), dtype=torch.bfloat16, device=DEV)
    sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
    with pytest.raises(pq.PQError) as e:
        pq.pq_calib_moments_static(x, sumsq)
    assert e.value.code == -4
    torch.cuda.synchronize()
    assert float(sumsq.abs().max()) == 0.0     # nothing was launched
