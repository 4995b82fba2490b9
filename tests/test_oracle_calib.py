"""Pins for the oracle's calibration statistics, sort, acceptance rule and product
(paper Sec. 3.2-3.3: Prop. 1, Eq. 8, Eq. 9, acceptance rule)."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import calib as C
from oracle import formats as F
from oracle import gemm as G
from oracle import quantize as Qz
from paper_2605_09503_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bf16(v):
    return F.bf16_bits_to_f64(synth.f64_to_bf16_bits(v))


def _partitions(items, g):
    """All ways to split items into unordered groups of size g."""
    items = list(items)
    if not items:
        yield []
        return
    first, rest = items[0], items[1:]
    for mates in itertools.combinations(rest, g - 1):
        left = [i for i in rest if i not in mates]
        for tail in _partitions(left, g):
            yield [(first,) + mates] + tail


def _partition_counts():
    out = []
    with open(os.path.join(GOLDEN, "partition_counts.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                out.append(tuple(int(t) for t in line.split()))
    return out


def test_partition_enumerator_visits_every_partition():
    for d, g, count in _partition_counts():
        assert sum(1 for _ in _partitions(range(d), g)) == count
        assert count == math.factorial(d) // (math.factorial(g) ** (d // g) * math.factorial(d // g))


# ------------------------------------------------------------------------------ moments

def test_column_sumsq_against_fsum_and_closed_form():
    rng = np.random.default_rng(20)
    x = _bf16(rng.standard_normal((300, 40)) * np.exp(3 * rng.standard_normal(40))[None, :])
    s = C.column_sumsq(x)
    for i in range(40):
        ref = math.fsum(float(v) * float(v) for v in x[:, i])
        assert abs(s[i] - ref) <= 1e-13 * ref
    const = np.full((1000, 3), 1.5)
    np.testing.assert_array_equal(C.column_sumsq(const), [2250.0] * 3)
    # a transposed operand would give row sums instead
    assert s.shape == (40,)
    assert C.absmax(np.array([[1.0, -7.5], [3.0, 2.0]])) == 7.5


# --------------------------------------------------------------------------------- sort

@pytest.mark.parametrize("d,g", [(6, 2), (8, 4), (9, 3), (8, 2)])
def test_sorted_partition_minimises_sum_of_group_maxima(d, g):
    # Prop. 1 and its closed form sum_k a_((k-1)g+1), against every partition
    rng = np.random.default_rng(21 + d + g)
    for _ in range(5):
        a = np.exp(2 * rng.standard_normal(d))
        perm = C.sort_descending(np.log(a))
        srt = np.sort(a)[::-1]
        closed = float(np.sum(srt[0::g]))
        assert np.isclose(C.partition_objective(a, perm, g), closed, rtol=1e-15)
        best = min(sum(max(a[i] for i in grp) for grp in part) for part in _partitions(range(d), g))
        assert np.isclose(best, closed, rtol=1e-12)
        # ascending order would be worse or equal, and strictly worse for distinct values
        # when g does not put the same sets together
        asc = perm[::-1]
        assert C.partition_objective(a, asc, g) >= closed * (1 - 1e-15)


def test_sort_is_descending_stable_bijection():
    key = np.array([1.0, 3.0, 3.0, -np.inf, 2.0, 3.0, -np.inf])
    p = C.sort_descending(key)
    np.testing.assert_array_equal(p, [1, 2, 5, 4, 0, 3, 6])
    rng = np.random.default_rng(22)
    key = rng.standard_normal(1000)
    p = C.sort_descending(key)
    assert sorted(p.tolist()) == list(range(1000))
    assert np.all(np.diff(key[p]) <= 0)


def test_joint_key_endpoints_and_order():
    rng = np.random.default_rng(23)
    sa = np.exp(rng.standard_normal(200))
    sw = np.exp(rng.standard_normal(200))
    # alpha = 1: activation statistics only; alpha = 0: weight statistics only
    np.testing.assert_array_equal(C.sort_descending(C.joint_key(sa, sw, 1.0)), np.argsort(-sa, kind="stable"))
    np.testing.assert_array_equal(C.sort_descending(C.joint_key(sa, sw, 0.0)), np.argsort(-sw, kind="stable"))
    # in between: same order as the power form of Eq. 9
    for a in (0.2, 0.4, 0.6, 0.8):
        v = sa ** a * sw ** (1 - a)
        np.testing.assert_array_equal(C.sort_descending(C.joint_key(sa, sw, a)), np.argsort(-v, kind="stable"))
    # a zero second moment on the side with zero weight does not matter; with weight it sorts last
    sa0 = sa.copy()
    sa0[7] = 0.0
    assert np.isfinite(C.joint_key(sa0, sw, 0.0)).all()
    assert C.sort_descending(C.joint_key(sa0, sw, 0.4))[-1] == 7


# -------------------------------------------------------------------- function preservation

def test_permuting_both_operands_preserves_the_product():
    # Eq. 8: X W = (X P)(P^T W)
    rng = np.random.default_rng(24)
    x = _bf16(rng.standard_normal((37, 96)))
    w = _bf16(0.02 * rng.standard_normal((53, 96)))
    perm = rng.permutation(96)
    y0 = G.plain_product(x, w)
    y1 = G.plain_product(x[:, perm], w[:, perm])
    assert np.max(np.abs(y0 - y1)) <= 1e-12 * np.max(np.abs(y0))
    assert y0.shape == (37, 53)
    # permuting only one side does change it
    assert np.max(np.abs(y0 - G.plain_product(x[:, perm], w))) > 1e-3 * np.max(np.abs(y0))


# -------------------------------------------------------------------------- acceptance

def _tiny_layer(rng, K, M=24, N=12):
    chan = np.exp(1.5 * rng.standard_normal(K))
    x = _bf16(rng.standard_normal((M, K)) * chan[None, :])
    w = _bf16(0.02 * rng.standard_normal((N, K)) * np.exp(0.5 * rng.standard_normal(K))[None, :])
    return x, w


@pytest.mark.parametrize("fmt,K,g", [(F.FMT_INT3, 6, 2), (F.FMT_INT4, 8, 4), (F.FMT_INT3, 8, 2)])
def test_acceptance_never_raises_calibration_error_bruteforce(fmt, K, g):
    rng = np.random.default_rng(30 + K + g)
    n_acc = 0
    for trial in range(6):
        x, w = _tiny_layer(rng, K)
        res = C.select_permutation(fmt, g, [x], w)
        e_out = C.calibration_error(fmt, g, [x], w, res.perm)
        e_id = C.calibration_error(fmt, g, [x], w, None)
        assert e_out <= e_id
        assert np.isclose(res.e_orig, e_id, rtol=1e-14)
        if res.accepted:
            n_acc += 1
            assert e_out < e_id and np.isclose(res.e_best, e_out, rtol=1e-14)
        else:
            np.testing.assert_array_equal(res.perm, np.arange(K))
        # every grouping of the channels: the output is never worse than the original order,
        # and nothing beats the global optimum
        errs = []
        for part in _partitions(range(K), g):
            p = np.array([i for grp in part for i in grp])
            errs.append(C.calibration_error(fmt, g, [x], w, p))
        assert min(errs) <= e_out * (1 + 1e-12)
        assert e_out <= e_id
    assert n_acc > 0


def test_acceptance_threshold_and_identity_candidate():
    rng = np.random.default_rng(40)
    x, w = _tiny_layer(rng, 32, M=64, N=16)
    r0 = C.select_permutation(F.FMT_INT4, 8, [x], w, tau=0.0)
    assert r0.accepted
    gain = (r0.e_orig - r0.e_best) / r0.e_orig
    assert 0 < gain < 1
    # a threshold just above the realised gain rejects, just below accepts (strict >)
    assert not C.select_permutation(F.FMT_INT4, 8, [x], w, tau=gain).accepted
    assert not C.select_permutation(F.FMT_INT4, 8, [x], w, tau=gain * 1.01).accepted
    assert C.select_permutation(F.FMT_INT4, 8, [x], w, tau=gain * 0.99).accepted
    # channels already in descending order for both sides: the sort returns the identity,
    # which is never "accepted"
    K = 16
    xs = np.tile(_bf16(2.0 ** -np.arange(K))[None, :], (4, 1))
    ws = np.tile(_bf16(2.0 ** -np.arange(K))[None, :], (3, 1))
    r = C.select_permutation(F.FMT_INT4, 4, [xs], ws)
    assert not r.accepted
    np.testing.assert_array_equal(r.perm, np.arange(K))
    np.testing.assert_array_equal(r.cand_perms[0], np.arange(K))


def test_alpha_search_picks_smallest_error_and_first_on_ties():
    rng = np.random.default_rng(41)
    x, w = _tiny_layer(rng, 64, M=128, N=32)
    res = C.select_permutation(F.FMT_INT3, 8, [x[:64], x[64:]], w)
    assert len(res.e_cand) == 6
    assert res.alpha_index == int(np.argmin(res.e_cand))
    assert res.e_best == min(res.e_cand)
    for a, p, e in zip(C.DEFAULT_ALPHAS, res.cand_perms, res.e_cand):
        assert np.isclose(e, C.calibration_error(F.FMT_INT3, 8, [x], w, p), rtol=1e-12)
    # two calibration batches count exactly like their concatenation
    res1 = C.select_permutation(F.FMT_INT3, 8, [x], w)
    np.testing.assert_array_equal(res.perm, res1.perm)
    assert np.isclose(res.e_best, res1.e_best, rtol=1e-12)
    # duplicated alphas give equal errors; the first one wins
    res2 = C.select_permutation(F.FMT_INT3, 8, [x], w, alphas=(0.4, 0.4, 1.0, 1.0))
    assert res2.alpha_index in (0, 2)


def test_calibration_error_is_a_sum_of_relative_errors():
    rng = np.random.default_rng(42)
    x, w = _tiny_layer(rng, 32, M=16, N=8)
    e = C.calibration_error(F.FMT_INT4, 8, [x], w, None)
    ex = np.sum((x - Qz.dequantize_int(Qz.quantize_int(x, 8, F.FMT_INT4), 8)) ** 2) / np.sum(x * x)
    ew = np.sum((w - Qz.dequantize_int(Qz.quantize_int(w, 8, F.FMT_INT4), 8)) ** 2) / np.sum(w * w)
    assert np.isclose(e, ex + ew, rtol=1e-14)
    # scaling either tensor by a power of two leaves E unchanged (relative errors)
    assert np.isclose(C.calibration_error(F.FMT_INT4, 8, [4 * x], 0.5 * w, None), e, rtol=1e-13)
    # within-group shuffles and (g | K) reversal leave E unchanged
    p = np.concatenate([k * 8 + rng.permutation(8) for k in range(4)])
    assert np.isclose(C.calibration_error(F.FMT_INT4, 8, [x], w, p), e, rtol=1e-13)
    assert np.isclose(C.calibration_error(F.FMT_INT4, 8, [x], w, np.arange(32)[::-1]), e, rtol=1e-13)


def test_reordering_lowers_the_error_bound():
    # with channel magnitudes spread over orders of magnitude, sorting by second moment puts
    # similar channels together: the bound of Eq. 4 drops.  The realised calibration error may
    # or may not (a group's largest element is always quantized well, which favours spreading
    # the large channels) -- that is what the acceptance rule is for.
    rng = np.random.default_rng(43)
    K = 128
    chan = np.exp(2.0 * rng.standard_normal(K))
    xs = [_bf16(rng.standard_normal((64, K)) * chan[None, :]) for _ in range(2)]
    w = _bf16(0.02 * rng.standard_normal((64, K)) * np.exp(1.0 * rng.standard_normal(K))[None, :])
    for fmt, g in ((F.FMT_NVFP4, 16), (F.FMT_INT4, 32), (F.FMT_INT3, 32)):
        res = C.select_permutation(fmt, g, xs, w)
        assert res.accepted == (res.e_best < res.e_orig)
        assert sorted(res.perm.tolist()) == list(range(K))
        assert res.min_key_gap > 0
        p_act = res.cand_perms[-1]            # alpha = 1: activation statistics only
        x = np.concatenate(xs)
        bound_id = np.sum(np.max(np.abs(x.reshape(len(x), -1, g)), axis=2) ** 2)
        bound_sorted = np.sum(np.max(np.abs(x[:, p_act].reshape(len(x), -1, g)), axis=2) ** 2)
        assert bound_sorted < bound_id
        sa = sum(C.column_sumsq(xb) for xb in xs)
        assert C.partition_objective(sa, p_act, g) < C.partition_objective(sa, np.arange(K), g)


def test_synthetic_config_runs_through_selection():
    cfg = synth.scaled(synth.CONFIGS["c0"], M=64, N=64, K=128, n_calib=2)
    st, calib, _ = synth.make_layer(cfg)
    xs = [F.bf16_bits_to_f64(b) for b in calib]
    w = F.bf16_bits_to_f64(st.w_bits)
    for fmt, g in ((F.FMT_NVFP4, 16), (F.FMT_INT4, 32), (F.FMT_INT3, 32)):
        res = C.select_permutation(fmt, g, xs, w)
        assert sorted(res.perm.tolist()) == list(range(128))
        assert res.e_best == min(res.e_cand)
        assert res.accepted == (res.e_best < res.e_orig)


# ---------------------------------------------------------------------------------- GEMM

def test_dequant_product_exact_small_integers():
    rng = np.random.default_rng(50)
    za = rng.integers(-1, 2, size=(9, 64)).astype(np.int8)
    zw = rng.integers(-1, 2, size=(7, 64)).astype(np.int8)
    qa = Qz.IntQuant(za, np.ones((9, 2), dtype=np.float32))
    qw = Qz.IntQuant(zw, np.ones((7, 2), dtype=np.float32))
    y = G.dequant_product(F.FMT_INT4, 32, qa, qw)
    np.testing.assert_array_equal(y, za.astype(np.int64) @ zw.astype(np.int64).T)


def test_dequant_product_per_token_per_channel_special_case():
    # g = K: textbook per-token x per-output-channel integer GEMM with outer-product scales
    rng = np.random.default_rng(51)
    x = _bf16(rng.standard_normal((11, 128)))
    w = _bf16(0.02 * rng.standard_normal((13, 128)))
    qa = Qz.quantize_int(x, 128, F.FMT_INT4)
    qw = Qz.quantize_int(w, 128, F.FMT_INT4)
    y = G.dequant_product(F.FMT_INT4, 128, qa, qw)
    acc = qa.z.astype(np.int64) @ qw.z.astype(np.int64).T
    ref = acc * (qa.scale.astype(np.float64) @ qw.scale.astype(np.float64).T)
    np.testing.assert_allclose(y, ref, rtol=1e-13)


@pytest.mark.parametrize("fmt,g", [(F.FMT_NVFP4, 16), (F.FMT_INT4, 64), (F.FMT_INT3, 32)])
def test_dequant_product_from_packed_and_error_bound(fmt, g):
    rng = np.random.default_rng(52)
    x = _bf16(rng.standard_normal((24, 256)))
    w = _bf16(0.02 * rng.standard_normal((20, 256)))
    ta = Qz.nvfp4_tensor_scale(np.max(np.abs(x))) if fmt == F.FMT_NVFP4 else np.float32(1)
    tw = Qz.nvfp4_tensor_scale(np.max(np.abs(w))) if fmt == F.FMT_NVFP4 else np.float32(1)
    qa = Qz.quantize(fmt, g, x, ta)
    qw = Qz.quantize(fmt, g, w, tw)
    y = G.dequant_product(fmt, g, qa, qw)
    y2 = G.dequant_product_from_packed(fmt, g, Qz.packed_codes(fmt, qa), qa.scale, ta,
                                       Qz.packed_codes(fmt, qw), qw.scale, tw)
    np.testing.assert_array_equal(y, y2)
    rows = [3, 7]
    np.testing.assert_array_equal(G.dequant_product(fmt, g, qa, qw, rows), y[rows])
    # |Y - Yq| <= ||ex|| ||w|| + ||xhat|| ||ew||  (Cauchy-Schwarz, row by row)
    xh, wh = Qz.dequantize(fmt, g, qa), Qz.dequantize(fmt, g, qw)
    y0 = G.plain_product(x, w)
    bound = (np.linalg.norm(x - xh, axis=1)[:, None] * np.linalg.norm(w, axis=1)[None, :]
             + np.linalg.norm(xh, axis=1)[:, None] * np.linalg.norm(w - wh, axis=1)[None, :])
    assert np.all(np.abs(y - y0) <= bound * (1 + 1e-12))
    assert np.max(np.abs(y - y0)) > 0


def test_bf16_round_of_product():
    y = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5, 0.0])
    bits = G.bf16_round(y)
    back = F.bf16_bits_to_f64(bits)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0)
    np.testing.assert_array_equal(back[:3], [1.0, 1.0, 1.015625])
    assert abs(back[3] + 3.0e-5) < 3.0e-5 * 2.0 ** -8


def test_add_bias_is_a_per_column_offset():
    y = np.arange(6.0).reshape(2, 3)
    out = G.add_bias(y, [10.0, 20.0, 30.0])
    assert out.tolist() == [[10.0, 21.0, 32.0], [13.0, 24.0, 35.0]]


def test_output_error_brute_force_and_invariances():
    """E_out from explicit loops on a tiny layer; zero when nothing is lost; the unquantized product
    does not depend on the order, so a permutation inside one group changes nothing."""
    rng = np.random.default_rng(11)
    K, g, M, N = 8, 4, 3, 2
    x = _bf16(rng.normal(size=(M, K)) * np.array([9, 1, 1, 1, 9, 1, 1, 1.0]))
    w = _bf16(rng.normal(size=(N, K)))
    perm = np.array([0, 4, 1, 2, 3, 5, 6, 7])
    xq = Qz.dequantize(1, g, Qz.quantize(1, g, x[:, perm]))
    wq = Qz.dequantize(1, g, Qz.quantize(1, g, w[:, perm]))
    num = den = 0.0
    for m in range(M):
        for n in range(N):
            y = sum(x[m, k] * w[n, k] for k in range(K))
            yq = sum(xq[m, k] * wq[n, k] for k in range(K))
            num += (y - yq) ** 2
            den += y ** 2
    got = C.output_error(1, g, [x], w, perm)
    assert abs(got - num / den) <= 1e-13 * (num / den)
    # two batches: numerators and denominators add before the division
    x2 = _bf16(rng.normal(size=(M, K)))
    both = C.output_error(1, g, [x, x2], w, perm)
    a = C.output_error(1, g, [x], w, perm)
    b = C.output_error(1, g, [x2], w, perm)
    da = float(np.sum((x @ w.T) ** 2))
    db = float(np.sum((x2 @ w.T) ** 2))
    assert abs(both - (a * da + b * db) / (da + db)) <= 1e-13
    # codes that are exact (integers up to 7 with the group maximum 7) lose nothing
    xi = np.array([[7.0, -3, 2, 0, 7, 1, -1, 5]])
    wi = np.array([[7.0, 7, -7, 1, 7, 0, 2, -4]])
    assert C.output_error(1, g, [xi], wi, None) == 0.0
    # reordering inside a group leaves every group's content, hence the error, unchanged
    inside = np.array([1, 0, 3, 2, 4, 5, 7, 6])
    assert abs(C.output_error(1, g, [x], w, inside) - C.output_error(1, g, [x], w, None)) <= 1e-15


def test_select_permutation_by_output_error():
    """With the layer-output metric the selection follows output_error: argmin over the grid,
    acceptance against the original order; the candidate orders are those of the tensor metric."""
    rng = np.random.default_rng(12)
    K, g = 64, 16
    chan = np.exp(1.5 * rng.normal(size=K))
    xs = [_bf16(rng.normal(size=(24, K)) * chan) for _ in range(2)]
    w = _bf16(0.05 * rng.normal(size=(20, K)) / np.sqrt(chan))
    a = C.select_permutation(1, g, xs, w, metric="tensor")
    b = C.select_permutation(1, g, xs, w, metric="output")
    assert all(np.array_equal(p, q) for p, q in zip(a.cand_perms, b.cand_perms))
    errs = [C.output_error(1, g, xs, w, p) for p in b.cand_perms]
    assert b.e_cand == errs and b.alpha_index == int(np.argmin(errs))
    assert b.e_orig == C.output_error(1, g, xs, w, None)
    assert b.accepted == (errs[b.alpha_index] < b.e_orig)
    assert np.array_equal(b.perm, b.cand_perms[b.alpha_index] if b.accepted else np.arange(K))
    with pytest.raises(ValueError):
        C.select_permutation(1, g, xs, w, metric="other")
