"""GPU parity at the full sizes of the five configurations, in the launch configuration the
benchmark times.  The oracle cannot afford whole tensors here, so it checks sampled token rows
and output channels (rows of a quantized tensor are independent; an output needs one row of
each operand), always including the first and last ones and tile-boundary neighbours.  Moments
are compared on the whole tensor (a plain column sum is cheap)."""
import concurrent.futures as cf
import sys
import time

import numpy as np
import pytest
import torch

from oracle import calib as OC
from oracle import formats as OF
from oracle import gemm as OG
from oracle import quantize as OQ
from paper_2605_09503_amd import pq, synth

import pq_testlib as T

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _sample(n, count, rng, extra=()):
    base = {0, n - 1}
    for e in extra:
        for d in (-1, 0, 1):
            if 0 <= e + d < n:
                base.add(e + d)
    pick = set(rng.choice(n, size=min(count, n), replace=False).tolist())
    return np.array(sorted(base | pick), dtype=np.int64)


# (config, calibration batches used for the moments check)
CASES = [("c1", 8), ("c2", 3), ("c3up", 2), ("c3down", 2), ("c4", 2)]


@pytest.mark.parametrize("name,nb", CASES)
def test_forward_path_full_size(name, nb):
    cfg = synth.CONFIGS[name]
    fmt, g, M, N, K = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K
    _say("full-size %s: fmt=%d g=%d M=%d N=%d K=%d" % (name, fmt, g, M, N, K))
    t0 = time.time()
    st = synth.make_struct(cfg)
    batches = [synth.make_batch(st, b) for b in range(nb)]
    x_bits = synth.make_batch(st, cfg.n_calib)
    _say("  inputs generated in %.1f s" % (time.time() - t0))
    rng = np.random.default_rng(4000 + cfg.cfg_id)
    perm = rng.permutation(K).astype(np.int32)          # any channel order exercises the same kernels
    perm_dev = torch.from_numpy(perm).to(DEV)

    # ---- moments over the calibration batches (one launch) and over W ----------------------
    xs = [pq.bf16_from_bits(b, DEV) for b in batches]
    w = pq.bf16_from_bits(st.w_bits, DEV)
    sa = torch.zeros(K, dtype=torch.float64, device=DEV)
    sw = torch.zeros(K, dtype=torch.float64, device=DEV)
    amax_a = torch.zeros(1, dtype=torch.float32, device=DEV)
    amax_w = torch.zeros(1, dtype=torch.float32, device=DEV)
    pq.pq_calib_moments_batched(xs, sa, amax_a)
    pq.pq_calib_moments(w, sw, amax_w)
    torch.cuda.synchronize()
    ref_sa = np.zeros(K)
    ref_amax_a = 0.0
    for b in batches:
        v = OF.bf16_bits_to_f64(b)
        ref_sa += OC.column_sumsq(v)
        ref_amax_a = max(ref_amax_a, OC.absmax(v))
    w64 = OF.bf16_bits_to_f64(st.w_bits)
    ref_sw = OC.column_sumsq(w64)
    assert np.all(np.abs(sa.cpu().numpy() - ref_sa) <= T.MOMENTS_RTOL * ref_sa)
    assert np.all(np.abs(sw.cpu().numpy() - ref_sw) <= T.MOMENTS_RTOL * ref_sw)
    assert amax_a.item() == np.float32(ref_amax_a)
    assert amax_w.item() == np.float32(OC.absmax(w64))
    _say("  moments ok (%.1f s)" % (time.time() - t0))
    del xs

    # ---- tensor scales, weight and activation quantization ---------------------------------
    ts_a = torch.ones(1, dtype=torch.float32, device=DEV)
    ts_w = torch.ones(1, dtype=torch.float32, device=DEV)
    ta = tw = None
    if fmt == pq.FMT_NVFP4:
        pq.pq_tensor_scale(amax_a, ts_a)
        ta = OQ.nvfp4_tensor_scale(ref_amax_a)
        tw = OQ.nvfp4_tensor_scale(OC.absmax(w64))
        assert np.float32(ts_a.item()) == ta
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    pq.pq_quantize_weights(fmt, g, w, perm_dev, w_codes, w_scales, ts_w)
    x = pq.bf16_from_bits(x_bits, DEV)
    x_perm = x.index_select(1, perm_dev.long()).contiguous()     # what the producer would emit
    pq.pq_quantize_act(fmt, g, x_perm, None, ts_a, a_codes, a_scales)
    torch.cuda.synchronize()
    if fmt == pq.FMT_NVFP4:
        assert np.float32(ts_w.item()) == tw

    rows = _sample(M, 192, rng, extra=(255, 256, 4095, 4096))
    cols = _sample(N, 256, rng, extra=(255, 256, 3071, 3072))
    qa_codes, qa_scales, qa = T.oracle_quantize_bits(fmt, g, x_bits[rows], perm, ta)
    qw_codes, qw_scales, qw = T.oracle_quantize_bits(fmt, g, st.w_bits[cols], perm, tw)
    rows_t = torch.from_numpy(rows).to(DEV)
    cols_t = torch.from_numpy(cols).to(DEV)
    np.testing.assert_array_equal(a_codes[rows_t].cpu().numpy(), qa_codes)
    np.testing.assert_array_equal(a_scales[rows_t].cpu().numpy().view(qa_scales.dtype), qa_scales)
    np.testing.assert_array_equal(w_codes[cols_t].cpu().numpy(), qw_codes)
    np.testing.assert_array_equal(w_scales[cols_t].cpu().numpy().view(qw_scales.dtype), qw_scales)
    _say("  quantizers ok on %d rows / %d channels (%.1f s)" % (len(rows), len(cols), time.time() - t0))

    # ---- GEMM on the sampled outputs ---------------------------------------------------------
    y16 = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm(fmt, g, a_codes, a_scales, ts_a, w_codes, w_scales, ts_w, y16)
    torch.cuda.synchronize()
    y_ref = OG.dequant_product(fmt, g, qa, qw)
    got16 = y16[rows_t][:, cols_t].view(torch.int16).cpu().numpy().view(np.uint16)
    same = T.gemm_bf16_check(got16, y_ref, name)
    # the forward path the benchmark times: activations quantized straight into the operand layout,
    # weights packed into it, product from the packed operands -- the same bits as above, so every
    # check against the oracle carries over
    a_op = pq.pq_quantize_act_packed(fmt, g, x_perm, ts_a)
    ref_op = torch.zeros_like(a_op)
    got_op = torch.zeros_like(a_op)
    pq.pq_pack_operand(fmt, g, a_codes, a_scales, ref_op)
    pq.pq_quantize_act_packed(fmt, g, x_perm, ts_a, got_op)
    w_op = pq.pq_pack_operand(fmt, g, w_codes, w_scales)
    y16p = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_packed(fmt, g, a_op, ts_a, w_op, ts_w, y16p, M, N, K)
    torch.cuda.synchronize()
    assert torch.equal(got_op, ref_op), "fused quantizer and quantize + pack disagree"
    assert torch.equal(y16p.view(torch.int16), y16.view(torch.int16)), "packed and row-major products differ"
    del y16, y16p, a_op, ref_op, got_op, w_op
    y32 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_f32(fmt, g, a_codes, a_scales, ts_a, w_codes, w_scales, ts_w, y32)
    torch.cuda.synchronize()
    rel = T.gemm_f32_check(y32[rows_t][:, cols_t].cpu().numpy(), y_ref, T.abs_product(fmt, g, qa, qw), name, fmt=fmt)
    _say("  gemm ok: max rel %.2e (fp32 out), bf16 identical to rne(ref) on %.4f of outputs (%.1f s)"
         % (rel, same, time.time() - t0))


def _cand_error(args):
    fmt, g, bits, perm, ts = args
    return OC.squared_error(fmt, g, OF.bf16_bits_to_f64(bits), perm, ts)


def _oracle_selection(fmt, g, batches, w_bits, ta, tw, workers=8):
    """The oracle's selection with its error sums computed by a pool of threads, one (candidate, tensor)
    pair each (numpy releases the GIL in its array loops); the arithmetic is that of
    oracle.calib.select_permutation.  Returns (candidate orders incl. None first, E per order, key gaps,
    sum_x2, sum_w2)."""
    K = w_bits.shape[1]
    nb = len(batches)
    ref_sa = np.zeros(K)
    for b in batches:
        ref_sa += OC.column_sumsq(OF.bf16_bits_to_f64(b))
    ref_sw = OC.column_sumsq(OF.bf16_bits_to_f64(w_bits))
    cands = [None] + [OC.sort_descending(OC.joint_key(ref_sa, ref_sw, a)) for a in OC.DEFAULT_ALPHAS]
    gaps = [OC.min_relative_key_gap(OC.joint_key(ref_sa, ref_sw, a), p)
            for a, p in zip(OC.DEFAULT_ALPHAS, cands[1:])]
    tasks = [(fmt, g, bits, p, ts) for p in cands for bits, ts in [(b, ta) for b in batches] + [(w_bits, tw)]]
    with cf.ThreadPoolExecutor(max_workers=workers) as ex:
        errs = list(ex.map(_cand_error, tasks))
    errs = np.array(errs).reshape(len(cands), nb + 1)
    sum_x2, sum_w2 = float(np.sum(ref_sa)), float(np.sum(ref_sw))
    E = [float(sum(e[:nb])) / sum_x2 + float(e[nb]) / sum_w2 for e in errs]
    return cands, E, gaps, sum_x2, sum_w2


# (config, calibration batches: all eight for the benchmark's INT4 layer, two or three elsewhere -- the
# oracle's cost is in the rows, the kernels' launch shapes are in K, N and the format)
SELECT_CASES = [("c1", 8), ("c2", 3), ("c3up", 2), ("c3down", 2), ("c4", 2)]


@pytest.mark.parametrize("name,nb", SELECT_CASES)
def test_select_perm_full_size(name, nb):
    """Whole selection at the full shape of every configuration against the oracle: error sums of the
    original and the six candidate orders, argmin, acceptance and the permutation."""
    cfg = synth.CONFIGS[name]
    fmt, g, M, N, K = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K
    t0 = time.time()
    st = synth.make_struct(cfg)
    batches = [synth.make_batch(st, b) for b in range(nb)]
    _say("select full-size %s (K=%d, %d batches): inputs generated in %.1f s" % (name, K, nb, time.time() - t0))
    xs = [pq.bf16_from_bits(b, DEV) for b in batches]
    w = pq.bf16_from_bits(st.w_bits, DEV)
    sa = torch.zeros(K, dtype=torch.float64, device=DEV)
    sw = torch.zeros(K, dtype=torch.float64, device=DEV)
    amax_a = torch.zeros(1, dtype=torch.float32, device=DEV)
    amax_w = torch.zeros(1, dtype=torch.float32, device=DEV)
    pq.pq_calib_moments_batched(xs, sa, amax_a)
    pq.pq_calib_moments(w, sw, amax_w)
    ta = tw = None
    ts_a = ts_w = 1.0
    if fmt == pq.FMT_NVFP4:
        ta = OQ.nvfp4_tensor_scale(max(OC.absmax(OF.bf16_bits_to_f64(b)) for b in batches))
        tw = OQ.nvfp4_tensor_scale(OC.absmax(OF.bf16_bits_to_f64(st.w_bits)))
        assert np.float32(amax_a.item()) / np.float32(2688.0) == ta
        ts_a, ts_w = float(ta), float(tw)
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out)
    torch.cuda.synchronize()
    _say("  gpu: accepted=%s alpha_index=%d E_orig=%.8g E_best=%.8g (%.1f s)"
         % (rep.accepted, rep.alpha_index, rep.e_orig, rep.e_best, time.time() - t0))
    got_perm = perm_out.cpu().numpy()
    del xs, w

    cands, E, gaps, sum_x2, sum_w2 = _oracle_selection(fmt, g, batches, st.w_bits, ta, tw)
    _say("  oracle error sums done (%.1f s)" % (time.time() - t0))
    assert min(gaps) > 1e-11, "ill-posed: sort keys closer than the moments are accurate"
    j = int(np.argmin(E[1:]))
    accepted = (not np.array_equal(cands[1 + j], np.arange(K))) and (E[0] - E[1 + j]) / E[0] > 0.0
    assert abs((E[0] - E[1 + j]) / E[0]) > 1e-6, "acceptance margin too small for an exact comparison"
    np.testing.assert_allclose(rep.e_orig, E[0], rtol=T.ERRSUM_RTOL)
    np.testing.assert_allclose(rep.e_cand, E[1:], rtol=T.ERRSUM_RTOL)
    np.testing.assert_allclose(rep.sum_x2, sum_x2, rtol=T.MOMENTS_RTOL)
    np.testing.assert_allclose(rep.sum_w2, sum_w2, rtol=T.MOMENTS_RTOL)
    runner_up = np.sort(np.asarray(E[1:]))
    if runner_up[1] - runner_up[0] > 1e-9 * runner_up[0]:      # else several alphas give the same order
        assert rep.alpha_index == j
    assert rep.accepted == accepted
    want = cands[1 + j] if accepted else np.arange(K, dtype=np.int32)
    np.testing.assert_array_equal(got_perm, want)
    # with / without the permutation: the accepted order never raises the calibration error
    assert (not rep.accepted) or rep.e_best < rep.e_orig
