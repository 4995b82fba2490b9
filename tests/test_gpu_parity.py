"""GPU parity: the HIP library against the CPU oracle on the same seeded bits, through the
C ABI.  Sizes are small enough for the oracle to finish in seconds while still spanning
several tiles and ragged tails.  Codes, scales, permutations: bit-exact.  Moments: 1e-12.
Error sums: 1e-10.  GEMM: see pq_testlib."""
import sys

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

FMTS = [(pq.FMT_NVFP4, 16), (pq.FMT_INT4, 64), (pq.FMT_INT4, 32), (pq.FMT_INT3, 32),
        (pq.FMT_INT4, 128), (pq.FMT_INT3, 256)]


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _rand_bits(rng, rows, K, spread=2.0, outliers=4):
    chan = np.exp(spread * 0.5 * rng.standard_normal(K))
    if outliers:
        chan[rng.choice(K, outliers, replace=False)] *= 30.0
    v = rng.standard_normal((rows, K)) * chan[None, :]
    return synth.f64_to_bf16_bits(v)


def _to_dev(bits):
    return pq.bf16_from_bits(bits, DEV)


# ------------------------------------------------------------------------------ moments

@pytest.mark.parametrize("rows,K,ld", [(256, 512, 512), (1000, 264, 264), (37, 1032, 1040), (4608, 3072, 3072),
                                        (1, 8, 8)])
def test_calib_moments(rows, K, ld):
    _say("moments rows=%d K=%d ld=%d" % (rows, K, ld))
    rng = np.random.default_rng(100 + rows)
    bits = _rand_bits(rng, rows, ld)
    x = _to_dev(bits)
    sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
    absmax = torch.zeros(1, dtype=torch.float32, device=DEV)
    pq.pq_calib_moments(x, sumsq, absmax, rows=rows, K=K, ld=ld)
    pq.pq_calib_moments(x, sumsq, absmax, rows=rows, K=K, ld=ld)        # accumulates (in/out)
    torch.cuda.synchronize()
    xf = OF.bf16_bits_to_f64(bits)[:, :K]
    ref = 2.0 * OC.column_sumsq(xf)
    got = sumsq.cpu().numpy()
    assert np.all(np.abs(got - ref) <= T.MOMENTS_RTOL * ref)
    assert absmax.item() == np.float32(OC.absmax(xf))
    # determinism: a second run gives the same bits
    s2 = torch.zeros(K, dtype=torch.float64, device=DEV)
    pq.pq_calib_moments(x, s2, None, rows=rows, K=K, ld=ld)
    pq.pq_calib_moments(x, s2, None, rows=rows, K=K, ld=ld)
    assert torch.equal(s2, sumsq)


@pytest.mark.parametrize("nb,rows,K", [(3, 200, 520), (8, 96, 1024), (19, 40, 256)])
def test_calib_moments_batched(nb, rows, K):
    _say("moments batched nb=%d rows=%d K=%d" % (nb, rows, K))
    rng = np.random.default_rng(150 + nb)
    bits = [_rand_bits(rng, rows, K) for _ in range(nb)]
    xs = [_to_dev(b) for b in bits]
    sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
    absmax = torch.zeros(1, dtype=torch.float32, device=DEV)
    pq.pq_calib_moments_batched(xs, sumsq, absmax)
    torch.cuda.synchronize()
    x64 = [OF.bf16_bits_to_f64(b) for b in bits]
    ref = sum(OC.column_sumsq(x) for x in x64)
    assert np.all(np.abs(sumsq.cpu().numpy() - ref) <= T.MOMENTS_RTOL * ref)
    assert absmax.item() == np.float32(max(OC.absmax(x) for x in x64))


def test_calib_moments_dirty_workspace_and_graph_replays():
    """The workspace of the moments call is scratch nobody clears: whatever bytes it holds, the sums are
    the same, and a captured call gives them again on every replay."""
    rows, K = 1500, 1160
    rng = np.random.default_rng(170)
    bits = _rand_bits(rng, rows, K)
    x = _to_dev(bits)
    xf = OF.bf16_bits_to_f64(bits)
    ref = OC.column_sumsq(xf)
    nbytes = pq.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, 0, 0, rows, 0, K, 1)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for fill in ("ones", "random", "zeros"):
        if fill == "random":
            ws = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=gen)
        else:
            ws = torch.full((nbytes,), 0xFF if fill == "ones" else 0, dtype=torch.uint8, device=DEV)
        sumsq = torch.zeros(K, dtype=torch.float64, device=DEV)
        absmax = torch.zeros(1, dtype=torch.float32, device=DEV)
        pq.pq_calib_moments(x, sumsq, absmax, workspace=ws)
        torch.cuda.synchronize()
        assert np.all(np.abs(sumsq.cpu().numpy() - ref) <= T.MOMENTS_RTOL * ref), fill
        assert absmax.item() == np.float32(OC.absmax(xf))
    # eager result, then a graph of two launches (same workspace) replayed three times with eager work between
    eager = torch.zeros(K, dtype=torch.float64, device=DEV)
    pq.pq_calib_moments(x, eager, None, workspace=ws)
    pq.pq_calib_moments(x, eager, None, workspace=ws)
    torch.cuda.synchronize()
    out = torch.zeros(K, dtype=torch.float64, device=DEV)
    amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    g_ = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_):
        pq.pq_calib_moments(x, out, amax, workspace=ws)
        pq.pq_calib_moments(x, out, amax, workspace=ws)
    for replay in range(3):
        out.zero_()
        amax.zero_()
        torch.cuda.synchronize()
        g_.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from the eager result" % replay
        assert amax.item() == np.float32(OC.absmax(xf))
        scratch = torch.zeros(K, dtype=torch.float64, device=DEV)
        pq.pq_calib_moments(x, scratch, None, workspace=ws)          # eager use of the same workspace in between
        torch.cuda.synchronize()


# ---------------------------------------------------------------------------- quantizers

def _quantize_act_gpu(fmt, g, x, M, K, ld, perm, T_dev):
    codes, scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    codes.fill_(0xAB)
    pq.pq_quantize_act(fmt, g, x, perm, T_dev, codes, scales, M=M, K=K, ld=ld)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy()


@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("M,K", [(256, 512), (67, 768), (1, 256), (515, 2304)])
def test_quantize_act_contiguous(fmt, g, M, K):
    if K % g:
        pytest.skip("K not a multiple of the group")
    _say("quantize_act fmt=%d g=%d M=%d K=%d" % (fmt, g, M, K))
    rng = np.random.default_rng(200 + M + K + g)
    bits = _rand_bits(rng, M, K)
    bits[0, :g] = 0                      # an all-zero group
    bits[M - 1, -1] = 0x8000             # -0.0
    x = _to_dev(bits)
    ts = OQ.nvfp4_tensor_scale(OC.absmax(OF.bf16_bits_to_f64(bits))) if fmt == pq.FMT_NVFP4 else None
    T_dev = torch.tensor([ts], dtype=torch.float32, device=DEV) if ts is not None else None
    codes, scales = _quantize_act_gpu(fmt, g, x, M, K, K, None, T_dev)
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(fmt, g, bits, None, ts)
    np.testing.assert_array_equal(scales.view(ref_scales.dtype), ref_scales)
    np.testing.assert_array_equal(codes, ref_codes)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
def test_quantize_act_strided_and_permuted(fmt, g):
    M, K, ld = 131, 1024, 1040
    _say("quantize_act strided/perm fmt=%d g=%d" % (fmt, g))
    rng = np.random.default_rng(300 + g)
    bits = _rand_bits(rng, M, ld)
    x = _to_dev(bits)
    xb = bits[:, :K]
    ts = OQ.nvfp4_tensor_scale(OC.absmax(OF.bf16_bits_to_f64(xb))) if fmt == pq.FMT_NVFP4 else None
    T_dev = torch.tensor([ts], dtype=torch.float32, device=DEV) if ts is not None else None
    codes, scales = _quantize_act_gpu(fmt, g, x, M, K, ld, None, T_dev)
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(fmt, g, xb, None, ts)
    np.testing.assert_array_equal(codes, ref_codes)
    np.testing.assert_array_equal(scales.view(ref_scales.dtype), ref_scales)
    perm = rng.permutation(K).astype(np.int32)
    perm_dev = torch.from_numpy(perm).to(DEV)
    codes, scales = _quantize_act_gpu(fmt, g, x, M, K, ld, perm_dev, T_dev)
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(fmt, g, xb, perm, ts)
    np.testing.assert_array_equal(codes, ref_codes)
    np.testing.assert_array_equal(scales.view(ref_scales.dtype), ref_scales)


def test_quantize_act_nvfp4_live_values_above_calibration_max():
    # static tensor scale from a smaller calibration maximum: block scales and codes saturate
    M, K = 64, 256
    rng = np.random.default_rng(310)
    bits = _rand_bits(rng, M, K)
    xf = OF.bf16_bits_to_f64(bits)
    ts = OQ.nvfp4_tensor_scale(OC.absmax(xf) / 37.0)
    T_dev = torch.tensor([ts], dtype=torch.float32, device=DEV)
    codes, scales = _quantize_act_gpu(pq.FMT_NVFP4, 16, _to_dev(bits), M, K, K, None, T_dev)
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(pq.FMT_NVFP4, 16, bits, None, ts)
    assert ref_scales.max() == 126
    np.testing.assert_array_equal(codes, ref_codes)
    np.testing.assert_array_equal(scales, ref_scales)
    # zero tensor scale (all-zero calibration set): everything quantizes to signed zero
    T0 = torch.zeros(1, dtype=torch.float32, device=DEV)
    codes, scales = _quantize_act_gpu(pq.FMT_NVFP4, 16, _to_dev(bits), M, K, K, None, T0)
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(pq.FMT_NVFP4, 16, bits, None, np.float32(0))
    np.testing.assert_array_equal(codes, ref_codes)
    np.testing.assert_array_equal(scales, ref_scales)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
@pytest.mark.parametrize("use_perm", [False, True])
def test_quantize_weights(fmt, g, use_perm):
    N, K = 203, 1280
    _say("quantize_weights fmt=%d g=%d perm=%s" % (fmt, g, use_perm))
    rng = np.random.default_rng(400 + g + use_perm)
    bits = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)) * np.exp(0.3 * rng.standard_normal(K)))
    w = _to_dev(bits)
    perm = rng.permutation(K).astype(np.int32) if use_perm else None
    perm_dev = torch.from_numpy(perm).to(DEV) if use_perm else None
    codes, scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    ts_out = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    pq.pq_quantize_weights(fmt, g, w, perm_dev, codes, scales, ts_out)
    torch.cuda.synchronize()
    if fmt == pq.FMT_NVFP4:
        ts = OQ.nvfp4_tensor_scale(OC.absmax(OF.bf16_bits_to_f64(bits)))
        assert np.float32(ts_out.item()) == ts
    else:
        ts = None
        assert ts_out.item() == 1.0
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(fmt, g, bits, perm, ts)
    np.testing.assert_array_equal(codes.cpu().numpy(), ref_codes)
    np.testing.assert_array_equal(scales.cpu().numpy().view(ref_scales.dtype), ref_scales)


# ------------------------------------------------------------------------------ selection

def _layer_on_gpu(cfg):
    st, calib, test = synth.make_layer(cfg)
    xs = [_to_dev(b) for b in calib]
    w = _to_dev(st.w_bits)
    return st, calib, test, xs, w


def _gpu_moments(xs, w, K):
    sa = torch.zeros(K, dtype=torch.float64, device=DEV)
    sw = torch.zeros(K, dtype=torch.float64, device=DEV)
    amax_a = torch.zeros(1, dtype=torch.float32, device=DEV)
    amax_w = torch.zeros(1, dtype=torch.float32, device=DEV)
    for xb in xs:
        pq.pq_calib_moments(xb, sa, amax_a)
    pq.pq_calib_moments(w, sw, amax_w)
    torch.cuda.synchronize()
    return sa, sw, amax_a.item(), amax_w.item()


@pytest.mark.parametrize("name,fmt,g,M,N,K,nb", [
    ("c0", pq.FMT_NVFP4, 16, 256, 512, 512, 4),
    ("c1", pq.FMT_INT4, 64, 160, 192, 768, 3),
    ("c2", pq.FMT_NVFP4, 16, 96, 128, 1024, 2),
    ("c3down", pq.FMT_NVFP4, 16, 64, 96, 2048, 2),
    ("c4", pq.FMT_INT3, 32, 200, 160, 640, 3),
    # wide rows: the sort at 96 / 128 key chunks and the error evaluation with two rows (K = 12288, the
    # down projection's width) or one row (K = 16384) resident in LDS, identity + six candidates
    ("c3down", pq.FMT_NVFP4, 16, 64, 96, 12288, 2),
    ("c4", pq.FMT_INT3, 32, 40, 48, 12288, 2),
    ("c1", pq.FMT_INT4, 64, 48, 64, 16384, 2),
    ("c2", pq.FMT_NVFP4, 16, 40, 48, 16384, 2),
])
def test_select_perm_matches_oracle(name, fmt, g, M, N, K, nb):
    _say("select_perm %s fmt=%d g=%d M=%d N=%d K=%d" % (name, fmt, g, M, N, K))
    base = synth.CONFIGS[name]
    cfg = synth.scaled(base, M=M, N=N, K=K, n_calib=nb, n_outlier=min(base.n_outlier, K // 64))
    st, calib, test, xs, w = _layer_on_gpu(cfg)
    sa, sw, amax_a, amax_w = _gpu_moments(xs, w, K)
    xs64 = [OF.bf16_bits_to_f64(b) for b in calib]
    w64 = OF.bf16_bits_to_f64(st.w_bits)
    ts_a = ts_w = 1.0
    if fmt == pq.FMT_NVFP4:
        ts_a = float(OQ.nvfp4_tensor_scale(max(OC.absmax(x) for x in xs64)))
        ts_w = float(OQ.nvfp4_tensor_scale(OC.absmax(w64)))
        assert np.float32(amax_a) == np.float32(max(OC.absmax(x) for x in xs64))
    ref = OC.select_permutation(fmt, g, xs64, w64, act_tensor_scale=np.float32(ts_a) if fmt == pq.FMT_NVFP4 else None)
    assert ref.min_key_gap > 1e-11, "ill-posed case (sort keys closer than the moments are accurate): reseed"
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out)
    torch.cuda.synchronize()
    np.testing.assert_allclose(rep.e_orig, ref.e_orig, rtol=T.ERRSUM_RTOL)
    np.testing.assert_allclose(rep.e_cand, ref.e_cand, rtol=T.ERRSUM_RTOL)
    margin = abs((ref.e_orig - ref.e_best) / ref.e_orig)
    assert margin > 1e-6, "acceptance margin too small for a bit-exact comparison: reseed"
    assert rep.accepted == ref.accepted
    assert rep.alpha_index == ref.alpha_index
    np.testing.assert_array_equal(perm_out.cpu().numpy(), ref.perm)
    # every candidate order of the grid, not only the winner (the same key / rank kernels, one alpha a call)
    order = torch.empty(K, dtype=torch.int32, device=DEV)
    for a, p_ref in zip(OC.DEFAULT_ALPHAS, ref.cand_perms):
        pq.pq_order_by_score(sa, sw, a, order)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(order.cpu().numpy(), p_ref)
    # the variant that reads the tensor scales from device memory: the same numbers bit for bit
    perm_dev = torch.empty(K, dtype=torch.int32, device=DEV)
    ta_d = torch.tensor([ts_a], dtype=torch.float32, device=DEV)
    tw_d = torch.tensor([ts_w], dtype=torch.float32, device=DEV)
    rep_d = pq.pq_select_perm_device_scales(fmt, g, sa, sw, xs, w, ta_d, tw_d, perm_dev)
    torch.cuda.synchronize()
    assert rep_d == rep and torch.equal(perm_dev, perm_out)
    if fmt != pq.FMT_NVFP4:                 # the integer formats have no tensor scale: the pointers may be NULL
        rep_n = pq.pq_select_perm_device_scales(fmt, g, sa, sw, xs, w, None, None, perm_dev)
        torch.cuda.synchronize()
        assert rep_n == rep and torch.equal(perm_dev, perm_out)
    # acceptance never raises the calibration error
    assert rep.e_best <= rep.e_orig or not rep.accepted
    # tau above the realised gain rejects and returns the identity
    rep2 = pq.pq_select_perm(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out, tau=0.999)
    torch.cuda.synchronize()
    assert not rep2.accepted
    np.testing.assert_array_equal(perm_out.cpu().numpy(), np.arange(K))


@pytest.mark.parametrize("name,fmt,g,M,N,K,nb", [
    ("c0", pq.FMT_NVFP4, 16, 256, 512, 512, 4),
    ("c1", pq.FMT_INT4, 64, 160, 192, 768, 3),
    ("c4", pq.FMT_INT3, 32, 200, 150, 640, 2),      # N not a multiple of 8: padded fp32 rows
])
def test_select_perm_output_error_matches_oracle(name, fmt, g, M, N, K, nb):
    """The selection with the layer-output metric.  Both products accumulate in fp32 on the GPU, the
    oracle in fp64: the error ratios agree to 1e-4 (their difference of nearly equal numbers amplifies
    the 1e-7 of the accumulation), and argmin / acceptance are compared only where the oracle's margins
    are far above that."""
    _say("select_perm_output_error %s fmt=%d g=%d M=%d N=%d K=%d" % (name, fmt, g, M, N, K))
    base = synth.CONFIGS[name]
    cfg = synth.scaled(base, M=M, N=N, K=K, n_calib=nb, n_outlier=min(base.n_outlier, K // 64))
    st, calib, test, xs, w = _layer_on_gpu(cfg)
    sa, sw, amax_a, amax_w = _gpu_moments(xs, w, K)
    xs64 = [OF.bf16_bits_to_f64(b) for b in calib]
    w64 = OF.bf16_bits_to_f64(st.w_bits)
    ts_a = ts_w = 1.0
    if fmt == pq.FMT_NVFP4:
        ts_a = float(OQ.nvfp4_tensor_scale(max(OC.absmax(x) for x in xs64)))
        ts_w = float(OQ.nvfp4_tensor_scale(OC.absmax(w64)))
    ref = OC.select_permutation(fmt, g, xs64, w64, act_tensor_scale=np.float32(ts_a) if fmt == pq.FMT_NVFP4 else None,
                                metric="output")
    assert ref.min_key_gap > 1e-11
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm_output_error(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out)
    torch.cuda.synchronize()
    np.testing.assert_allclose(rep.e_orig, ref.e_orig, rtol=1e-4)
    np.testing.assert_allclose(rep.e_cand, ref.e_cand, rtol=1e-4)
    np.testing.assert_allclose(rep.sum_x2, sum(float(np.sum((x @ w64.T) ** 2)) for x in xs64), rtol=1e-6)
    e = np.sort(np.asarray(ref.e_cand))
    assert (e[1] - e[0]) / e[0] > 1e-3 and abs(ref.e_orig - ref.e_best) / ref.e_orig > 1e-3, \
        "margins too small for comparing the decisions: reseed"
    assert rep.alpha_index == ref.alpha_index and rep.accepted == ref.accepted
    np.testing.assert_array_equal(perm_out.cpu().numpy(), ref.perm)
    # determinism: a second run gives the same numbers bit for bit
    rep_b = pq.pq_select_perm_output_error(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out)
    assert rep_b.e_cand == rep.e_cand and rep_b.e_orig == rep.e_orig
    # a threshold above any gain rejects
    rep2 = pq.pq_select_perm_output_error(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out, tau=0.999)
    torch.cuda.synchronize()
    assert not rep2.accepted
    np.testing.assert_array_equal(perm_out.cpu().numpy(), np.arange(K))


def test_select_perm_candidates_and_ties():
    # equal second moments: the sort must keep ascending channel index (stable)
    K, M, N = 256, 32, 32
    xb = np.tile(synth.f64_to_bf16_bits(np.repeat(2.0 ** -np.arange(K // 16), 16))[None, :], (M, 1))
    wb = np.tile(synth.f64_to_bf16_bits(np.repeat(2.0 ** -np.arange(K // 16), 16))[None, :], (N, 1))
    xs = [_to_dev(xb)]
    w = _to_dev(wb)
    sa, sw, _, _ = _gpu_moments(xs, w, K)
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(pq.FMT_INT4, 32, sa, sw, xs, w, 1.0, 1.0, perm_out)
    torch.cuda.synchronize()
    assert not rep.accepted          # every candidate is the identity
    np.testing.assert_array_equal(perm_out.cpu().numpy(), np.arange(K))
    ref = OC.select_permutation(pq.FMT_INT4, 32, [OF.bf16_bits_to_f64(xb)], OF.bf16_bits_to_f64(wb))
    assert not ref.accepted
    np.testing.assert_allclose(rep.e_cand, ref.e_cand, rtol=1e-10, atol=1e-300)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
def test_quant_error(fmt, g):
    rows, K = 77, 1024
    rng = np.random.default_rng(500 + g)
    bits = _rand_bits(rng, rows, K)
    x = _to_dev(bits)
    x64 = OF.bf16_bits_to_f64(bits)
    ts = float(OQ.nvfp4_tensor_scale(OC.absmax(x64))) if fmt == pq.FMT_NVFP4 else 1.0
    perm = rng.permutation(K).astype(np.int32)
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    for p in (None, perm):
        pq.pq_quant_error(fmt, g, x, None if p is None else torch.from_numpy(p).to(DEV), ts, out)
        torch.cuda.synchronize()
        ref = OC.squared_error(fmt, g, x64, p, np.float32(ts) if fmt == pq.FMT_NVFP4 else None)
        np.testing.assert_allclose(out.item(), ref, rtol=T.ERRSUM_RTOL)


# Shapes that walk the launch variants of the error evaluation: one, two or four rows resident in
# LDS (by K), workgroup sizes that do and do not divide K / 8, row counts with ragged tails.
@pytest.mark.parametrize("fmt,g,rows,K", [
    (pq.FMT_NVFP4, 16, 5, 272),       # 34 chunks of 8: a single wave with idle lanes
    (pq.FMT_INT4, 32, 13, 4096),      # two rows resident
    (pq.FMT_INT4, 64, 9, 8192),       # two rows resident, one workgroup per compute unit
    (pq.FMT_INT4, 64, 5, 16384),      # one row resident
    (pq.FMT_INT3, 32, 70, 3072),      # four rows resident, 384 threads, 70 = 4 * 17 + 2 rows
    (pq.FMT_NVFP4, 16, 3, 12288),     # widest configuration, fewer rows than a workgroup covers
    (pq.FMT_INT4, 256, 1, 256),       # one row, one group
])
def test_quant_error_launch_variants(fmt, g, rows, K):
    _say("quant_error variants fmt=%d g=%d rows=%d K=%d" % (fmt, g, rows, K))
    rng = np.random.default_rng(900 + K + rows)
    bits = _rand_bits(rng, rows, K)
    x = _to_dev(bits)
    x64 = OF.bf16_bits_to_f64(bits)
    ts = float(OQ.nvfp4_tensor_scale(OC.absmax(x64))) if fmt == pq.FMT_NVFP4 else 1.0
    perm = rng.permutation(K).astype(np.int32)
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    for p in (None, perm):
        pq.pq_quant_error(fmt, g, x, None if p is None else torch.from_numpy(p).to(DEV), ts, out)
        torch.cuda.synchronize()
        ref = OC.squared_error(fmt, g, x64, p, np.float32(ts) if fmt == pq.FMT_NVFP4 else None)
        np.testing.assert_allclose(out.item(), ref, rtol=T.ERRSUM_RTOL)


@pytest.mark.parametrize("shrink", [2.0, 5.0, 64.0, 4096.0, 1e9])
def test_quant_error_nvfp4_tensor_scale_too_small(shrink):
    """A tensor scale smaller than the data calls for saturates block scales at 448: up to a factor 7
    the kernel keeps its exact fp32 group sums, beyond it the wave takes the element-wise fp64 sum;
    either way the error is the oracle's (which clips the block scale the same way)."""
    rows, K = 41, 1536
    _say("quant_error nvfp4 shrunken tensor scale / %g" % shrink)
    rng = np.random.default_rng(1700)
    bits = _rand_bits(rng, rows, K)
    x = _to_dev(bits)
    x64 = OF.bf16_bits_to_f64(bits)
    ts = float(np.float32(float(OQ.nvfp4_tensor_scale(OC.absmax(x64))) / shrink))
    perm = rng.permutation(K).astype(np.int32)
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    for p in (None, perm):
        pq.pq_quant_error(pq.FMT_NVFP4, 16, x, None if p is None else torch.from_numpy(p).to(DEV), ts, out)
        torch.cuda.synchronize()
        ref = OC.squared_error(pq.FMT_NVFP4, 16, x64, p, np.float32(ts))
        np.testing.assert_allclose(out.item(), ref, rtol=T.ERRSUM_RTOL)


def test_nvfp4_error_of_exactly_representable_data_is_zero():
    """Tensors made of E2M1 values times a power-of-two block scale times the tensor scale quantize
    without loss in the original order (every group carries its own 6 s T); a reorder mixes block scales
    inside groups and does lose.  NVFP4 errors are computed as a difference (sum of squares minus the
    cross terms), so the kernel's raw sum is zero only up to a rounding of that difference:
    pq_quant_error returns it clamped at zero (at most 1e-13 of the sum of squares), pq_select_perm
    reports exactly 0, as the oracle does, and keeps the original order."""
    K, M, N, g = 512, 48, 32, 16
    rng = np.random.default_rng(4242)
    e2m1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    ts = 2.0 ** -7

    def exact(rows, t):
        q = rng.choice(e2m1, size=(rows, K)) * rng.choice([-1.0, 1.0], size=(rows, K))
        q[:, ::g] = 6.0                                         # every group's maximum fixes its scale
        scale = 2.0 ** rng.integers(-3, 4, size=(rows, K // g))
        scale[0, 0] = 448.0                                     # the tensor's maximum is 6 * 448 * t
        return synth.f64_to_bf16_bits(q * np.repeat(scale, g, axis=1) * t)

    ts_w = 2.0 ** -10
    xb, wb = exact(M, ts), exact(N, ts_w)
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    assert float(OQ.nvfp4_tensor_scale(OC.absmax(w64))) == ts_w      # the scale the oracle derives for W
    assert OC.squared_error(pq.FMT_NVFP4, g, x64, None, np.float32(ts)) == 0.0
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    pq.pq_quant_error(pq.FMT_NVFP4, g, _to_dev(xb), None, ts, out)
    torch.cuda.synchronize()
    assert 0.0 <= out.item() <= 1e-13 * np.sum(x64 * x64)
    xs, w = [_to_dev(xb)], _to_dev(wb)
    sa, sw, _, _ = _gpu_moments(xs, w, K)
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(pq.FMT_NVFP4, g, sa, sw, xs, w, ts, ts_w, perm_out)
    torch.cuda.synchronize()
    ref = OC.select_permutation(pq.FMT_NVFP4, g, [x64], w64, act_tensor_scale=np.float32(ts))
    assert rep.e_orig == 0.0 and ref.e_orig == 0.0 and not rep.accepted and not ref.accepted
    np.testing.assert_allclose(rep.e_cand, ref.e_cand, rtol=1e-10, atol=1e-13)
    assert min(rep.e_cand) > 1e-6                              # every reorder loses
    np.testing.assert_array_equal(perm_out.cpu().numpy(), np.arange(K))


@pytest.mark.parametrize("fmt,g", [(pq.FMT_INT4, 32), (pq.FMT_NVFP4, 16)])
def test_select_perm_repeated_orders(fmt, g):
    """Weights whose columns all have the same second moment: alpha = 0 sorts equal keys, i.e. keeps the
    original order, and every alpha > 0 sorts by the activations' moments alone -- five times the same
    order.  The library evaluates an order once and hands its error to the repeats: e_cand[0] is e_orig
    bit for bit, e_cand[1..5] are one number, and everything equals the oracle, which evaluates all seven."""
    K, M, N = 768, 40, 24
    _say("select repeated orders fmt=%d" % fmt)
    rng = np.random.default_rng(808 + fmt)
    col = 1.03 ** rng.permutation(K)                           # well separated column scales
    xb = synth.f64_to_bf16_bits(rng.standard_normal((M, K)) * col[None, :])
    wb = synth.f64_to_bf16_bits(np.sign(rng.standard_normal((N, K))))      # every column: N ones
    xs, w = [_to_dev(xb)], _to_dev(wb)
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    sa, sw, _, _ = _gpu_moments(xs, w, K)
    assert torch.all(sw == float(N))
    ts_a = float(OQ.nvfp4_tensor_scale(OC.absmax(x64))) if fmt == pq.FMT_NVFP4 else 1.0
    ts_w = float(OQ.nvfp4_tensor_scale(OC.absmax(w64))) if fmt == pq.FMT_NVFP4 else 1.0
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(fmt, g, sa, sw, xs, w, ts_a, ts_w, perm_out)
    torch.cuda.synchronize()
    ref = OC.select_permutation(fmt, g, [x64], w64)
    np.testing.assert_array_equal(ref.cand_perms[0], np.arange(K))
    for j in range(2, 6):
        np.testing.assert_array_equal(ref.cand_perms[j], ref.cand_perms[1])
    assert rep.e_cand[0] == rep.e_orig and len(set(rep.e_cand[1:6])) == 1
    np.testing.assert_allclose(rep.e_orig, ref.e_orig, rtol=1e-10)
    np.testing.assert_allclose(rep.e_cand, ref.e_cand, rtol=1e-10)
    assert rep.accepted == ref.accepted and rep.alpha_index == ref.alpha_index
    np.testing.assert_array_equal(perm_out.cpu().numpy(), ref.perm)


def test_select_perm_equal_keys_across_sort_chunks():
    """Two key values alternating over 1280 channels (five 256-key chunks of the counting sort):
    the stable descending order is all even channels, then all odd ones.  Every alpha gives the
    same order, so a threshold below any gain returns exactly that order."""
    K, M, N = 1280, 24, 40
    pattern = np.where(np.arange(K) % 2 == 0, 1.0, 0.25)
    rng = np.random.default_rng(77)
    xb = synth.f64_to_bf16_bits(np.sign(rng.standard_normal((M, K))) * pattern[None, :])
    wb = synth.f64_to_bf16_bits(np.sign(rng.standard_normal((N, K))) * pattern[None, :])
    xs = [_to_dev(xb)]
    w = _to_dev(wb)
    sa, sw, _, _ = _gpu_moments(xs, w, K)
    want = np.concatenate([np.arange(0, K, 2), np.arange(1, K, 2)]).astype(np.int32)
    for a in OC.DEFAULT_ALPHAS:
        np.testing.assert_array_equal(OC.sort_descending(OC.joint_key(sa.cpu().numpy(), sw.cpu().numpy(), a)), want)
    perm_out = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(pq.FMT_INT4, 64, sa, sw, xs, w, 1.0, 1.0, perm_out, tau=-1e30)
    torch.cuda.synchronize()
    # groups of equal magnitudes leave only the rounding of the scale amax / Q as error
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    e_ref = (OC.squared_error(pq.FMT_INT4, 64, x64, want, None) / np.sum(x64 * x64)
             + OC.squared_error(pq.FMT_INT4, 64, w64, want, None) / np.sum(w64 * w64))
    assert rep.accepted and rep.alpha_index == 0 and rep.e_orig > 1e-4
    assert e_ref < 1e-12
    np.testing.assert_allclose(rep.e_best, e_ref, rtol=T.ERRSUM_RTOL)
    np.testing.assert_array_equal(perm_out.cpu().numpy(), want)


# ----------------------------------------------------------------------------------- GEMM

def _gemm_case(fmt, g, M, N, K, seed, ldy_pad=0):
    rng = np.random.default_rng(seed)
    xb = _rand_bits(rng, M, K)
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)) * np.exp(0.3 * rng.standard_normal(K)))
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    if fmt == pq.FMT_NVFP4:
        ta, tw = OQ.nvfp4_tensor_scale(OC.absmax(x64)), OQ.nvfp4_tensor_scale(OC.absmax(w64))
    else:
        ta = tw = None
    qa = OQ.quantize(fmt, g, x64, ta)
    qw = OQ.quantize(fmt, g, w64, tw)
    y_ref = OG.dequant_product(fmt, g, qa, qw)
    # GPU operands come from the GPU quantizers (already checked bit-exact above)
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    Ta = torch.tensor([ta if ta is not None else 1.0], dtype=torch.float32, device=DEV)
    Tw = torch.empty(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_act(fmt, g, _to_dev(xb), None, Ta, a_codes, a_scales)
    pq.pq_quantize_weights(fmt, g, _to_dev(wb), None, w_codes, w_scales, Tw)
    np.testing.assert_array_equal(a_codes.cpu().numpy(), OQ.packed_codes(fmt, qa))
    np.testing.assert_array_equal(w_codes.cpu().numpy(), OQ.packed_codes(fmt, qw))
    ldy = (N + 7) // 8 * 8 + ldy_pad
    y32 = torch.full((M, ldy), 777.0, dtype=torch.float32, device=DEV)
    y16 = torch.full((M, ldy), 777.0, dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_f32(fmt, g, a_codes, a_scales, Ta, w_codes, w_scales, Tw, y32, M=M, N=N, K=K, ldy=ldy)
    pq.pq_qgemm(fmt, g, a_codes, a_scales, Ta, w_codes, w_scales, Tw, y16, M=M, N=N, K=K, ldy=ldy)
    torch.cuda.synchronize()
    y32h = y32.cpu().numpy()
    y16h = y16.view(torch.int16).cpu().numpy().view(np.uint16)
    rel = T.gemm_f32_check(y32h[:, :N], y_ref, T.abs_product(fmt, g, qa, qw), "fmt=%d g=%d" % (fmt, g), fmt=fmt)
    same = T.gemm_bf16_check(y16h[:, :N], y_ref, "fmt=%d g=%d" % (fmt, g))
    # nothing written beyond column N
    assert np.all(y32h[:, N:] == 777.0)
    _say("  gemm fmt=%d g=%d %dx%dx%d: max rel %.2e, bf16 identical %.4f" % (fmt, g, M, N, K, rel, same))


@pytest.mark.parametrize("fmt,g", FMTS)
def test_qgemm_small_ragged(fmt, g):
    # 128x128 tiles, several of them, ragged in M and N
    K = 512 if g <= 128 else 768
    _gemm_case(fmt, g, 200, 328, K, 600 + g)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
def test_qgemm_large_tile_path(fmt, g):
    # enough outputs to select the large-tile kernel -- here the 224 x 256 tile (wave rows of 128 + 96),
    # 11 x 15 of them; ragged edges; odd tile count
    _gemm_case(fmt, g, 2304 + 40, 3584 + 72, 256, 700 + g, ldy_pad=8)


@pytest.mark.parametrize("fmt,g", [(pq.FMT_NVFP4, 16), (pq.FMT_INT4, 64)])
def test_qgemm_square_tile_path(fmt, g):
    # 16 x 16 tiles of 256 x 256 fill the compute units exactly (tiles 224 rows high would need a second
    # round), so the square tile is chosen; ragged last row and column of tiles
    _gemm_case(fmt, g, 4096 - 6, 4096 - 9, 128, 750 + g)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
def test_qgemm_tiny(fmt, g):
    _gemm_case(fmt, g, 1, 8, 2 * max(g, 32), 800 + g)
    _gemm_case(fmt, g, 33, 17, 64 if g <= 64 else g, 810 + g)


@pytest.mark.parametrize("fmt,g", FMTS[:4])
def test_qgemm_prep_then_run_equals_one_call(fmt, g):
    M, N, K = 300, 264, 512
    rng = np.random.default_rng(850 + g)
    xb = _rand_bits(rng, M, K)
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)))
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    Ta = torch.tensor([0.01], dtype=torch.float32, device=DEV)
    Tw = torch.empty(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_act(fmt, g, _to_dev(xb), None, Ta, a_codes, a_scales)
    pq.pq_quantize_weights(fmt, g, _to_dev(wb), None, w_codes, w_scales, Tw)
    ws = torch.empty(max(16, pq.pq_workspace_bytes(pq.OP_QGEMM, fmt, g, M, N, K)), dtype=torch.uint8, device=DEV)
    y1 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    y2 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm(fmt, g, a_codes, a_scales, Ta, w_codes, w_scales, Tw, y1, workspace=ws)
    ws.zero_()
    pq.pq_qgemm_prep(fmt, g, a_scales, w_scales, M, N, K, ws)
    pq.pq_qgemm_run(fmt, g, a_codes, a_scales, Ta, w_codes, w_scales, Tw, y2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))


def test_qgemm_int_exact_small_integers():
    # all scales 1 (h = Q), codes in {-1, 0, 1}: the accumulator holds Q^2 times an exact small
    # integer; the epilogue's two fp32 factors 2^E/Q each round once (<= 3 roundings in all)
    M, N, K, g = 70, 90, 256, 64
    rng = np.random.default_rng(900)
    za = rng.integers(-1, 2, size=(M, K))
    zw = rng.integers(-1, 2, size=(N, K))
    a_codes = torch.from_numpy(OF.pack_nibbles(OF.int_to_nibble(za))).to(DEV)
    w_codes = torch.from_numpy(OF.pack_nibbles(OF.int_to_nibble(zw))).to(DEV)
    sa = torch.ones((M, K // g), dtype=torch.float32, device=DEV)
    sw = torch.ones((N, K // g), dtype=torch.float32, device=DEV)
    y = torch.zeros((M, 96), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_f32(pq.FMT_INT4, g, a_codes, sa, None, w_codes, sw, None, y, M=M, N=N, K=K, ldy=96)
    torch.cuda.synchronize()
    np.testing.assert_allclose(y.cpu().numpy()[:, :N], (za @ zw.T).astype(np.float32), rtol=3 * 2.0 ** -24, atol=0)


def test_qgemm_int_wide_scale_range():
    # groups spanning 2^20 in magnitude inside one row stay exact in the fp16 operands
    M, N, K, g = 64, 64, 512, 64
    rng = np.random.default_rng(910)
    scale_a = 2.0 ** rng.integers(-10, 10, size=K // g)
    xb = synth.f64_to_bf16_bits(rng.standard_normal((M, K)) * np.repeat(scale_a, g)[None, :])
    wb = synth.f64_to_bf16_bits(rng.standard_normal((N, K)) * np.repeat(scale_a[::-1], g)[None, :])
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    qa, qw = OQ.quantize(pq.FMT_INT4, g, x64), OQ.quantize(pq.FMT_INT4, g, w64)
    y_ref = OG.dequant_product(pq.FMT_INT4, g, qa, qw)
    a_codes, a_scales = pq.alloc_quantized(pq.FMT_INT4, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(pq.FMT_INT4, g, N, K, DEV)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_act(pq.FMT_INT4, g, _to_dev(xb), None, None, a_codes, a_scales)
    pq.pq_quantize_weights(pq.FMT_INT4, g, _to_dev(wb), None, w_codes, w_scales, one)
    y = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_f32(pq.FMT_INT4, g, a_codes, a_scales, None, w_codes, w_scales, None, y)
    torch.cuda.synchronize()
    # Outputs here cancel heavily, so the error is measured against sum_k |xhat_k * what_k|: fp32
    # accumulation of K terms stays within a few units of 2^-24 of it, while operands rounded
    # to fp16 (instead of folded exactly) would be off by ~2^-12 / sqrt(K) of it.
    mag = np.abs(OQ.dequantize(pq.FMT_INT4, g, qa)) @ np.abs(OQ.dequantize(pq.FMT_INT4, g, qw)).T
    err = np.abs(y.cpu().numpy().astype(np.float64) - y_ref)
    assert np.all(err <= 32 * 2.0 ** -24 * mag), float((err / mag).max())


def test_qgemm_int_group_far_below_row_maximum():
    """Documented edge of the INT product: the operand of a row holds h * 2^-E with E from the row's largest
    group maximum h, in fp16.  A group 2^26 below the row maximum is then a subnormal fp16 number and loses
    low bits of h; its terms are below 2^-24 of the row's largest terms, which is the resolution of the fp32
    accumulation, so the result still meets the accumulation bound against sum_k |xhat_k what_k|."""
    M, N, K, g = 48, 40, 256, 64
    rng = np.random.default_rng(915)
    scale_a = np.array([1.0, 2.0 ** -26, 2.0 ** -13, 2.0 ** -30])          # per group of X
    xb = synth.f64_to_bf16_bits(rng.standard_normal((M, K)) * np.repeat(scale_a, g)[None, :])
    wb = synth.f64_to_bf16_bits(rng.standard_normal((N, K)))
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    qa, qw = OQ.quantize(pq.FMT_INT4, g, x64), OQ.quantize(pq.FMT_INT4, g, w64)
    y_ref = OG.dequant_product(pq.FMT_INT4, g, qa, qw)
    a_codes, a_scales = pq.alloc_quantized(pq.FMT_INT4, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(pq.FMT_INT4, g, N, K, DEV)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_act(pq.FMT_INT4, g, _to_dev(xb), None, None, a_codes, a_scales)
    pq.pq_quantize_weights(pq.FMT_INT4, g, _to_dev(wb), None, w_codes, w_scales, one)
    np.testing.assert_array_equal(a_scales.cpu().numpy(), qa.scale)          # the stored scales are still exact
    y = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_f32(pq.FMT_INT4, g, a_codes, a_scales, None, w_codes, w_scales, None, y)
    torch.cuda.synchronize()
    mag = np.abs(OQ.dequantize(pq.FMT_INT4, g, qa)) @ np.abs(OQ.dequantize(pq.FMT_INT4, g, qw)).T
    err = np.abs(y.cpu().numpy().astype(np.float64) - y_ref)
    assert np.all(err <= T.GEMM_ACC_UNITS * 2.0 ** -24 * mag), float((err / mag).max())
    # and what is lost is really there: the far group's own contribution is not reproduced to its own precision
    far = slice(3 * g, 4 * g)
    part_ref = OQ.dequantize(pq.FMT_INT4, g, qa)[:, far] @ OQ.dequantize(pq.FMT_INT4, g, qw)[:, far].T
    assert np.abs(part_ref).max() < 2.0 ** -24 * mag.min()


def test_qgemm_check_int_scales():
    """Scales written by the quantizers are of the form the product kernel reproduces exactly; arbitrary fp32
    scales are counted."""
    M, K, g = 70, 512, 64
    rng = np.random.default_rng(916)
    xb = _rand_bits(rng, M, K)
    a_codes, a_scales = pq.alloc_quantized(pq.FMT_INT4, g, M, K, DEV)
    pq.pq_quantize_act(pq.FMT_INT4, g, _to_dev(xb), None, None, a_codes, a_scales)
    assert pq.pq_qgemm_check_int_scales(pq.FMT_INT4, g, a_scales, M, K) == 0
    bad = a_scales.clone()
    bad[3, 2] = 0.1234567            # not a bf16 value divided by 7
    bad[5, 0] = -bad[5, 0].abs() - 1.0
    bad[9, 7] = float("inf")
    assert pq.pq_qgemm_check_int_scales(pq.FMT_INT4, g, bad, M, K) == 3
    with pytest.raises(pq.PQError) as e:
        pq.pq_qgemm_check_int_scales(pq.FMT_NVFP4, 16, a_scales, M, K)
    assert e.value.code == -3


# ------------------------------------------------------------------- packed GEMM operands

@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("M,N,K", [(300, 264, 1056), (64, 520, 96), (513, 257, 2048)])
def test_qgemm_packed_equals_row_major(fmt, g, M, N, K):
    """The product from operands in the panel layout is the product from the stored layout, bit
    for bit (same kernel, same order of additions; only the addresses differ).  Shapes: ragged
    tiles in both directions, a K that ends in a half step (96 = 64 + 32), several tiles."""
    if K % g:
        pytest.skip("K is not a multiple of this group size")
    _say("packed gemm fmt=%d g=%d %dx%dx%d" % (fmt, g, M, N, K))
    rng = np.random.default_rng(7000 + M + K + g)
    xb = _rand_bits(rng, M, K)
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)) * np.exp(0.3 * rng.standard_normal(K)))
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    Ta = torch.ones(1, dtype=torch.float32, device=DEV)
    Tw = torch.ones(1, dtype=torch.float32, device=DEV)
    x = _to_dev(xb)
    if fmt == pq.FMT_NVFP4:
        amax = torch.zeros(1, dtype=torch.float32, device=DEV)
        pq.pq_calib_moments(x, torch.zeros(K, dtype=torch.float64, device=DEV), amax)
        pq.pq_tensor_scale(amax, Ta)
    pq.pq_quantize_act(fmt, g, x, None, Ta, a_codes, a_scales)
    pq.pq_quantize_weights(fmt, g, _to_dev(wb), None, w_codes, w_scales, Tw)
    a_op = pq.pq_pack_operand(fmt, g, a_codes, a_scales)
    w_op = pq.pq_pack_operand(fmt, g, w_codes, w_scales)
    ldy = (N + 7) // 8 * 8
    for dtype, plain, packed in ((torch.bfloat16, pq.pq_qgemm, pq.pq_qgemm_packed),
                                 (torch.float32, pq.pq_qgemm_f32, pq.pq_qgemm_packed_f32)):
        y0 = torch.full((M, ldy), 3.0, dtype=dtype, device=DEV)
        y1 = torch.full((M, ldy), 3.0, dtype=dtype, device=DEV)
        plain(fmt, g, a_codes, a_scales, Ta, w_codes, w_scales, Tw, y0, M=M, N=N, K=K, ldy=ldy)
        packed(fmt, g, a_op, Ta, w_op, Tw, y1, M, N, K, ldy=ldy)
        torch.cuda.synchronize()
        assert torch.equal(y0.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           y1.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


def test_pack_operand_then_gemm_matches_oracle():
    """End to end through the packed path against the fp64 product (the row-major path is checked
    against the oracle above; this pins the packed one directly)."""
    fmt, g, M, N, K = pq.FMT_INT4, 64, 200, 136, 1024
    rng = np.random.default_rng(4242)
    xb = _rand_bits(rng, M, K)
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)))
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    qa, qw = OQ.quantize(fmt, g, x64, None), OQ.quantize(fmt, g, w64, None)
    y_ref = OG.dequant_product(fmt, g, qa, qw)
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_act(fmt, g, _to_dev(xb), None, one, a_codes, a_scales)
    pq.pq_quantize_weights(fmt, g, _to_dev(wb), None, w_codes, w_scales, one)
    y32 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_packed_f32(fmt, g, pq.pq_pack_operand(fmt, g, a_codes, a_scales), one,
                           pq.pq_pack_operand(fmt, g, w_codes, w_scales), one, y32, M, N, K)
    torch.cuda.synchronize()
    T.gemm_f32_check(y32.cpu().numpy(), y_ref, T.abs_product(fmt, g, qa, qw), "packed int4 g64")


@pytest.mark.parametrize("M,K,pad", [(300, 1056, 0), (37, 96, 40), (1, 16, 0), (2100, 3072, 8)])
def test_dynamic_tensor_scale_two_pass(M, K, pad):
    """The two-pass NVFP4 activation path: T from the live tensor on the device, then the quantizer.
    T and the codes equal the oracle's for T = absmax / 2688; columns beyond K (here far larger than
    the data) are not read."""
    _say("dynamic tensor scale M=%d K=%d ld=%d" % (M, K, K + pad))
    rng = np.random.default_rng(7800 + M + K)
    bits = _rand_bits(rng, M, K + pad)
    if pad:
        bits[:, K:] = synth.f64_to_bf16_bits(np.full((M, pad), 3.0e4))
    x = _to_dev(bits)[:, :K]
    T_dev = torch.full((1,), 123.0, dtype=torch.float32, device=DEV)
    pq.pq_dynamic_tensor_scale(x, T_dev, K=K)
    codes, scales = pq.alloc_quantized(pq.FMT_NVFP4, 16, M, K, DEV)
    pq.pq_quantize_act(pq.FMT_NVFP4, 16, x, None, T_dev, codes, scales)
    torch.cuda.synchronize()
    x64 = OF.bf16_bits_to_f64(bits[:, :K])
    t_ref = OQ.nvfp4_tensor_scale(OC.absmax(x64))
    assert np.float32(T_dev.item()) == t_ref
    ref_codes, ref_scales, _ = T.oracle_quantize_bits(pq.FMT_NVFP4, 16, bits[:, :K], None, t_ref)
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    assert np.array_equal(scales.cpu().numpy(), ref_scales)
    # with the tensor's own absmax no block scale saturates: the largest E4M3 byte is 448's
    assert scales.max().item() == 0x7E


@pytest.mark.parametrize("fmt,g", [(pq.FMT_NVFP4, 16), (pq.FMT_INT4, 64), (pq.FMT_INT3, 32)])
@pytest.mark.parametrize("M,N,K", [(300, 264, 1088), (37, 520, 96)])
def test_qgemm_packed_bias(fmt, g, M, N, K):
    """y = Q(X) Q(W)^T + b: the bias is added in fp32 before the one rounding to bf16.  Against the
    fp64 product plus bias: half a bf16 step (at most 2^-8 relative) for the rounding, plus the accumulation
    bound of the product; and a zero bias reproduces the plain product except for the sign of zeros."""
    if K % g:
        pytest.skip("K is not a multiple of this group size")
    _say("packed gemm with bias fmt=%d g=%d %dx%dx%d" % (fmt, g, M, N, K))
    rng = np.random.default_rng(7700 + M + K + g)
    xb = _rand_bits(rng, M, K)
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)))
    bias_bits = synth.f64_to_bf16_bits(0.5 * rng.standard_normal(N))
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    ta = OQ.nvfp4_tensor_scale(OC.absmax(x64)) if fmt == pq.FMT_NVFP4 else None
    tw = OQ.nvfp4_tensor_scale(OC.absmax(w64)) if fmt == pq.FMT_NVFP4 else None
    qa, qw = OQ.quantize(fmt, g, x64, ta), OQ.quantize(fmt, g, w64, tw)
    bias64 = OF.bf16_bits_to_f64(bias_bits)
    y_ref = OG.add_bias(OG.dequant_product(fmt, g, qa, qw), bias64)
    Ta = torch.full((1,), float(ta) if ta is not None else 1.0, dtype=torch.float32, device=DEV)
    Tw = torch.ones(1, dtype=torch.float32, device=DEV)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    pq.pq_quantize_weights(fmt, g, _to_dev(wb), None, w_codes, w_scales, Tw)
    a_op = pq.pq_quantize_act_packed(fmt, g, _to_dev(xb), Ta)
    w_op = pq.pq_pack_operand(fmt, g, w_codes, w_scales)
    ldy = (N + 7) // 8 * 8
    y = torch.full((M, ldy), 3.0, dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_packed_bias(fmt, g, a_op, Ta, w_op, Tw, _to_dev(bias_bits), y, M, N, K, ldy=ldy)
    y0 = torch.full((M, ldy), 3.0, dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_packed_bias(fmt, g, a_op, Ta, w_op, Tw, torch.zeros(N, dtype=torch.bfloat16, device=DEV), y0, M, N, K, ldy=ldy)
    y_plain = torch.full((M, ldy), 3.0, dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_packed(fmt, g, a_op, Ta, w_op, Tw, y_plain, M, N, K, ldy=ldy)
    torch.cuda.synchronize()
    got = y[:, :N].float().cpu().numpy().astype(np.float64)
    mag = T.abs_product(fmt, g, qa, qw) + np.abs(bias64)[None, :]
    tol = 2.0 ** -8 * np.abs(y_ref) + T.GEMM_ACC_UNITS * 2.0 ** -24 * mag
    err = np.abs(got - y_ref)
    assert np.all(err <= tol), "worst %g of tolerance" % float((err / tol).max())
    assert torch.all(y[:, N:] == 3.0)
    assert torch.equal(y0.float(), y_plain.float())          # -0 + 0 = +0: compare values, not bits


@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("M,K,pad", [(300, 1056, 0), (7, 96, 0), (64, 2048, 16), (1, 256, 0), (515, 3072, 0)])
def test_quantize_act_packed_equals_quantize_then_pack(fmt, g, M, K, pad):
    """The fused quantizer leaves exactly the bytes that pq_quantize_act followed by pq_pack_operand
    leaves (buffers cleared first: the layout has alignment gaps), and its optional row-major
    copies are pq_quantize_act's outputs.  Shapes: ragged row blocks, a K ending in a half step,
    a row stride, a single row, the FLUX width."""
    if K % g:
        pytest.skip("K is not a multiple of this group size")
    _say("quantize_act_packed fmt=%d g=%d M=%d K=%d ld=%d" % (fmt, g, M, K, K + pad))
    rng = np.random.default_rng(8100 + M + K + g)
    bits = _rand_bits(rng, M, K + pad)
    x = _to_dev(bits)[:, :K]
    Ta = torch.ones(1, dtype=torch.float32, device=DEV)
    if fmt == pq.FMT_NVFP4:
        Ta.fill_(float(OQ.nvfp4_tensor_scale(OC.absmax(OF.bf16_bits_to_f64(bits[:, :K])))))
    codes, scales = pq.alloc_quantized(fmt, g, M, K, DEV)
    pq.pq_quantize_act(fmt, g, x, None, Ta, codes, scales)
    nbytes = max(pq.pq_operand_bytes(fmt, g, M, K), 16)
    ref_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_pack_operand(fmt, g, codes, scales, ref_op)
    got_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    codes2, scales2 = pq.alloc_quantized(fmt, g, M, K, DEV)
    codes2.fill_(0xEE)
    pq.pq_quantize_act_packed(fmt, g, x, Ta, got_op, codes2, scales2, K=K)
    torch.cuda.synchronize()
    assert torch.equal(got_op, ref_op)
    assert torch.equal(codes2, codes)
    assert torch.equal(scales2.view(torch.uint8), scales.view(torch.uint8))
    # and without the row-major copies
    got2 = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, x, Ta, got2, K=K)
    torch.cuda.synchronize()
    assert torch.equal(got2, ref_op)
