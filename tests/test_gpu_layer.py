"""The pieces composed into one layer, through the C ABI, against the oracle's chain in fp64:
    y = Q(P AdaLN(x)) Q(P^T W)^T + b                       (paper App. C + Eq. 8)
    y = Q(x H P) Q((W H) P)^T                              (paper App. D + Eq. 8)
The quantizer sees bf16 values that can differ from the oracle's by one rounding step on a few
outputs of the normalisation / rotation (see test_gpu_norm.py), so the products are compared with
the tolerance of the product kernel plus the effect of those steps; the Hadamard case also checks the
qualitative claim that rotation plus reorder lowers the layer's output error on outlier-heavy
activations."""
import sys

import numpy as np
import pytest
import torch

from oracle import calib as OC
from oracle import formats as OF
from oracle import gemm as OG
from oracle import hadamard as OH
from oracle import norm as ON
from oracle import quantize as OQ
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


def _host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _weights_operand(fmt, g, w_bits, perm_d):
    N, K = w_bits.shape
    codes, scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    tw = torch.ones(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_weights(fmt, g, _dev(w_bits), perm_d, codes, scales, tw)
    return pq.pq_pack_operand(fmt, g, codes, scales), tw


@pytest.mark.parametrize("fmt,g", [(pq.FMT_INT4, 64), (pq.FMT_NVFP4, 16)])
def test_adaln_quantize_gemm_bias_layer(fmt, g):
    M, N, K, per = 96, 72, 768, 40
    _say("layer adaln fmt=%d g=%d" % (fmt, g))
    rng = np.random.default_rng(9990 + fmt)
    chan = np.exp(0.4 * rng.standard_normal(K))
    chan[rng.choice(K, 8, replace=False)] *= 20.0
    x_bits = _bits(rng.standard_normal((M, K)) * chan + 0.2)
    w_bits = _bits(0.03 * rng.standard_normal((N, K)))
    n_mod = -(-M // per)
    s_bits = _bits(0.3 * rng.standard_normal((n_mod, K)))
    b_bits = _bits(0.3 * rng.standard_normal((n_mod, K)))
    bias_bits = _bits(0.5 * rng.standard_normal(N))
    perm = rng.permutation(K).astype(np.int32)
    perm_d = torch.from_numpy(perm).to(DEV)

    # oracle chain
    y_norm = ON.adaln_reordered(OF.bf16_bits_to_f64(x_bits), OF.bf16_bits_to_f64(s_bits), OF.bf16_bits_to_f64(b_bits),
                                per, 1e-6, perm)
    a64 = OF.bf16_bits_to_f64(ON.to_bf16_bits(y_norm))
    w64 = OF.bf16_bits_to_f64(w_bits)[:, perm]
    ta = OQ.nvfp4_tensor_scale(OC.absmax(a64)) if fmt == pq.FMT_NVFP4 else None
    tw = OQ.nvfp4_tensor_scale(OC.absmax(w64)) if fmt == pq.FMT_NVFP4 else None
    qa, qw = OQ.quantize(fmt, g, a64, ta), OQ.quantize(fmt, g, w64, tw)
    y_ref = OG.add_bias(OG.dequant_product(fmt, g, qa, qw), OF.bf16_bits_to_f64(bias_bits))

    # library chain
    Ta = torch.full((1,), float(ta) if ta is not None else 1.0, dtype=torch.float32, device=DEV)
    a_op = pq.pq_norm_quantize_act_packed(pq.NORM_ADALN, fmt, g, _dev(x_bits), 1e-6, Ta, perm_d, None, _dev(s_bits),
                                          _dev(b_bits), per)
    w_op, Tw = _weights_operand(fmt, g, w_bits, perm_d)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    pq.pq_qgemm_packed_bias(fmt, g, a_op, Ta, w_op, Tw, _dev(bias_bits), y, M, N, K)
    torch.cuda.synchronize()
    got = OF.bf16_bits_to_f64(_host_bits(y))
    # one bf16 step on an activation moves it by at most 2^-8 |a|; it reaches the output through at most
    # one quantization step of its group: bound the whole effect by a small multiple of the layer's scale
    scale = np.sqrt(np.mean(y_ref ** 2))
    assert np.abs(got - y_ref).max() <= 0.02 * scale + 2.0 ** -8 * np.abs(y_ref).max()
    assert np.mean(np.abs(got - y_ref) <= 2.0 ** -8 * np.abs(y_ref) + 1e-3 * scale) > 0.99


def test_hadamard_then_reorder_layer_lowers_the_output_error():
    M, N, K, fmt, g = 128, 96, 1024, pq.FMT_INT4, 64
    rng = np.random.default_rng(9995)
    chan = np.exp(0.3 * rng.standard_normal(K))
    chan[rng.choice(K, 6, replace=False)] *= 40.0            # massive outlier channels
    x_bits = _bits(rng.standard_normal((M, K)) * chan)
    w_bits = _bits(0.03 * rng.standard_normal((N, K)))
    x64, w64 = OF.bf16_bits_to_f64(x_bits), OF.bf16_bits_to_f64(w_bits)
    y_true = x64 @ w64.T
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)

    def rel_err(yq):
        return float(np.sum((OF.bf16_bits_to_f64(_host_bits(yq)) - y_true) ** 2) / np.sum(y_true ** 2))

    # plain W4A4
    w_op, _ = _weights_operand(fmt, g, w_bits, None)
    pq.pq_qgemm_packed(fmt, g, pq.pq_quantize_act_packed(fmt, g, _dev(x_bits), one), one, w_op, one, y, M, N, K)
    torch.cuda.synchronize()
    e_plain = rel_err(y)

    # PermuQuant-H: rotate both sides, select the order on the rotated tensors, quantize, multiply
    xr = pq.pq_hadamard_reorder(_dev(x_bits))
    wr = pq.pq_hadamard_reorder(_dev(w_bits))
    sa = torch.zeros(K, dtype=torch.float64, device=DEV)
    sw = torch.zeros(K, dtype=torch.float64, device=DEV)
    pq.pq_calib_moments(xr, sa)
    pq.pq_calib_moments(wr, sw)
    perm_d = torch.empty(K, dtype=torch.int32, device=DEV)
    rep = pq.pq_select_perm(fmt, g, sa, sw, [xr], wr, 1.0, 1.0, perm_d)
    a_op = pq.pq_hadamard_quantize_act_packed(fmt, g, _dev(x_bits), one, perm_d)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, DEV)
    pq.pq_quantize_weights(fmt, g, wr, perm_d, w_codes, w_scales, torch.ones(1, dtype=torch.float32, device=DEV))
    pq.pq_qgemm_packed(fmt, g, a_op, one, pq.pq_pack_operand(fmt, g, w_codes, w_scales), one, y, M, N, K)
    torch.cuda.synchronize()
    e_h = rel_err(y)
    _say("output error: plain %.4g, Hadamard + reorder %.4g (accepted=%s)" % (e_plain, e_h, rep.accepted))
    assert e_h < 0.75 * e_plain

    # and the oracle's chain gives the same product up to the tolerance of the pieces
    perm = perm_d.cpu().numpy()
    a64 = OF.bf16_bits_to_f64(OH.to_bf16_bits(OH.rotate_reordered(x64, perm)))
    wr64 = OF.bf16_bits_to_f64(OH.to_bf16_bits(OH.rotate(w64)))[:, perm]
    y_ref = OG.dequant_product(fmt, g, OQ.quantize(fmt, g, a64), OQ.quantize(fmt, g, wr64))
    got = OF.bf16_bits_to_f64(_host_bits(y))
    scale = np.sqrt(np.mean(y_ref ** 2))
    assert np.abs(got - y_ref).max() <= 0.03 * scale + 2.0 ** -8 * np.abs(y_ref).max()


def test_forward_path_replays_from_a_captured_graph():
    """The forward entry points allocate nothing and never synchronise, so a caller can capture them in a
    graph: three replays on refreshed inputs, with eager work and synchronisations in between, each equal
    to the eager result bit for bit."""
    M, N, K, fmt, g = 200, 136, 1024, pq.FMT_INT4, 64
    rng = np.random.default_rng(9996)
    perm_d = torch.from_numpy(rng.permutation(K).astype(np.int32)).to(DEV)
    gamma = _dev(_bits(1.0 + 0.2 * rng.standard_normal(K)))
    bias = _dev(_bits(0.5 * rng.standard_normal(N)))
    w_op, Tw = _weights_operand(fmt, g, _bits(0.03 * rng.standard_normal((N, K))), perm_d)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    x = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    a_op = torch.zeros(pq.pq_operand_bytes(fmt, g, M, K), dtype=torch.uint8, device=DEV)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)

    def forward(out):
        pq.pq_norm_quantize_act_packed(pq.NORM_RMS, fmt, g, x, 1e-6, one, perm_d, gamma, operand=a_op)
        pq.pq_qgemm_packed_bias(fmt, g, a_op, one, w_op, Tw, bias, out, M, N, K)

    x.copy_(_dev(_bits(rng.standard_normal((M, K)))))
    forward(y)                                   # warm-up outside the capture (first-use set-up of the kernels)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        forward(y)
    for i in range(3):
        x.copy_(_dev(_bits(rng.standard_normal((M, K)) * (1.0 + i))))
        y_eager = torch.empty_like(y)
        forward(y_eager)
        torch.cuda.synchronize()
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y_eager.view(torch.int16)), "replay %d differs" % i


@pytest.mark.parametrize("fmt,g,M,N,K", [(pq.FMT_NVFP4, 16, 300, 264, 1088), (pq.FMT_INT4, 64, 520, 200, 1024),
                                          (pq.FMT_NVFP4, 16, 4608, 512, 12288)])
def test_forward_path_in_a_hip_graph(fmt, g, M, N, K):
    """The deployment path (activations quantized straight into the GEMM's operand layout, then the product)
    captured into a HIP graph: every replay, with eager work and synchronisations in between, gives the
    bits of the eager run.  Nothing in the two calls allocates, synchronises or clears memory, so they can be
    captured as they are.  (The third shape takes the large-tensor quantizer and the 224 x 256 product tile.)"""
    _say("forward path in a graph fmt=%d g=%d %dx%dx%d" % (fmt, g, M, N, K))
    rng = np.random.default_rng(9970 + g + M)
    x = _dev(_bits(rng.standard_normal((M, K)) * np.exp(0.5 * rng.standard_normal(K))))
    w_op, tw = _weights_operand(fmt, g, _bits(0.02 * rng.standard_normal((N, K))), None)
    ta = torch.full((1,), 0.002, dtype=torch.float32, device=DEV)
    a_op = torch.zeros(pq.pq_operand_bytes(fmt, g, M, K), dtype=torch.uint8, device=DEV)   # alignment gaps stay zero
    y_eager = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, x, ta, a_op)
    pq.pq_qgemm_packed(fmt, g, a_op, ta, w_op, tw, y_eager, M, N, K)
    torch.cuda.synchronize()
    a_eager = a_op.clone()
    y = torch.empty_like(y_eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pq.pq_quantize_act_packed(fmt, g, x, ta, a_op)
        pq.pq_qgemm_packed(fmt, g, a_op, ta, w_op, tw, y, M, N, K)
    for replay in range(3):
        a_op.zero_()
        y.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(a_op, a_eager), "operand of replay %d differs" % replay
        assert torch.equal(y.view(torch.int16), y_eager.view(torch.int16)), "output of replay %d differs" % replay
        # eager use of the same buffers between the replays
        pq.pq_quantize_act_packed(fmt, g, x, ta, a_op)
        torch.cuda.synchronize()
