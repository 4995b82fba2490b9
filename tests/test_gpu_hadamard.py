"""GPU parity of the Hadamard rotation with the reorder absorbed into its output order (paper
App. D, x H P), through the C ABI, against the CPU oracle (dense fp64 matrix product).

Bar as for the normalisation layer: the kernel's fast transform adds in fp32 (at most log2(K) + 20
additions per output), the oracle in fp64, so every output lies within one bf16 step (2^-8 relative)
plus 2^-18 of the row's largest magnitude of the oracle's and at least 99.5 % of the outputs are
bit-identical; with integer inputs of a small range every fp32 sum is exact and the scaling by
1 / sqrt(K) a power of two when K is a power of four: then all bits agree, and so does the
quantized operand."""
import sys

import numpy as np
import pytest
import torch

from oracle import formats as OF
from oracle import hadamard as OH
from paper_2605_09503_amd import pq, synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
FMTS = [(pq.FMT_NVFP4, 16), (pq.FMT_INT4, 64), (pq.FMT_INT4, 32), (pq.FMT_INT3, 32), (pq.FMT_INT4, 128),
        (pq.FMT_INT3, 256)]


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _bits(v):
    return synth.f64_to_bf16_bits(np.asarray(v, dtype=np.float64))


def _dev(bits):
    return pq.bf16_from_bits(bits, DEV)


def _host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _activations(rng, rows, K):
    chan = np.exp(rng.standard_normal(K))
    chan[rng.choice(K, max(1, K // 64), replace=False)] *= 25.0
    return _bits(rng.standard_normal((rows, K)) * chan[None, :])


def _check_close(got_bits, ref64, label, min_same=0.995):
    got = OF.bf16_bits_to_f64(got_bits)
    ref_bits = OH.to_bf16_bits(ref64)
    row_max = np.abs(ref64).max(axis=1, keepdims=True)
    tol = 2.0 ** -8 * np.abs(ref64) + 2.0 ** -18 * row_max
    err = np.abs(got - ref64)
    bad = err > tol
    assert not bad.any(), "%s: %d outputs off, worst %g at %s" % (
        label, int(bad.sum()), float((err / np.maximum(tol, 1e-300)).max()), np.argwhere(bad)[:4].tolist())
    same = float((got_bits == ref_bits).mean())
    assert same >= min_same, "%s: only %.4f of the outputs bit-identical" % (label, same)


# widths: powers of two with every last-pass radix (2, 4, 8, 16), the Paley factors 12 and 20 alone and
# combined with Sylvester digits (12 * 2^k from 192 on takes the Paley pass on the matrix unit, below that
# on the vector unit), the FLUX widths
WIDTHS = [8, 16, 32, 64, 128, 512, 4096, 24, 48, 96, 192, 768, 3072, 40, 160, 2560,
          8192, 12288, 5120, 24576]          # wider than 4096: four waves share a row


@pytest.mark.parametrize("K", WIDTHS)
@pytest.mark.parametrize("with_perm", [True, False])
def test_hadamard_reorder_matches_oracle(K, with_perm):
    rows = 19 if K <= 768 else 9
    _say("hadamard_reorder K=%d perm=%s rows=%d" % (K, with_perm, rows))
    rng = np.random.default_rng(9900 + K)
    pad = 8 if K % 16 else 0
    x_bits = _activations(rng, rows, K + pad)
    perm = rng.permutation(K).astype(np.int32) if with_perm else None
    x = _dev(x_bits)[:, :K]
    y = torch.full((rows, K + 8), 7.0, dtype=torch.bfloat16, device=DEV)
    pq.pq_hadamard_reorder(x, None if perm is None else torch.from_numpy(perm).to(DEV), y=y, K=K)
    torch.cuda.synchronize()
    ref = OH.rotate_reordered(OF.bf16_bits_to_f64(x_bits[:, :K]), perm)
    _check_close(_host_bits(y[:, :K]), ref, "hadamard_reorder K=%d" % K)
    assert torch.all(y[:, K:] == 7.0)


def test_unit_vectors_give_the_rows_of_the_matrix():
    """Row i of the identity is mapped to row i of H: every entry +-1/sqrt(K) with the oracle's sign
    (pins the index conventions of the fast transform: digit order, Paley orientation)."""
    for K in (48, 160, 192, 256, 768):
        x_bits = _bits(np.eye(K) * 4.0)
        y = pq.pq_hadamard_reorder(_dev(x_bits))
        torch.cuda.synchronize()
        got = OF.bf16_bits_to_f64(_host_bits(y))
        ref = OF.bf16_bits_to_f64(OH.to_bf16_bits(4.0 * OH.hadamard_matrix(K)))
        assert np.array_equal(got, ref), K


def test_wide_exact_inputs_and_fused_quantizer():
    """K = 16384 = 4^7 with integer inputs: exact arithmetic, four waves per row; and the quantizing call
    equals rotation followed by quantizer."""
    rows, K = 5, 16384
    rng = np.random.default_rng(9955)
    x_bits = _bits(rng.integers(-8, 9, size=(rows, K)).astype(np.float64))
    perm = rng.permutation(K).astype(np.int32)
    perm_d = torch.from_numpy(perm).to(DEV)
    ref_bits = OH.to_bf16_bits(OH.rotate_reordered(OF.bf16_bits_to_f64(x_bits), perm))
    y = pq.pq_hadamard_reorder(_dev(x_bits), perm_d)
    torch.cuda.synchronize()
    assert np.array_equal(_host_bits(y), ref_bits)
    for fmt, g in ((pq.FMT_INT4, 64), (pq.FMT_NVFP4, 16), (pq.FMT_INT3, 256)):
        Ta = torch.full((1,), 0.01, dtype=torch.float32, device=DEV)
        want = pq.pq_quantize_act_packed(fmt, g, y, Ta, torch.zeros(pq.pq_operand_bytes(fmt, g, rows, K), dtype=torch.uint8, device=DEV))
        got = pq.pq_hadamard_quantize_act_packed(fmt, g, _dev(x_bits), Ta, perm_d, operand=torch.zeros_like(want))
        torch.cuda.synchronize()
        assert torch.equal(got, want), (fmt, g)


@pytest.mark.parametrize("fmt,g", FMTS)
def test_exact_inputs_bit_identical_to_oracle_chain(fmt, g):
    """Integer inputs in [-8, 8] and K = 1024 = 4^5: all fp32 sums are exact integers below 2^24 and the
    scale 1/32 is a power of two, so the bf16 output equals the oracle's bit for bit and the quantized
    operand equals the quantizer's output on the oracle's bits."""
    rows, K = 37, 1024
    _say("hadamard exact fmt=%d g=%d" % (fmt, g))
    rng = np.random.default_rng(9950 + fmt * 10 + g)
    x_bits = _bits(rng.integers(-8, 9, size=(rows, K)).astype(np.float64))
    perm = rng.permutation(K).astype(np.int32)
    perm_d = torch.from_numpy(perm).to(DEV)
    ref_bits = OH.to_bf16_bits(OH.rotate_reordered(OF.bf16_bits_to_f64(x_bits), perm))
    Ta = torch.full((1,), 0.01, dtype=torch.float32, device=DEV)
    nbytes = max(pq.pq_operand_bytes(fmt, g, rows, K), 16)
    got_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    y = torch.empty((rows, K), dtype=torch.bfloat16, device=DEV)
    pq.pq_hadamard_quantize_act_packed(fmt, g, _dev(x_bits), Ta, perm_d, operand=got_op, y=y)
    want_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, _dev(ref_bits), Ta, want_op)
    torch.cuda.synchronize()
    assert np.array_equal(_host_bits(y), ref_bits)
    assert torch.equal(got_op, want_op)


@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("rows,K,pad", [(37, 256, 0), (20, 3072, 0), (9, 1280, 16)])
def test_fused_quantizer_equals_rotate_then_quantize(fmt, g, rows, K, pad):
    if K % g:
        pytest.skip("K is not a multiple of this group size")
    _say("hadamard fused fmt=%d g=%d rows=%d K=%d" % (fmt, g, rows, K))
    rng = np.random.default_rng(9960 + fmt * 10 + g + rows)
    x = _dev(_activations(rng, rows, K + pad))[:, :K]
    perm_d = torch.from_numpy(rng.permutation(K).astype(np.int32)).to(DEV)
    Ta = torch.full((1,), 0.05, dtype=torch.float32, device=DEV)
    y_ref = pq.pq_hadamard_reorder(x, perm_d, K=K)
    nbytes = max(pq.pq_operand_bytes(fmt, g, rows, K), 16)
    want = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, y_ref, Ta, want)
    got = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    y = torch.empty((rows, K), dtype=torch.bfloat16, device=DEV)
    pq.pq_hadamard_quantize_act_packed(fmt, g, x, Ta, perm_d, operand=got, y=y, K=K)
    got2 = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_hadamard_quantize_act_packed(fmt, g, x, Ta, perm_d, operand=got2, K=K)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    assert torch.equal(got, want) and torch.equal(got2, want)


def test_rotated_layer_keeps_the_product():
    """(x H)(W H)^T = x W^T: activations and weights rotated by the library, multiplied in fp64 on the
    host from the bf16 results; the difference to the plain product is the bf16 rounding of the two
    rotated tensors (2^-9 relative each, random signs over K terms)."""
    M, N, K = 24, 16, 3072
    rng = np.random.default_rng(9970)
    x_bits = _bits(rng.standard_normal((M, K)))
    w_bits = _bits(0.05 * rng.standard_normal((N, K)))
    perm_d = torch.from_numpy(rng.permutation(K).astype(np.int32)).to(DEV)
    xr = OF.bf16_bits_to_f64(_host_bits(pq.pq_hadamard_reorder(_dev(x_bits), perm_d)))
    wr = OF.bf16_bits_to_f64(_host_bits(pq.pq_hadamard_reorder(_dev(w_bits), perm_d)))
    torch.cuda.synchronize()
    x64, w64 = OF.bf16_bits_to_f64(x_bits), OF.bf16_bits_to_f64(w_bits)
    y, y_rot = x64 @ w64.T, xr @ wr.T
    scale = np.sqrt(np.sum(x64 ** 2, axis=1))[:, None] * np.sqrt(np.sum(w64 ** 2, axis=1))[None, :]
    assert np.abs(y_rot - y).max() <= 2.0 ** -7 * scale.max() / np.sqrt(K) * 8


def test_full_size_sampled_rows():
    rows, K = 4608, 3072
    rng = np.random.default_rng(9980)
    x_bits = _activations(rng, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    sample = np.unique(np.concatenate([[0, 5, 6, rows - 1], rng.integers(0, rows, 44)]))
    y = pq.pq_hadamard_reorder(_dev(x_bits), torch.from_numpy(perm).to(DEV))
    torch.cuda.synchronize()
    ref = OH.rotate_reordered(OF.bf16_bits_to_f64(x_bits[sample]), perm)
    _check_close(_host_bits(y)[sample], ref, "full size")
    assert torch.isfinite(y.float()).all()


def test_unsupported_widths_are_refused():
    for K in (1152, 3840, 56):
        x = torch.zeros((8, K), dtype=torch.bfloat16, device=DEV)
        with pytest.raises(pq.PQError) as e:
            pq.pq_hadamard_reorder(x)
        assert e.value.code == -2
