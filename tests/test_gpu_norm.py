"""GPU parity of the normalisation layer with the absorbed channel reorder (paper App. C),
through the C ABI, against the CPU oracle on the same seeded bits.

Bar: the kernel computes statistics and the affine part in fp32 and rounds once to bf16; the
oracle works in fp64.  An fp32 result sits within a few 2^-24 (relative to the row's largest
output) of the fp64 one, which now and then falls on the other side of a bf16 rounding
boundary.  So: every output within one bf16 step of the oracle's (2^-8 relative) plus 2^-18 of
the row's largest magnitude (outputs near zero come from a cancellation), and at least 99.5 % of
the outputs bit-identical.  Where the arithmetic is exact in both precisions the bits must agree
everywhere, and so must the quantized operand built from them."""
import sys

import numpy as np
import pytest
import torch

from oracle import formats as OF
from oracle import norm as ON
from paper_2605_09503_amd import pq, synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
RMS, ADALN = pq.NORM_RMS, pq.NORM_ADALN
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
    """Token rows with channels of very different size, a few outlier channels and a per-row offset."""
    chan = np.exp(rng.standard_normal(K))
    chan[rng.choice(K, max(1, K // 64), replace=False)] *= 25.0
    return _bits(rng.standard_normal((rows, K)) * chan[None, :] + 0.5 * rng.standard_normal((rows, 1)))


def _oracle(kind, x_bits, perm, gamma_bits, s_bits, b_bits, rows_per_mod, eps):
    x = OF.bf16_bits_to_f64(x_bits)
    K = x.shape[1]
    if kind == RMS:
        gamma = np.ones(K) if gamma_bits is None else OF.bf16_bits_to_f64(gamma_bits)
        return ON.rmsnorm_reordered(x, gamma, eps, perm)
    n_mod = 1 if rows_per_mod <= 0 else -(-x.shape[0] // rows_per_mod)
    s = np.zeros((n_mod, K)) if s_bits is None else OF.bf16_bits_to_f64(s_bits)
    b = np.zeros((n_mod, K)) if b_bits is None else OF.bf16_bits_to_f64(b_bits)
    return ON.adaln_reordered(x, s, b, rows_per_mod if rows_per_mod > 0 else x.shape[0], eps, perm)


def _check_close(got_bits, ref64, label, min_same=0.995):
    got = OF.bf16_bits_to_f64(got_bits)
    ref_bits = ON.to_bf16_bits(ref64)
    row_max = np.abs(ref64).max(axis=1, keepdims=True)
    tol = 2.0 ** -8 * np.abs(ref64) + 2.0 ** -18 * row_max
    err = np.abs(got - ref64)
    bad = err > tol
    assert not bad.any(), "%s: %d outputs off, worst %g at %s" % (
        label, int(bad.sum()), float((err / np.maximum(tol, 1e-300)).max()), np.argwhere(bad)[:4].tolist())
    same = float((got_bits == ref_bits).mean())
    assert same >= min_same, "%s: only %.4f of the outputs bit-identical" % (label, same)
    return same


CASES = [  # rows, K, ld pad, rows_per_mod
    (37, 256, 0, 12),          # ragged last workgroup, sample boundaries inside workgroups
    (64, 3072, 0, 32),         # the FLUX width
    (19, 200, 8, 5),           # K not a multiple of 64, padded rows
    (1, 8, 0, 0),              # smallest
    (130, 1032, 24, 0),        # one modulation row for all tokens
]


@pytest.mark.parametrize("rows,K,pad,rows_per_mod", CASES)
@pytest.mark.parametrize("with_perm", [True, False])
@pytest.mark.parametrize("kind", [RMS, ADALN])
def test_norm_reorder_matches_oracle(kind, with_perm, rows, K, pad, rows_per_mod):
    _say("norm_reorder kind=%d perm=%s rows=%d K=%d ld=%d rpm=%d" % (kind, with_perm, rows, K, K + pad, rows_per_mod))
    rng = np.random.default_rng(9000 + 7 * rows + K + kind)
    x_bits = _activations(rng, rows, K + pad)
    perm = rng.permutation(K).astype(np.int32) if with_perm else None
    n_mod = 1 if rows_per_mod <= 0 else -(-rows // rows_per_mod)
    gamma_bits = _bits(1.0 + 0.3 * rng.standard_normal(K))
    s_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    b_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    eps = 1e-6
    x = _dev(x_bits)[:, :K]
    perm_d = None if perm is None else torch.from_numpy(perm).to(DEV)
    y = torch.full((rows, K + 8), 7.0, dtype=torch.bfloat16, device=DEV)      # ldy > K: the margin must survive
    pq.pq_norm_reorder(kind, x, eps, perm_d, _dev(gamma_bits), _dev(s_bits), _dev(b_bits), rows_per_mod, y=y, K=K)
    torch.cuda.synchronize()
    ref = _oracle(kind, x_bits[:, :K], perm, gamma_bits, s_bits, b_bits, rows_per_mod, eps)
    _check_close(_host_bits(y[:, :K]), ref, "norm_reorder")
    assert torch.all(y[:, K:] == 7.0)


@pytest.mark.parametrize("kind", [RMS, ADALN])
def test_norm_reorder_default_vectors(kind):
    """NULL gamma means ones; NULL scale / shift mean zeros (plain LayerNorm)."""
    rows, K = 24, 512
    rng = np.random.default_rng(9100 + kind)
    x_bits = _activations(rng, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    y = pq.pq_norm_reorder(kind, _dev(x_bits), 1e-5, torch.from_numpy(perm).to(DEV))
    torch.cuda.synchronize()
    ref = _oracle(kind, x_bits, perm, None, None, None, 0, 1e-5)
    _check_close(_host_bits(y), ref, "default vectors")


def _exact_case(rng, kind, rows, K):
    """Inputs for which fp32 and fp64 give the same normalised values: every |x| of a row is the same
    power of two c (half of each sign for LayerNorm), so the statistic is c^2 and 1 / sqrt is exact
    with eps = 0; vectors on a coarse binary grid."""
    c = 2.0 ** rng.integers(-3, 4, size=(rows, 1))
    sign = np.ones((rows, K))
    sign[:, : K // 2] = -1.0
    for m in range(rows):
        rng.shuffle(sign[m])
    x_bits = _bits(sign * c)
    grid = lambda shape: rng.integers(-128, 129, size=shape) / 64.0
    return x_bits, _bits(grid(K)), _bits(grid((-(-rows // 16), K))), _bits(grid((-(-rows // 16), K)))


@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("kind", [RMS, ADALN])
def test_exact_inputs_bit_identical_to_oracle_chain(kind, fmt, g):
    """With exact arithmetic the reordered bf16 output equals the oracle's bit for bit, and the
    quantized operand equals the quantizer's output on the oracle's bits."""
    rows, K = 45, 768
    _say("norm exact kind=%d fmt=%d g=%d" % (kind, fmt, g))
    rng = np.random.default_rng(9200 + kind * 100 + fmt * 10 + g)
    x_bits, gamma_bits, s_bits, b_bits = _exact_case(rng, kind, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    perm_d = torch.from_numpy(perm).to(DEV)
    ref = _oracle(kind, x_bits, perm, gamma_bits, s_bits, b_bits, 16, 0.0)
    ref_bits = ON.to_bf16_bits(ref)
    Ta = torch.full((1,), 0.004, dtype=torch.float32, device=DEV)
    nbytes = max(pq.pq_operand_bytes(fmt, g, rows, K), 16)
    got_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    y = torch.empty((rows, K), dtype=torch.bfloat16, device=DEV)
    pq.pq_norm_quantize_act_packed(kind, fmt, g, _dev(x_bits), 0.0, Ta, perm_d, _dev(gamma_bits), _dev(s_bits),
                                   _dev(b_bits), 16, operand=got_op, y=y)
    want_op = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, _dev(ref_bits), Ta, want_op)
    torch.cuda.synchronize()
    assert np.array_equal(_host_bits(y), ref_bits)
    assert torch.equal(got_op, want_op)


@pytest.mark.parametrize("fmt,g", FMTS)
@pytest.mark.parametrize("kind", [RMS, ADALN])
@pytest.mark.parametrize("rows,K,pad", [(37, 256, 0), (64, 3072, 0), (9, 1056, 16)])
def test_fused_quantizer_equals_norm_then_quantize(kind, fmt, g, rows, K, pad):
    """pq_norm_quantize_act_packed leaves the bytes of pq_quantize_act_packed(pq_norm_reorder(x)),
    with or without the optional bf16 output."""
    if K % g:
        pytest.skip("K is not a multiple of this group size")
    _say("norm fused kind=%d fmt=%d g=%d rows=%d K=%d" % (kind, fmt, g, rows, K))
    rng = np.random.default_rng(9300 + kind + fmt * 10 + g + rows)
    x_bits = _activations(rng, rows, K + pad)
    perm_d = torch.from_numpy(rng.permutation(K).astype(np.int32)).to(DEV)
    n_mod = -(-rows // 12)
    gamma = _dev(_bits(1.0 + 0.3 * rng.standard_normal(K)))
    s = _dev(_bits(0.5 * rng.standard_normal((n_mod, K))))
    b = _dev(_bits(0.5 * rng.standard_normal((n_mod, K))))
    x = _dev(x_bits)[:, :K]
    Ta = torch.full((1,), 0.004, dtype=torch.float32, device=DEV)
    y_ref = pq.pq_norm_reorder(kind, x, 1e-6, perm_d, gamma, s, b, 12, K=K)
    nbytes = max(pq.pq_operand_bytes(fmt, g, rows, K), 16)
    want = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_quantize_act_packed(fmt, g, y_ref, Ta, want)
    got = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    y = torch.empty((rows, K), dtype=torch.bfloat16, device=DEV)
    pq.pq_norm_quantize_act_packed(kind, fmt, g, x, 1e-6, Ta, perm_d, gamma, s, b, 12, operand=got, y=y, K=K)
    got2 = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    pq.pq_norm_quantize_act_packed(kind, fmt, g, x, 1e-6, Ta, perm_d, gamma, s, b, 12, operand=got2, K=K)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    assert torch.equal(got, want)
    assert torch.equal(got2, want)


def test_equivariance_on_the_device():
    """App. C: the fused kernel on (x, gamma, pi) equals the plain kernel on the gathered inputs
    (x P, gamma P, identity) bit for bit -- the statistics are those of the same numbers in another
    order only if the reduction order is kept, so this is checked for the element-wise part only:
    rows whose statistic is exact."""
    rows, K = 16, 1024
    rng = np.random.default_rng(9400)
    x_bits, gamma_bits, s_bits, b_bits = _exact_case(rng, ADALN, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    for kind in (RMS, ADALN):
        fused = pq.pq_norm_reorder(kind, _dev(x_bits), 0.0, torch.from_numpy(perm).to(DEV), _dev(gamma_bits),
                                   _dev(s_bits), _dev(b_bits), 16)
        plain = pq.pq_norm_reorder(kind, _dev(x_bits[:, perm]), 0.0, None, _dev(gamma_bits[perm]),
                                   _dev(s_bits[:, perm]), _dev(b_bits[:, perm]), 16)
        torch.cuda.synchronize()
        assert torch.equal(fused, plain)


def test_full_size_sampled_rows():
    """4608 x 3072 (the FLUX token count and width) in the launch shape the benchmark times; the
    layer is row-wise, so the oracle checks a sample of rows exactly as it would check all."""
    rows, K, per = 4608, 3072, 1152
    rng = np.random.default_rng(9500)
    x_bits = _activations(rng, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    n_mod = rows // per
    gamma_bits = _bits(1.0 + 0.3 * rng.standard_normal(K))
    s_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    b_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    sample = np.unique(np.concatenate([[0, 7, 8, per - 1, per, rows - 1], rng.integers(0, rows, 58)]))
    x = _dev(x_bits)
    perm_d = torch.from_numpy(perm).to(DEV)
    for kind in (RMS, ADALN):
        _say("norm full size kind=%d" % kind)
        y = pq.pq_norm_reorder(kind, x, 1e-6, perm_d, _dev(gamma_bits), _dev(s_bits), _dev(b_bits), per)
        torch.cuda.synchronize()
        got = _host_bits(y)[sample]
        if kind == RMS:
            ref = ON.rmsnorm_reordered(OF.bf16_bits_to_f64(x_bits[sample]), OF.bf16_bits_to_f64(gamma_bits), 1e-6, perm)
        else:
            s = OF.bf16_bits_to_f64(s_bits)[sample // per]
            b = OF.bf16_bits_to_f64(b_bits)[sample // per]
            ref = ON.adaln_reordered(OF.bf16_bits_to_f64(x_bits[sample]), s, b, 1, 1e-6, perm)
        _check_close(got, ref, "full size")
        # every output row is a bijection of the input row's channels: no row is left unwritten
        assert torch.isfinite(y.float()).all()


def test_too_wide_rows_are_refused():
    K = 32768                      # 6 K bytes of LDS for one row and the two vectors: more than a workgroup has
    x = torch.zeros((8, K), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(pq.PQError) as e:
        pq.pq_norm_reorder(ADALN, x, 1e-6)
    assert e.value.code == -2


@pytest.mark.parametrize("rows,K", [(21, 7680), (5, 24576)])
def test_widest_supported_rows(rows, K):
    """Wide rows leave room for fewer rows per workgroup; at K = 24576 a workgroup holds one row and
    the vectors (147 KB of LDS plus the group maxima)."""
    rng = np.random.default_rng(9600)
    x_bits = _activations(rng, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    s_bits = _bits(0.5 * rng.standard_normal((1, K)))
    b_bits = _bits(0.5 * rng.standard_normal((1, K)))
    perm_d = torch.from_numpy(perm).to(DEV)
    x, s, b = _dev(x_bits), _dev(s_bits), _dev(b_bits)
    y = torch.empty((rows, K), dtype=torch.bfloat16, device=DEV)
    op = pq.pq_norm_quantize_act_packed(ADALN, pq.FMT_INT4, 64, x, 1e-6, None, perm_d, None, s, b, 0, y=y)
    want = pq.pq_quantize_act_packed(pq.FMT_INT4, 64, y, None)
    torch.cuda.synchronize()
    _check_close(_host_bits(y), _oracle(ADALN, x_bits, perm, None, s_bits, b_bits, 0, 1e-6), "widest")
    n = pq.pq_operand_bytes(pq.FMT_INT4, 64, rows, K)
    L_codes = (K // 64) * rows * 32
    assert torch.equal(op[:L_codes], want[:L_codes])          # the code part has no alignment gaps


def test_layernorm_rows_with_a_dominant_mean():
    """Rows whose mean is far larger than their spread: the variance must come from the deviations
    (mean square minus squared mean would lose every digit in fp32)."""
    rows, K = 16, 1024
    rng = np.random.default_rng(9700)
    offset = np.array([[0.0], [3.0], [40.0], [-500.0]] * 4)
    x_bits = _bits(offset + rng.standard_normal((rows, K)))
    perm = rng.permutation(K).astype(np.int32)
    y = pq.pq_norm_reorder(ADALN, _dev(x_bits), 1e-6, torch.from_numpy(perm).to(DEV))
    torch.cuda.synchronize()
    # at an offset of 500 a bf16 input is a multiple of 2, so a row holds only a handful of distinct
    # outputs: if one of them sits next to a bf16 rounding boundary, all its copies round the other way
    _check_close(_host_bits(y), _oracle(ADALN, x_bits, perm, None, None, None, 0, 1e-6), "dominant mean",
                 min_same=0.9)


@pytest.mark.parametrize("kind", [RMS, ADALN])
@pytest.mark.parametrize("rows,K,rows_per_mod", [(13, 6144, 5), (7, 12288, 0), (3, 4104, 2)])
def test_wide_rows_share_a_workgroup(kind, rows, K, rows_per_mod):
    """Rows wider than 4096 channels are worked on by the four waves of a workgroup together: same
    results as the oracle, and the quantizing call still equals norm followed by quantizer."""
    _say("norm wide kind=%d rows=%d K=%d" % (kind, rows, K))
    rng = np.random.default_rng(9650 + kind + rows + K)
    x_bits = _activations(rng, rows, K)
    perm = rng.permutation(K).astype(np.int32)
    n_mod = 1 if rows_per_mod <= 0 else -(-rows // rows_per_mod)
    gamma_bits = _bits(1.0 + 0.3 * rng.standard_normal(K))
    s_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    b_bits = _bits(0.5 * rng.standard_normal((n_mod, K)))
    perm_d = torch.from_numpy(perm).to(DEV)
    x, gamma, s, b = _dev(x_bits), _dev(gamma_bits), _dev(s_bits), _dev(b_bits)
    y = pq.pq_norm_reorder(kind, x, 1e-6, perm_d, gamma, s, b, rows_per_mod)
    torch.cuda.synchronize()
    _check_close(_host_bits(y), _oracle(kind, x_bits, perm, gamma_bits, s_bits, b_bits, rows_per_mod, 1e-6), "wide")
    if K % 64 == 0:
        for fmt, g in ((pq.FMT_INT4, 64), (pq.FMT_NVFP4, 16), (pq.FMT_INT3, 256)):
            Ta = torch.full((1,), 0.004, dtype=torch.float32, device=DEV)
            want = pq.pq_quantize_act_packed(fmt, g, y, Ta, torch.zeros(pq.pq_operand_bytes(fmt, g, rows, K), dtype=torch.uint8, device=DEV))
            y2 = torch.empty_like(y)
            got = pq.pq_norm_quantize_act_packed(kind, fmt, g, x, 1e-6, Ta, perm_d, gamma, s, b, rows_per_mod,
                                                 operand=torch.zeros_like(want), y=y2)
            torch.cuda.synchronize()
            assert torch.equal(y2, y) and torch.equal(got, want), (fmt, g)
