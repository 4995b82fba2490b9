"""GPU parity of the dense 3-bit storage of INT3 codes against oracle/int3.py, through the C ABI:
bytes bit-exact in both directions, the quantizer's own codes round-tripped, the GEMM operand built
from the dense form equal to the one built from nibbles, and the W3A3 product from 3-bit weights
against the fp64 product."""
import sys

import numpy as np
import pytest
import torch

from oracle import formats as OF
from oracle import gemm as OG
from oracle import int3 as O3
from oracle import quantize as OQ
from paper_2605_09503_amd import pq, synth

import pq_testlib as T

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


# one piece; a partial workgroup; exactly one workgroup of 256 pieces; several workgroups and a tail
SHAPES = [(1, 32), (3, 96), (8, 1024), (37, 1056), (515, 3072), (4, 16384)]


@pytest.mark.parametrize("rows,K", SHAPES)
def test_pack_and_unpack_match_the_oracle(rows, K):
    _say("int3 dense rows=%d K=%d" % (rows, K))
    rng = np.random.default_rng(rows * 7 + K)
    z = rng.integers(-3, 4, size=(rows, K))
    z[0, :8] = [-4, 3, -3, 2, -2, 1, -1, 0]                 # every representable code
    nib = OF.pack_nibbles(OF.int_to_nibble(z))
    ref = O3.pack_dense(z)
    assert pq.pq_int3_dense_bytes(rows, K) == ref.size
    guard = 64
    dense = torch.full((ref.size + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    got = pq.pq_int3_pack(torch.from_numpy(nib).to(DEV), dense[:ref.size].view(rows, -1))
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref)
    assert bool((dense[ref.size:] == 0xA5).all()), "wrote past the end of the dense buffer"
    codes = torch.full((nib.size + guard,), 0x5A, dtype=torch.uint8, device=DEV)
    back = pq.pq_int3_unpack(torch.from_numpy(ref).to(DEV), K, codes[:nib.size].view(rows, -1))
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), nib)
    assert np.array_equal(OF.nibble_to_int(OF.unpack_nibbles(back.cpu().numpy())), O3.unpack_dense(ref, K))
    assert bool((codes[nib.size:] == 0x5A).all()), "wrote past the end of the nibble buffer"


def test_unpack_of_arbitrary_bytes():
    """Every byte string is a valid dense row."""
    rows, K = 9, 640
    rng = np.random.default_rng(11)
    p = rng.integers(0, 256, size=(rows, 3 * K // 8), dtype=np.uint8)
    back = pq.pq_int3_unpack(torch.from_numpy(p).to(DEV), K)
    torch.cuda.synchronize()
    assert np.array_equal(OF.nibble_to_int(OF.unpack_nibbles(back.cpu().numpy())), O3.unpack_dense(p, K))
    again = pq.pq_int3_pack(back)
    torch.cuda.synchronize()
    assert np.array_equal(again.cpu().numpy(), p)


@pytest.mark.parametrize("g", [32, 64, 128, 256])
def test_operand_from_dense_codes_equals_operand_from_nibbles(g):
    rows, K = 203, 1280
    _say("int3 operand from dense g=%d" % g)
    rng = np.random.default_rng(50 + g)
    wb = synth.f64_to_bf16_bits(0.05 * rng.standard_normal((rows, K)) * np.exp(rng.standard_normal(K))[None, :])
    codes, scales = pq.alloc_quantized(pq.FMT_INT3, g, rows, K, DEV)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    pq.pq_quantize_weights(pq.FMT_INT3, g, pq.bf16_from_bits(wb, DEV), None, codes, scales, one)
    torch.cuda.synchronize()
    q = OQ.quantize(pq.FMT_INT3, g, OF.bf16_bits_to_f64(wb), None)
    dense = pq.pq_int3_pack(codes)
    torch.cuda.synchronize()
    assert np.array_equal(dense.cpu().numpy(), O3.pack_dense(q.z))          # the quantizer's codes, 3 bits each
    n = pq.pq_operand_bytes(pq.FMT_INT3, g, rows, K)
    a = torch.zeros(n, dtype=torch.uint8, device=DEV)
    b = torch.zeros(n, dtype=torch.uint8, device=DEV)
    pq.pq_pack_operand(pq.FMT_INT3, g, codes, scales, a)
    pq.pq_pack_operand_int3(g, dense, scales, K, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_w3a3_product_from_dense_weights():
    """Weights kept at three bits per code, activations quantized on the fly: the product equals the
    fp64 product of the dequantized operands to the GEMM tolerance."""
    fmt, g, M, N, K = pq.FMT_INT3, 32, 150, 264, 1024
    rng = np.random.default_rng(808)
    chan = np.exp(rng.standard_normal(K))
    xb = synth.f64_to_bf16_bits(rng.standard_normal((M, K)) * chan[None, :])
    wb = synth.f64_to_bf16_bits(0.02 * rng.standard_normal((N, K)))
    x64, w64 = OF.bf16_bits_to_f64(xb), OF.bf16_bits_to_f64(wb)
    qa, qw = OQ.quantize(fmt, g, x64, None), OQ.quantize(fmt, g, w64, None)
    y_ref = OG.dequant_product(fmt, g, qa, qw)
    # offline: the oracle's codes in dense form are what a checkpoint would hold
    dense = torch.from_numpy(O3.pack_dense(qw.z)).to(DEV)
    w_scales = torch.from_numpy(np.ascontiguousarray(qw.scale)).to(DEV)
    w_op = pq.pq_pack_operand_int3(g, dense, w_scales, K)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    a_op = pq.pq_quantize_act_packed(fmt, g, pq.bf16_from_bits(xb, DEV), one)
    y32 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    pq.pq_qgemm_packed_f32(fmt, g, a_op, one, w_op, one, y32, M, N, K)
    torch.cuda.synchronize()
    T.gemm_f32_check(y32.cpu().numpy(), y_ref, T.abs_product(fmt, g, qa, qw), "w3a3 from dense weights")


def test_full_size_weight_round_trip():
    """The W3A3 weight of the largest INT3 configuration, [12288, 3072]: dense size, sampled rows against
    the oracle, exact round trip of the whole tensor."""
    rows, K = 12288, 3072
    g = torch.Generator(device="cpu").manual_seed(5)
    z = torch.randint(-3, 4, (rows, K), generator=g, dtype=torch.int8)
    zn = z.numpy().astype(np.int64)
    nib = torch.from_numpy(OF.pack_nibbles(OF.int_to_nibble(zn))).to(DEV)
    dense = pq.pq_int3_pack(nib)
    back = pq.pq_int3_unpack(dense, K)
    torch.cuda.synchronize()
    assert dense.numel() == rows * K * 3 // 8
    assert torch.equal(back, nib)
    d = dense.cpu().numpy()
    for r in (0, 1, 4095, 6001, rows - 1):
        assert np.array_equal(d[r], O3.pack_dense(zn[r:r + 1])[0])
