"""Helpers shared by the parity tests: run the oracle and the GPU library on the same bits."""
from __future__ import annotations

import numpy as np

from oracle import calib as OC
from oracle import formats as OF
from oracle import gemm as OG
from oracle import quantize as OQ

# tolerances of the parity bar
GEMM_F32_RTOL = 1e-3        # fp32-accumulator output vs fp64 reference, on |y_ref| > GEMM_ABS_FLOOR
GEMM_F32_RTOL_NVFP4 = 1e-4  # the stricter form, met where outputs do not cancel heavily (measured ~1e-7 on NVFP4)
GEMM_ABS_FLOOR = 1e-2
GEMM_ACC_UNITS = 32         # allowed accumulation error in units of 2^-24 of sum_k |terms|
MOMENTS_RTOL = 1e-12
ERRSUM_RTOL = 1e-10


def oracle_quantize_bits(fmt, g, bits_u16, perm=None, tensor_scale=None):
    """bf16 bits [rows, K] -> (packed codes u8 [rows, K/2], scales, quant tuple)."""
    x = OF.bf16_bits_to_f64(bits_u16)
    if perm is not None:
        x = x[:, np.asarray(perm)]
    q = OQ.quantize(fmt, g, x, tensor_scale)
    return OQ.packed_codes(fmt, q), q.scale, q


def bf16_ulp_distance(bits_a, bits_b):
    """Distance in bf16 units in the last place between two arrays of bf16 bit patterns."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(np.asarray(bits_a)) - key(np.asarray(bits_b)))


def abs_product(fmt, g, qa, qw):
    """sum_k |xhat[m, k] * what[n, k]|: the scale against which fp32 accumulation error is judged."""
    return np.abs(OQ.dequantize(fmt, g, qa)) @ np.abs(OQ.dequantize(fmt, g, qw)).T


def gemm_f32_check(y_gpu, y_ref, mag, label="", fmt=None):
    """fp32-accumulator output against the fp64 reference.

    (a) |err| <= 32 * 2^-24 * sum_k |terms| for every output: products are exact in the kernel,
        so the only error is the fp32 accumulation over K terms (worst case K * 2^-24 of the
        absolute sum, a few units of 2^-24 in practice) plus two roundings in the epilogue;
    (b) the task's form: max relative error <= 1e-3 on outputs with |y_ref| > 1e-2 -- 1e-4 for NVFP4
        (fmt == 0).  The INT configurations with outlier channels have outputs just above the floor that
        are the difference of terms thousands of times larger; there the relative form amplifies the
        2^-24 accumulation error to as much as 5e-4, and only (a) is a tight statement.
    Returns the largest relative error of (b)."""
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    err = np.abs(y_gpu - y_ref)
    worst = float((err / np.maximum(mag, 1e-300)).max())
    assert worst <= GEMM_ACC_UNITS * 2.0 ** -24, "%s accumulation error %.2f units of 2^-24 of sum|terms|" % (
        label, worst * 2.0 ** 24)
    big = np.abs(y_ref) > GEMM_ABS_FLOOR
    rel = err[big] / np.abs(y_ref[big])
    max_rel = float(rel.max()) if rel.size else 0.0
    rtol = GEMM_F32_RTOL_NVFP4 if fmt == 0 else GEMM_F32_RTOL
    assert max_rel <= rtol, "%s max rel err %.3e" % (label, max_rel)
    return max_rel


def gemm_bf16_check(y_bits_gpu, y_ref, label=""):
    """bf16 output equals bf16_rne(y_ref) or its neighbour."""
    ref_bits = OG.bf16_round(y_ref)
    d = bf16_ulp_distance(y_bits_gpu, ref_bits)
    # tiny outputs: fp32 accumulation noise can exceed one bf16 ulp of a near-zero result
    big = np.abs(y_ref) > GEMM_ABS_FLOOR
    assert d[big].max(initial=0) <= 1, "%s bf16 output off by %d ulp" % (label, int(d[big].max()))
    ref_f = OF.bf16_bits_to_f64(ref_bits)
    got_f = OF.bf16_bits_to_f64(np.asarray(y_bits_gpu))
    # below the floor: the fp32 path's absolute allowance plus one bf16 ulp at the floor (2^-14)
    assert np.all(np.abs(got_f[~big] - ref_f[~big]) <= GEMM_F32_RTOL * GEMM_ABS_FLOOR + 2.0 ** -14), label
    return float((d[big] == 0).mean()) if big.any() else 1.0
