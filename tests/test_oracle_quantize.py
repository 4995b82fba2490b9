"""Pins for the oracle's per-group quantizers (paper Sec. 3.1, Eq. 1-2, Eq. 4)."""
import os

import numpy as np
import pytest

from oracle import formats as F
from oracle import quantize as Qz
from paper_2605_09503_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bf16_values(rng, shape, spread=4.0):
    v = rng.standard_normal(shape) * np.exp(spread * rng.standard_normal(shape[-1]))[None, :]
    return F.bf16_bits_to_f64(synth.f64_to_bf16_bits(v))


def _worked_examples():
    ints, nvs = [], []
    with open(os.path.join(GOLDEN, "quantizer_worked_examples.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, xs, s, zs = [p.strip() for p in line.split("|")]
            kind, par = head.split()
            xs = np.array([float(t) for t in xs.split()])
            zs = np.array([int(t) for t in zs.split()])
            if kind == "int":
                ints.append((int(par), xs, float(s), zs))
            else:
                nvs.append((float(par), xs, int(s), zs))
    return ints, nvs


def test_int_worked_examples():
    ints, _ = _worked_examples()
    assert len(ints) >= 5
    for Q, x, s, z in ints:
        fmt = F.FMT_INT4 if Q == 7 else F.FMT_INT3
        q = Qz.quantize_int(x[None, :], len(x), fmt)
        assert q.scale[0, 0] == np.float32(s)
        np.testing.assert_array_equal(q.z[0], z)
        np.testing.assert_array_equal(Qz.dequantize_int(q, len(x))[0], s * z)


def test_nvfp4_worked_examples():
    _, nvs = _worked_examples()
    assert len(nvs) >= 2
    for T, x, sb, codes in nvs:
        q = Qz.quantize_nvfp4(x[None, :], np.float32(T))
        assert q.scale[0, 0] == sb
        np.testing.assert_array_equal(q.code[0], codes)
        # -0.0 keeps its sign bit although the magnitude is zero
        assert q.code[0, 10] == 8


@pytest.mark.parametrize("fmt,Q", [(F.FMT_INT4, 7), (F.FMT_INT3, 3)])
def test_int_codes_are_exactly_representable(fmt, Q):
    # every code times any scale quantizes back to itself when the group contains +-Q
    rng = np.random.default_rng(5)
    codes = np.arange(-Q, Q + 1)
    for _ in range(200):
        h = F.bf16_bits_to_f64(synth.f64_to_bf16_bits(np.exp(rng.uniform(-30, 30, 1))))[0]
        s = float(F.fl32(h / Q))
        x = s * codes.astype(np.float64)      # exact: 24-bit scale x 3-bit integer
        # x need not be bf16 here: the quantizer is defined on any binary32-representable input
        g = len(codes) + (len(codes) % 2)
        xx = np.zeros(g)
        xx[: len(codes)] = x
        q = Qz.quantize_int(xx[None, :], g, fmt)
        np.testing.assert_array_equal(q.z[0, : len(codes)], codes)


@pytest.mark.parametrize("fmt,g", [(F.FMT_INT4, 64), (F.FMT_INT4, 32), (F.FMT_INT3, 32), (F.FMT_INT3, 128)])
def test_int_error_bounds_and_group_max(fmt, g):
    Q = F.qmax(fmt)
    rng = np.random.default_rng(6)
    x = _bf16_values(rng, (64, 512))
    q = Qz.quantize_int(x, g, fmt)
    xh = Qz.dequantize_int(q, g)
    s = np.repeat(q.scale.astype(np.float64), g, axis=1)
    # round-to-nearest: |e| <= s/2 (App. A.1), up to the binary32 rounding of s and 1/s
    assert np.all(np.abs(x - xh) <= 0.5 * s * (1 + 2.0 ** -20))
    # Eq. 4 holds sample-wise: ||e||^2 <= g/(4Q^2) * sum_k max|x|^2
    amax = np.max(np.abs(x.reshape(64, -1, g)), axis=2)
    lhs = np.sum((x - xh) ** 2, axis=1)
    rhs = g / (4.0 * Q * Q) * np.sum(amax ** 2, axis=1)
    assert np.all(lhs <= rhs * (1 + 1e-6))
    # the largest element of each group lands on +-Q
    zz = np.abs(q.z.reshape(64, -1, g)).max(axis=2)
    assert np.all(zz[amax > 0] == Q)
    assert np.all(np.abs(q.z) <= Q)


def test_int_per_token_special_case_is_plain_rint():
    # g = K: per-token quantization, z = rint(x / s) away from exact ties
    rng = np.random.default_rng(7)
    x = _bf16_values(rng, (128, 256), spread=1.0)
    for fmt in (F.FMT_INT4, F.FMT_INT3):
        Q = F.qmax(fmt)
        q = Qz.quantize_int(x, 256, fmt)
        s = (np.max(np.abs(x), axis=1) / Q).astype(np.float32).astype(np.float64)
        ref = np.clip(np.rint(x / s[:, None]), -Q, Q)
        _, tie = Qz.quantize_int_exact(x, 256, fmt)
        assert tie.mean() < 0.05
        np.testing.assert_array_equal(q.z[~tie], ref[~tie].astype(np.int8))
        np.testing.assert_array_equal(q.scale[:, 0], s.astype(np.float32))


@pytest.mark.parametrize("fmt,g", [(F.FMT_INT4, 64), (F.FMT_INT3, 32)])
def test_int_pinned_sequence_equals_exact_eq2_except_on_ties(fmt, g):
    rng = np.random.default_rng(8)
    x = _bf16_values(rng, (256, 1024))
    q = Qz.quantize_int(x, g, fmt)
    z_exact, tie = Qz.quantize_int_exact(x, g, fmt)
    differ = q.z != z_exact
    assert not np.any(differ & ~tie)
    assert tie.sum() > 0                      # bf16 inputs do produce exact ties
    # on a tie the two candidates are the neighbours of the half-integer
    assert np.all(np.abs(q.z.astype(int) - z_exact.astype(int))[tie] <= 1)


@pytest.mark.parametrize("fmt,g", [(F.FMT_INT4, 64), (F.FMT_INT3, 32)])
def test_int_dynamic_idempotence(fmt, g):
    rng = np.random.default_rng(9)
    x = _bf16_values(rng, (32, 512))
    q1 = Qz.quantize_int(x, g, fmt)
    xh = Qz.dequantize_int(q1, g)             # exact fp64 values, binary32-representable
    q2 = Qz.quantize_int(xh, g, fmt)
    np.testing.assert_array_equal(q1.z, q2.z)
    s1, s2 = q1.scale.astype(np.float64), q2.scale.astype(np.float64)
    assert np.all(np.abs(s1 - s2) <= np.spacing(q1.scale).astype(np.float64))


def test_int_zero_and_subnormal_groups():
    x = np.zeros((1, 64))
    q = Qz.quantize_int(x, 64, F.FMT_INT4)
    assert q.scale[0, 0] == 0 and not q.z.any()
    tiny = 2.0 ** -130                         # bf16 subnormal; scale becomes subnormal
    x = np.full((1, 64), tiny)
    q = Qz.quantize_int(x, 64, F.FMT_INT4)
    assert q.scale[0, 0] == np.float32(tiny / 7.0) and not q.z.any()


def test_int_shuffle_inside_group_and_reversal_leave_error_unchanged():
    # Eq. 1: the scale depends on the set of channels in a group, not on their order
    rng = np.random.default_rng(10)
    x = _bf16_values(rng, (16, 256))
    g = 32
    base = np.sum((x - Qz.dequantize_int(Qz.quantize_int(x, g, F.FMT_INT4), g)) ** 2)
    perm = np.concatenate([k * g + rng.permutation(g) for k in range(256 // g)])
    xs = x[:, perm]
    e1 = np.sum((xs - Qz.dequantize_int(Qz.quantize_int(xs, g, F.FMT_INT4), g)) ** 2)
    xr = x[:, ::-1]
    e2 = np.sum((xr - Qz.dequantize_int(Qz.quantize_int(xr, g, F.FMT_INT4), g)) ** 2)
    assert np.isclose(e1, base, rtol=1e-13) and np.isclose(e2, base, rtol=1e-13)


# ------------------------------------------------------------------------------- NVFP4

def test_nvfp4_codes_are_exactly_representable_at_fixed_scale():
    # grid * block scale * T quantizes back to the same code whenever the block keeps its scale
    rng = np.random.default_rng(11)
    for _ in range(200):
        T = np.float32(np.exp(rng.uniform(-8, 8)))
        sb = int(rng.integers(8, 120))
        d = F.e4m3_decode(sb) * np.float64(T)
        mags = F.E2M1_VALUES
        x = np.concatenate([mags, -mags]) * d
        # the block contains +-6*d, so amax/6 = d and the block scale is recovered unless
        # fl32 rounding moves it to a neighbouring E4M3 value; check the precondition
        q = Qz.quantize_nvfp4(x[None, :], T)
        if q.scale[0, 0] != sb:
            continue
        want = np.concatenate([np.arange(8), 8 + np.arange(8)])
        np.testing.assert_array_equal(q.code[0], want)


def test_nvfp4_band_errors_sign_and_saturation():
    rng = np.random.default_rng(12)
    x = _bf16_values(rng, (64, 512), spread=2.0)
    T = Qz.nvfp4_tensor_scale(np.max(np.abs(x)))
    q = Qz.quantize_nvfp4(x, T)
    d = np.repeat(F.e4m3_decode(q.scale) * np.float64(T), 16, axis=1)
    ok = d > 0
    v = np.abs(x[ok]) / d[ok]
    mag = F.e2m1_decode(q.code[ok] & 7)
    err = np.abs(v - mag)
    unsat = v <= 6.0
    band = np.where(mag < 2, 0.25, np.where(mag < 4, 0.5, 1.0))
    # nearest code: error at most half the local spacing (the spacing above the code
    # bounds it for values rounded down, the one below for values rounded up)
    assert np.all(err[unsat] <= np.maximum(band[unsat], 0.25) * (1 + 1e-6) + 1e-12)
    assert np.all(mag[~unsat] == 6.0)
    # block scale is rounded to nearest (not up), so |v| may exceed 6, but never by more
    # than the relative half-spacing of E4M3 (1/16)
    assert v.max() <= 6.0 * (1 + 1.0 / 16 + 1e-6)
    np.testing.assert_array_equal((q.code >> 3).astype(bool), np.signbit(x))


def test_nvfp4_nearest_code_by_brute_force():
    # A million elements.  The pinned binary32 sequence and the exact-real quotient disagree only within
    # 2^-18 (relative) of an E2M1 midpoint; bf16 inputs land that close to a midpoint more often than a
    # continuous distribution would (both x and the scale have few significant bits): 4.4e-4 of the
    # elements here, none of them outside the near-tie window.
    rng = np.random.default_rng(13)
    n_bad = n_all = 0
    for _ in range(4):
        x = _bf16_values(rng, (1024, 256), spread=1.0)
        T = Qz.nvfp4_tensor_scale(np.max(np.abs(x)))
        q = Qz.quantize_nvfp4(x, T)
        d = np.repeat(F.e4m3_decode(q.scale) * np.float64(T), 16, axis=1)
        ok = d > 0
        v = np.abs(x[ok]) / d[ok]
        dist = np.abs(v[:, None] - F.E2M1_VALUES[None, :])
        chosen = np.abs(v - F.e2m1_decode(q.code[ok] & 7))
        # agreement with the exact-real nearest code except within 2^-18 (relative) of a midpoint
        bad = chosen > dist.min(axis=1)
        mids = 0.5 * (F.E2M1_VALUES[:-1] + F.E2M1_VALUES[1:])
        near = np.min(np.abs(v[:, None] - mids[None, :]) / mids[None, :], axis=1) < 2.0 ** -18
        assert not np.any(bad & ~near)
        n_bad += int(bad.sum())
        n_all += bad.size
    assert n_all >= 1000000 and n_bad < 1e-3 * n_all, (n_bad, n_all)


def test_nvfp4_block_scale_against_direct_definition():
    # block scale = E4M3 image of amax / (6 T), up to the binary32 rounding of the two steps
    rng = np.random.default_rng(14)
    x = _bf16_values(rng, (64, 256), spread=2.0)
    T = Qz.nvfp4_tensor_scale(np.max(np.abs(x)))
    q = Qz.quantize_nvfp4(x, T)
    amax = np.max(np.abs(x.reshape(64, -1, 16)), axis=2)
    direct = F.e4m3_rne_sat(amax / (6.0 * np.float64(T)))
    diff = np.abs(direct - q.scale.astype(np.int64))
    assert np.all(diff <= 1) and (diff != 0).mean() < 1e-3
    # the largest block reaches the top of the E4M3 range (that is what T is for)
    assert q.scale.max() == 126


def test_nvfp4_idempotence():
    rng = np.random.default_rng(15)
    x = _bf16_values(rng, (32, 256), spread=1.0)
    T = Qz.nvfp4_tensor_scale(np.max(np.abs(x)))
    q1 = Qz.quantize_nvfp4(x, T)
    xh = Qz.dequantize_nvfp4(q1)
    q2 = Qz.quantize_nvfp4(xh, T)
    # blocks whose largest code is 6 keep their scale and therefore all their codes
    top = (q1.code.reshape(32, -1, 16) & 7).max(axis=2) == 7
    same_scale = q1.scale == q2.scale
    assert np.all(same_scale[top])
    c1 = q1.code.reshape(32, -1, 16)[top]
    c2 = q2.code.reshape(32, -1, 16)[top]
    nz = (c1 & 7) != 0                       # signed zero: sign of xhat = sign bit kept
    np.testing.assert_array_equal(c1[nz], c2[nz])


def test_nvfp4_zero_tensor_and_overflowing_activations():
    q = Qz.quantize_nvfp4(np.zeros((2, 32)), np.float32(0.0))
    assert not q.scale.any() and not (q.code & 7).any()
    # live activations 100x above the calibration maximum: block scale saturates at 448,
    # codes saturate at +-6
    x = np.full((1, 16), 1000.0)
    x[0, 1] = -1000.0
    T = Qz.nvfp4_tensor_scale(10.0)
    q = Qz.quantize_nvfp4(x, T)
    assert q.scale[0, 0] == 126
    assert q.code[0, 0] == 7 and q.code[0, 1] == 15


def test_uniform_noise_model_sanity():
    # App. A.3: under the uniform-noise model E[e^2] = s^2/12, i.e. the measured INT error is
    # about g/(12 Q^2) * sum_k max^2 -- loose statistical check (factor 2 either way)
    rng = np.random.default_rng(16)
    x = F.bf16_bits_to_f64(synth.f64_to_bf16_bits(rng.standard_normal((512, 1024))))
    g, Q = 64, 7
    q = Qz.quantize_int(x, g, F.FMT_INT4)
    err = np.sum((x - Qz.dequantize_int(q, g)) ** 2)
    amax = np.max(np.abs(x.reshape(512, -1, g)), axis=2)
    model = g / (12.0 * Q * Q) * np.sum(amax ** 2)
    assert 0.5 * model < err < 2.0 * model


def test_packed_codes_layout():
    x = np.array([[7.0, -7.0, 1.0, 0.0] * 4])
    q = Qz.quantize_int(x, 16, F.FMT_INT4)
    p = Qz.packed_codes(F.FMT_INT4, q)
    assert p.shape == (1, 8) and p[0, 0] == (7 | (9 << 4)) and p[0, 1] == 1


# ----------------------------------------------------------------------------------------------
# The binary32 steps of the quantizers, re-derived in exact rational arithmetic.
#
# Where a floating-point value decides an integer code, oracle and kernels take the decision in
# binary32, step by step:  INT    s = fl(amax / Q), r = fl(1 / s), v = fl(x r), z = rint(v);
#                          NVFP4  r_T = fl(1 / T), t = fl(fl(amax r_T) / 6), byte = E4M3(t),
#                                 d = fl(E4M3(byte) T), r = fl(1 / d), v = fl(x r), code = E2M1(|v|).
# Below every fl() is a rounding of an exact fraction to 24 significant bits, ties to even, written
# with integers only; E4M3 and E2M1 are nearest-value searches over their value lists.  The inputs
# were picked (by a search over bf16 values) so that leaving out any single fl() changes a code or
# a scale byte: a sequence with one step kept in higher precision fails here.
from fractions import Fraction


def _rn24(q: Fraction) -> Fraction:
    if q == 0:
        return q
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1) and -126 <= e <= 127
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return (fl * ulp) if q > 0 else -(fl * ulp)


def _rint_half_even(q: Fraction) -> int:
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def _nearest(values, q: Fraction) -> int:
    """Index of the value nearest to q >= 0 in an ascending list, ties to the even index, saturating."""
    best = 0
    for i, v in enumerate(values):
        d, db = abs(v - q), abs(values[best] - q)
        if d < db or (d == db and i % 2 == 0):
            best = i
    return best


_E4M3_VALUES = [Fraction(m, 8) * Fraction(2) ** -6 for m in range(8)] + \
               [(1 + Fraction(m, 8)) * Fraction(2) ** e for e in range(-6, 9) for m in range(8)][:-1]
_E2M1_VALUES = [Fraction(v) for v in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]


def _int_codes_rational(x, Q):
    xs = [Fraction(float(v)) for v in x]
    amax = max(abs(v) for v in xs)
    s = _rn24(amax / Q)
    r = _rn24(1 / s)
    return s, [max(-Q, min(Q, _rint_half_even(_rn24(v * r)))) for v in xs]


def _nvfp4_rational(x, T):
    xs = [Fraction(float(v)) for v in x]
    T = Fraction(float(np.float32(T)))
    amax = max(abs(v) for v in xs)
    t = _rn24(_rn24(amax * _rn24(1 / T)) / 6)
    byte = _nearest(_E4M3_VALUES, t)
    d = _rn24(_E4M3_VALUES[byte] * T)
    r = _rn24(1 / d)
    return byte, [_nearest(_E2M1_VALUES, abs(_rn24(v * r))) for v in xs]


def test_e4m3_value_list_of_the_rational_check():
    assert len(_E4M3_VALUES) == 127 and _E4M3_VALUES[-1] == 448 and _E4M3_VALUES[1] == Fraction(1, 512)
    assert [float(v) for v in _E4M3_VALUES] == [float(v) for v in F.e4m3_decode(np.arange(127))]


_INT_SENSITIVE = [
    (7, [-1.025910023599863e-09, 0.000583648681640625, -0.00116729736328125, 3.119930624961853e-08]),
    (7, [-0.0025482177734375, -2.8172507882118225e-08, 0.005096435546875, 0.00025177001953125]),
    (7, [2.293381839990616e-08, 210.0, 75.0, -0.0069580078125]),
    (3, [976.0, 944.0, 4.678964614868164e-06, -5664.0]),
    (7, [-5.125999450683594e-06, 2.3365020751953125e-05, -1.6689300537109375e-06, -1.3262033462524414e-06]),
    (7, [0.00677490234375, -3.623426891863346e-09, 1.2922100722789764e-08, -0.0135498046875]),
    (7, [91.0, 32.5, -32.5, 6.5]),
]


@pytest.mark.parametrize("Q,x", _INT_SENSITIVE)
def test_int_binary32_sequence_in_rational_arithmetic(Q, x):
    fmt = F.FMT_INT4 if Q == 7 else F.FMT_INT3
    q = Qz.quantize_int(np.array([x]), len(x), fmt)
    s, z = _int_codes_rational(x, Q)
    assert Fraction(float(q.scale[0, 0])) == s
    assert q.z[0].tolist() == z


_NVFP4_SENSITIVE = [
    # (T, amax element, +-x): the reciprocal of the block scale, then the product, decide a code
    (1.0, [1.4375, 0.29296875, -0.29296875]),
    (1.0, [1.4375, 0.5859375, -0.5859375]),
    (1.0, [0.859375, 0.03515625, -0.03515625]),
    (1.0, [0.859375, 0.17578125, -0.17578125]),
    # the reciprocal of T, then the product with the block maximum, decide the scale byte
    (0.29891306161880493, [0.040283203125, 0.01, -0.02]),
    (0.394097238779068, [0.006927490234375, 0.001, -0.003]),
]


@pytest.mark.parametrize("T,head", _NVFP4_SENSITIVE)
def test_nvfp4_binary32_sequence_in_rational_arithmetic(T, head):
    x = np.zeros(16)
    x[:len(head)] = F.bf16_bits_to_f64(F.f64_to_bf16_bits_rne(np.array(head)))
    q = Qz.quantize_nvfp4(x[None, :], np.float32(T))
    byte, idx = _nvfp4_rational(x, T)
    assert int(q.scale[0, 0]) == byte
    assert (q.code[0] & 7).tolist() == idx


def test_binary32_sequence_on_random_rows():
    rng = np.random.default_rng(77)
    for trial in range(40):
        x = F.bf16_bits_to_f64(F.f64_to_bf16_bits_rne(rng.standard_normal(16) * np.exp(rng.standard_normal(16))))
        Q = 7 if trial % 2 else 3
        q = Qz.quantize_int(x[None, :], 16, F.FMT_INT4 if Q == 7 else F.FMT_INT3)
        s, z = _int_codes_rational(x, Q)
        assert Fraction(float(q.scale[0, 0])) == s and q.z[0].tolist() == z
        T = np.float32(rng.uniform(0.001, 0.01))
        qn = Qz.quantize_nvfp4(x[None, :], T)
        byte, idx = _nvfp4_rational(x, T)
        assert int(qn.scale[0, 0]) == byte and (qn.code[0] & 7).tolist() == idx
