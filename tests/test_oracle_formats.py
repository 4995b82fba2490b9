"""Pins for the oracle's number formats: fixtures, library casts, closed-form properties."""
import os

import numpy as np
import pytest
import torch

from oracle import formats as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_values():
    out = {"e2m1": {}, "e4m3": {}}
    with open(os.path.join(GOLDEN, "e2m1_e4m3_values.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, code, val = line.split()
            out[name][int(code)] = float(val)
    return out


def test_e2m1_decode_matches_published_values():
    g = _golden_values()["e2m1"]
    assert len(g) == 8
    for code, val in g.items():
        assert F.e2m1_decode(code) == val


def test_e4m3_decode_matches_published_landmarks():
    for code, val in _golden_values()["e4m3"].items():
        assert F.e4m3_decode(code) == val


def test_e4m3_decode_agrees_with_torch_for_all_codes():
    codes = torch.arange(127, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(F.e4m3_decode(np.arange(127)), ref)


def test_e4m3_roundtrip_all_codes():
    v = F.e4m3_decode(np.arange(127))
    np.testing.assert_array_equal(F.e4m3_rne_sat(v), np.arange(127))


def test_e4m3_midpoints_go_to_even_code():
    v = F.e4m3_decode(np.arange(127))
    mid = 0.5 * (v[:-1] + v[1:])
    got = F.e4m3_rne_sat(mid)
    lo = np.arange(126)
    want = np.where(lo % 2 == 0, lo, lo + 1)
    np.testing.assert_array_equal(got, want)
    # just off the midpoint goes to the nearer neighbour
    np.testing.assert_array_equal(F.e4m3_rne_sat(np.nextafter(mid, 0.0)), lo)
    np.testing.assert_array_equal(F.e4m3_rne_sat(np.nextafter(mid, np.inf)), lo + 1)


def test_e4m3_saturation_and_underflow():
    assert F.e4m3_rne_sat(448.0) == 126
    assert F.e4m3_rne_sat(463.9) == 126
    assert F.e4m3_rne_sat(464.0) == 126
    assert F.e4m3_rne_sat(1e30) == 126
    assert F.e4m3_rne_sat(np.inf) == 126
    assert F.e4m3_rne_sat(2.0 ** -10) == 0          # tie between 0 and 2^-9 -> even code 0
    assert F.e4m3_rne_sat(np.nextafter(2.0 ** -10, 1.0)) == 1
    assert F.e4m3_rne_sat(0.0) == 0


def test_e4m3_rne_agrees_with_torch_cast_in_range():
    rng = np.random.default_rng(1)
    # fp32 values across the whole finite range below the saturation point
    x = np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), size=200000)).astype(np.float32)
    x = np.concatenate([x, np.float32([0.0, 448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10])])
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = F.e4m3_rne_sat(x.astype(np.float64))
    np.testing.assert_array_equal(got, ref.astype(np.int64))


def test_e2m1_rounding_bands_and_ties():
    # the eight values map to themselves
    np.testing.assert_array_equal(F.e2m1_rne_sat(F.E2M1_VALUES), np.arange(8))
    # ties: 0.25->0, 0.75->1.0, 1.25->1.0, 1.75->2.0, 2.5->2.0, 3.5->4.0, 5->4.0
    ties = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    np.testing.assert_array_equal(F.e2m1_rne_sat(ties), [0, 2, 2, 4, 4, 6, 6])
    eps = 1e-9
    np.testing.assert_array_equal(F.e2m1_rne_sat(ties - eps), [0, 1, 2, 3, 4, 5, 6])
    np.testing.assert_array_equal(F.e2m1_rne_sat(ties + eps), [1, 2, 3, 4, 5, 6, 7])
    assert F.e2m1_rne_sat(6.0) == 7 and F.e2m1_rne_sat(1e9) == 7 and F.e2m1_rne_sat(np.inf) == 7


def test_e2m1_nearest_by_brute_force():
    rng = np.random.default_rng(2)
    a = rng.uniform(0, 7, size=20000)
    idx = F.e2m1_rne_sat(a)
    dist = np.abs(a[:, None] - F.E2M1_VALUES[None, :])
    np.testing.assert_array_equal(np.abs(a - F.E2M1_VALUES[idx]), dist.min(axis=1))


def test_fl32_is_ieee_binary32_arithmetic():
    rng = np.random.default_rng(3)
    a = rng.standard_normal(100000).astype(np.float32) * np.float32(37.0)
    b = (rng.standard_normal(100000).astype(np.float32) + np.float32(3.0))
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    np.testing.assert_array_equal(F.fl32(a64 * b64), (a * b).astype(np.float64))
    np.testing.assert_array_equal(F.fl32(a64 / b64), (a / b).astype(np.float64))
    np.testing.assert_array_equal(F.fl32(1.0 / b64), (np.float32(1.0) / b).astype(np.float64))
    np.testing.assert_array_equal(F.fl32(a64 + b64), (a + b).astype(np.float64))


def test_bf16_widening_and_rounding_agree_with_torch():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite]
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(F.bf16_bits_to_f64(bits), ref)
    rng = np.random.default_rng(4)
    v = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))
    # include exact midpoints between neighbouring bf16 values
    b0 = rng.integers(0x0100, 0x7F00, size=4000).astype(np.uint16)
    mid = 0.5 * (F.bf16_bits_to_f64(b0) + F.bf16_bits_to_f64((b0 + 1).astype(np.uint16)))
    v = np.concatenate([v, mid, -mid, [0.0, -0.0]])
    # torch narrows fp64 through fp32 first; feed both sides fp32-representable values so
    # that only the bf16 rounding itself is compared
    v = v.astype(np.float32).astype(np.float64)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(F.f64_to_bf16_bits_rne(v), want)


def test_nibble_packing_layout():
    codes = np.array([[1, 2, 15, 0, 7, 8]], dtype=np.uint8)
    packed = F.pack_nibbles(codes)
    np.testing.assert_array_equal(packed, [[0x21, 0x0F, 0x87]])
    np.testing.assert_array_equal(F.unpack_nibbles(packed), codes)
    z = np.arange(-8, 8)
    np.testing.assert_array_equal(F.nibble_to_int(F.int_to_nibble(z)), z)
    assert F.int_to_nibble(-1) == 0xF and F.int_to_nibble(-7) == 0x9


def test_qmax():
    assert F.qmax(F.FMT_INT4) == 7 and F.qmax(F.FMT_INT3) == 3
    with pytest.raises(ValueError):
        F.qmax(F.FMT_NVFP4)
