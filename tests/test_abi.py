"""The C-ABI library loads, exports what include/permuquant.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed: no valid call is made)."""
import ctypes as C
import os
import re

import pytest

from paper_2605_09503_amd import pq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "permuquant.h")

PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_FORMAT, PQ_ERR_WORKSPACE = -1, -2, -3, -4


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pq.lib_path()):
        from paper_2605_09503_amd import build
        build.build(verbose=False)
    return pq.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pq_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = _declared_functions()
    assert {"pq_calib_moments", "pq_select_perm", "pq_quantize_weights", "pq_quantize_act",
            "pq_qgemm"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "missing export " + n
    assert lib.pq_version() >= 100
    assert isinstance(pq.pq_last_error(), str)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(pq, "_lib", None)
    monkeypatch.setattr(pq, "_LIB_PATH", "/nonexistent/libpermuquant.so")
    with pytest.raises(pq.PQError):
        pq.load()


FAKE = C.c_void_p(0x1000)          # non-NULL, 16-byte aligned, never dereferenced on the host


def test_calib_moments_validation(lib):
    f = lib.pq_calib_moments
    assert f(None, 8, 64, 64, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert f(FAKE, 8, 64, 64, None, None, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert f(FAKE, 0, 64, 64, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert f(FAKE, 8, 60, 64, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_SHAPE      # K % 8
    assert f(FAKE, 8, 64, 32, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_SHAPE      # ld < K
    assert f(C.c_void_p(0x1004), 8, 64, 64, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert f(FAKE, 8, 64, 64, FAKE, None, None, 0, None) == PQ_ERR_WORKSPACE
    assert f(FAKE, 8, 64, 64, FAKE, None, FAKE, 8, None) == PQ_ERR_WORKSPACE
    assert "workspace" in pq.pq_last_error()


def test_calib_moments_static_validation(lib):
    """The variant with library-held scratch: same argument checks, and shapes whose partial sums do not
    fit the array are refused on the host (no launch, no GPU needed)."""
    f = lib.pq_calib_moments_static
    assert f(None, 8, 64, 64, FAKE, None, None) == PQ_ERR_NULL
    assert f(FAKE, 8, 64, 64, None, None, None) == PQ_ERR_NULL
    assert f(FAKE, 0, 64, 64, FAKE, None, None) == PQ_ERR_SHAPE
    assert f(FAKE, 8, 60, 64, FAKE, None, None) == PQ_ERR_SHAPE
    assert f(FAKE, 8, 64, 32, FAKE, None, None) == PQ_ERR_SHAPE
    assert f(C.c_void_p(0x1004), 8, 64, 64, FAKE, None, None) == PQ_ERR_SHAPE
    # the benchmark's tensors fit; a tensor half a million channels wide does not
    for rows, K in [(4608, 3072), (4608, 12288), (8192, 3072), (12288, 3072), (3072, 12288)]:
        assert lib.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, 0, 0, rows, 0, K, 1) <= pq.STATIC_SCRATCH_BYTES
    assert lib.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, 0, 0, 64, 0, 524288, 1) > pq.STATIC_SCRATCH_BYTES
    assert f(FAKE, 64, 524288, 524288, FAKE, None, None) == PQ_ERR_WORKSPACE
    assert "scratch" in pq.pq_last_error()
    text = open(HEADER).read()
    assert "#define PQ_STATIC_SCRATCH_BYTES ((size_t)3 << 20)" in text and pq.STATIC_SCRATCH_BYTES == 3 << 20


def test_select_width_limit_is_checked_on_the_host(lib):
    """A row of the error evaluation must fit LDS: K above 34128 is refused before any launch, and
    pq_workspace_bytes says so by returning 0."""
    assert lib.pq_workspace_bytes(pq.OP_SELECT_PERM, pq.FMT_INT4, 64, 64, 64, 34112, 2) > 0
    assert lib.pq_workspace_bytes(pq.OP_SELECT_PERM, pq.FMT_INT4, 64, 64, 64, 34176, 2) == 0
    assert lib.pq_workspace_bytes(pq.OP_QUANT_ERROR, pq.FMT_INT4, 64, 64, 0, 34176, 0) == 0
    qe = lib.pq_quant_error
    assert qe(pq.FMT_INT4, 64, FAKE, 8, 34176, None, C.c_float(1.0), FAKE, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert "LDS" in pq.pq_last_error()
    chk = lib.pq_qgemm_check_int_scales
    n = C.c_int64(0)
    assert chk(pq.FMT_INT4, 64, None, 8, 64, C.byref(n), FAKE, 256, None) == PQ_ERR_NULL
    assert chk(pq.FMT_NVFP4, 16, FAKE, 8, 64, C.byref(n), FAKE, 256, None) == PQ_ERR_FORMAT
    assert chk(pq.FMT_INT4, 64, FAKE, 8, 64, C.byref(n), FAKE, 16, None) == PQ_ERR_WORKSPACE
    assert chk(pq.FMT_INT4, 64, FAKE, 0, 64, C.byref(n), FAKE, 256, None) == PQ_ERR_SHAPE


def test_quantize_validation(lib):
    qa = lib.pq_quantize_act
    assert qa(pq.FMT_NVFP4, 16, None, 4, 64, 64, None, FAKE, FAKE, FAKE, None) == PQ_ERR_NULL
    assert qa(pq.FMT_NVFP4, 16, FAKE, 4, 64, 64, None, None, FAKE, FAKE, None) == PQ_ERR_NULL   # no T
    assert qa(7, 16, FAKE, 4, 64, 64, None, FAKE, FAKE, FAKE, None) == PQ_ERR_FORMAT
    assert qa(pq.FMT_NVFP4, 32, FAKE, 4, 64, 64, None, FAKE, FAKE, FAKE, None) == PQ_ERR_FORMAT
    assert qa(pq.FMT_INT4, 16, FAKE, 4, 64, 64, None, None, FAKE, FAKE, None) == PQ_ERR_FORMAT
    assert qa(pq.FMT_INT3, 48, FAKE, 4, 96, 96, None, None, FAKE, FAKE, None) == PQ_ERR_FORMAT
    assert qa(pq.FMT_INT4, 64, FAKE, 4, 96, 96, None, None, FAKE, FAKE, None) == PQ_ERR_SHAPE    # K % g
    assert qa(pq.FMT_INT4, 64, FAKE, 0, 64, 64, None, None, FAKE, FAKE, None) == PQ_ERR_SHAPE
    assert qa(pq.FMT_INT4, 64, FAKE, 4, 64, 32, None, None, FAKE, FAKE, None) == PQ_ERR_SHAPE    # ld < K
    assert qa(pq.FMT_INT4, 64, FAKE, 4, -64, 64, None, None, FAKE, FAKE, None) == PQ_ERR_SHAPE
    qw = lib.pq_quantize_weights
    assert qw(pq.FMT_INT4, 64, FAKE, 4, 64, None, FAKE, FAKE, None, None) == PQ_ERR_NULL
    assert qw(pq.FMT_INT4, 64, FAKE, 4, 65, None, FAKE, FAKE, FAKE, None) == PQ_ERR_SHAPE
    assert qw(pq.FMT_INT4, 64, FAKE, -1, 64, None, FAKE, FAKE, FAKE, None) == PQ_ERR_SHAPE


def test_select_and_error_validation(lib):
    f = lib.pq_select_perm
    ptrs = (C.c_void_p * 1)(0x2000)
    al = (C.c_double * 2)(0.0, 1.0)
    rep = pq._Report()
    ok_args = dict(fmt=pq.FMT_INT4, group=64, sa=FAKE, sw=FAKE, K=128, xs=ptrs, nb=1, M=8, w=FAKE, N=8,
                   ta=1.0, tw=1.0, al=al, na=2, tau=0.0, out=FAKE, rep=C.byref(rep), ws=FAKE,
                   wsb=1 << 30, st=None)

    def call(**kw):
        a = dict(ok_args)
        a.update(kw)
        return f(a["fmt"], a["group"], a["sa"], a["sw"], a["K"], a["xs"], a["nb"], a["M"], a["w"], a["N"],
                 a["ta"], a["tw"], a["al"], a["na"], a["tau"], a["out"], a["rep"], a["ws"], a["wsb"], a["st"])

    assert call(sa=None) == PQ_ERR_NULL
    assert call(out=None) == PQ_ERR_NULL
    assert call(na=0) == PQ_ERR_SHAPE
    assert call(na=16) == PQ_ERR_SHAPE
    assert call(nb=0) == PQ_ERR_SHAPE
    assert call(K=100) == PQ_ERR_SHAPE
    assert call(group=48) == PQ_ERR_FORMAT
    assert call(al=(C.c_double * 2)(0.0, 1.5)) == PQ_ERR_SHAPE
    assert call(tau=float("nan")) == PQ_ERR_SHAPE
    assert call(xs=(C.c_void_p * 1)(None)) == PQ_ERR_NULL
    assert call(wsb=16) == PQ_ERR_WORKSPACE
    assert call(ws=None) == PQ_ERR_WORKSPACE
    # the variant with the tensor scales in device memory: NVFP4 needs both pointers, the integer formats none
    f = lib.pq_select_perm_device_scales
    assert call(fmt=pq.FMT_NVFP4, group=16, ta=None, tw=FAKE) == PQ_ERR_NULL
    assert call(fmt=pq.FMT_NVFP4, group=16, ta=FAKE, tw=None) == PQ_ERR_NULL
    assert "tensor scales" in pq.pq_last_error()
    assert call(ta=None, tw=None, wsb=16) == PQ_ERR_WORKSPACE       # past the pointer check, stopped later
    assert call(ta=None, tw=None, na=0) == PQ_ERR_SHAPE
    e = lib.pq_quant_error
    assert e(pq.FMT_INT3, 32, None, 4, 64, None, 1.0, FAKE, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert e(pq.FMT_INT3, 32, FAKE, 4, 64, None, 1.0, FAKE, FAKE, 8, None) == PQ_ERR_WORKSPACE
    assert e(pq.FMT_INT3, 32, FAKE, 4, 72, None, 1.0, FAKE, FAKE, 1 << 20, None) == PQ_ERR_SHAPE


def test_qgemm_validation(lib):
    for f in (lib.pq_qgemm, lib.pq_qgemm_f32):
        def call(fmt=pq.FMT_INT4, group=64, a=FAKE, sa=FAKE, ta=None, w=FAKE, sw=FAKE, tw=None, M=8, N=8,
                 K=128, y=FAKE, ldy=8, ws=FAKE, wsb=1 << 30):
            return f(fmt, group, a, sa, ta, w, sw, tw, M, N, K, y, ldy, ws, wsb, None)
        assert call(a=None) == PQ_ERR_NULL
        assert call(y=None) == PQ_ERR_NULL
        assert call(fmt=pq.FMT_NVFP4, group=16) == PQ_ERR_NULL            # tensor scales missing
        assert call(fmt=pq.FMT_NVFP4, group=16, ta=FAKE, tw=FAKE, K=48) == PQ_ERR_SHAPE   # K % 32
        assert call(M=0) == PQ_ERR_SHAPE
        assert call(ldy=4) == PQ_ERR_SHAPE
        assert call(ldy=9, N=8) == PQ_ERR_SHAPE
        assert call(group=16) == PQ_ERR_FORMAT
        assert call(wsb=0) == PQ_ERR_WORKSPACE
        assert call(ws=None) == PQ_ERR_WORKSPACE
        assert call(a=C.c_void_p(0x1008)) == PQ_ERR_SHAPE


def test_workspace_sizes(lib):
    w = pq.pq_workspace_bytes
    assert w(pq.OP_QGEMM, pq.FMT_NVFP4, 16, 4608, 9216, 3072) == 0
    need = w(pq.OP_QGEMM, pq.FMT_INT4, 64, 4608, 3072, 3072)
    assert need >= (4608 + 3072) * (3072 // 64) * 2 + (4608 + 3072) * 4
    assert w(pq.OP_CALIB_MOMENTS, 0, 0, 4608, 0, 3072, 1) >= 3072 * 8
    assert w(pq.OP_CALIB_MOMENTS, 0, 0, 4608, 0, 3072, 8) >= 8 * 3072 * 8
    assert w(pq.OP_SELECT_PERM, pq.FMT_INT4, 64, 4608, 3072, 3072, 8) > 15 * 3072 * 4
    assert w(pq.OP_QUANT_ERROR, pq.FMT_INT4, 64, 100, 0, 64) >= 800
    assert w(pq.OP_QGEMM, pq.FMT_INT4, 64, 0, 0, 0) == 0
    assert w(99, 0, 0, 1, 1, 1) == 0


def test_packed_operand_validation(lib):
    ob = pq.pq_operand_bytes
    # codes + scale units + (INT) row factors, each part rounded up to 256 bytes
    assert ob(pq.FMT_INT4, 64, 4608, 3072) >= 4608 * 3072 // 2 + 4608 * (3072 // 64) * 2 + 4608 * 4
    assert ob(pq.FMT_NVFP4, 16, 4608, 3072) >= 4608 * 3072 // 2 + 4608 * (3072 // 16)
    assert ob(pq.FMT_NVFP4, 16, 4, 96) >= 2 * 4 * 32 + 3 * 4 * 2     # 96 = one and a half steps
    assert ob(pq.FMT_INT4, 64, 0, 3072) == 0 and ob(pq.FMT_INT4, 48, 8, 96) == 0 and ob(pq.FMT_NVFP4, 16, 8, 48) == 0
    f = lib.pq_pack_operand
    assert f(1, 64, None, FAKE, 8, 64, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert f(1, 64, FAKE, FAKE, 8, 64, None, 1 << 20, None) == PQ_ERR_NULL
    assert f(1, 64, FAKE, FAKE, 0, 64, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert f(0, 16, FAKE, FAKE, 8, 48, FAKE, 1 << 20, None) == PQ_ERR_SHAPE      # K % 32
    assert f(1, 48, FAKE, FAKE, 8, 96, FAKE, 1 << 20, None) == PQ_ERR_FORMAT
    assert f(1, 64, FAKE, FAKE, 8, 64, FAKE, 16, None) == PQ_ERR_WORKSPACE
    assert f(1, 64, C.c_void_p(0x1004), FAKE, 8, 64, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    g = lib.pq_qgemm_packed
    assert g(1, 64, None, None, FAKE, None, 8, 8, 64, FAKE, 8, None) == PQ_ERR_NULL
    assert g(0, 16, FAKE, None, FAKE, FAKE, 8, 8, 64, FAKE, 8, None) == PQ_ERR_NULL   # NVFP4 tensor scales
    assert g(1, 64, FAKE, None, FAKE, None, 8, 8, 64, FAKE, 4, None) == PQ_ERR_SHAPE   # ldy < N
    assert g(1, 64, FAKE, None, FAKE, None, 8, 8, 48, FAKE, 8, None) == PQ_ERR_SHAPE   # K % group
    assert g(2, 16, FAKE, None, FAKE, None, 8, 8, 64, FAKE, 8, None) == PQ_ERR_FORMAT
    gb = lib.pq_qgemm_packed_bias
    assert gb(1, 64, FAKE, None, FAKE, None, 8, 8, 64, None, FAKE, 8, None) == PQ_ERR_NULL          # no bias
    assert gb(1, 64, FAKE, None, FAKE, None, 8, 8, 64, C.c_void_p(0x1002), FAKE, 8, None) == PQ_ERR_SHAPE
    assert lib.pq_probe_mfma(0, FAKE, None, None) == PQ_ERR_SHAPE
    assert lib.pq_probe_stream(None, 16, FAKE, 0, None) == PQ_ERR_NULL
    assert lib.pq_probe_stream(FAKE, 24, FAKE, 0, None) == PQ_ERR_SHAPE


def test_select_output_error_validation(lib):
    w = lib.pq_workspace_bytes
    # the workspace holds the fp32 reference products of all batches
    assert w(pq.OP_SELECT_PERM_OUTPUT, pq.FMT_INT4, 64, 4608, 3072, 3072, 8) > 8 * 4608 * 3072 * 4
    assert w(pq.OP_SELECT_PERM_OUTPUT, pq.FMT_INT4, 64, 64, 64, 96, 1) == 0          # K % group
    assert w(pq.OP_SELECT_PERM_OUTPUT, pq.FMT_NVFP4, 16, 64, 64, 48, 1) == 0         # K % 32
    f = lib.pq_select_perm_output_error
    al = (C.c_double * 2)(0.0, 1.0)
    rep = pq._Report()
    xs = (C.c_void_p * 1)(0x1000)
    args = lambda K=64, ws=FAKE, size=1 << 30: (1, 32, FAKE, FAKE, K, xs, 1, 8, FAKE, 8, 1.0, 1.0, al, 2, 0.0, FAKE,
                                                C.byref(rep), ws, size, None)
    assert f(*args(K=48)) == PQ_ERR_SHAPE              # K % group
    assert f(1, 16, FAKE, FAKE, 48, xs, 1, 8, FAKE, 8, 1.0, 1.0, al, 2, 0.0, FAKE, C.byref(rep), FAKE, 1 << 30,
             None) == PQ_ERR_FORMAT                    # INT4 with group 16 is not offered
    assert f(0, 16, FAKE, FAKE, 48, xs, 1, 8, FAKE, 8, 1.0, 1.0, al, 2, 0.0, FAKE, C.byref(rep), FAKE, 1 << 30,
             None) == PQ_ERR_SHAPE                     # NVFP4, K = 48: not a multiple of 32
    assert f(*args(ws=None)) == PQ_ERR_WORKSPACE
    assert f(*args(size=16)) == PQ_ERR_WORKSPACE


def test_criteria_validation(lib):
    w = lib.pq_workspace_bytes
    assert w(pq.OP_CHANNEL_STATS, 0, 0, 4608, 0, 3072, 0) >= 3072 * 12 and w(pq.OP_CHANNEL_STATS, 0, 0, 0, 0, 64, 0) == 0
    assert w(pq.OP_ORDER, 0, 0, 0, 0, 3072, 0) >= 3072 * 12
    f = lib.pq_calib_channel_stats
    assert f(None, 8, 64, 64, FAKE, FAKE, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert f(FAKE, 8, 64, 64, None, None, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert f(FAKE, 8, 60, 64, FAKE, None, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert f(FAKE, 8, 64, 64, FAKE, None, FAKE, 8, None) == PQ_ERR_WORKSPACE
    s = lib.pq_channel_statistic
    assert s(0, None, FAKE, None, 8, 64, FAKE, None) == PQ_ERR_NULL          # variance needs the sums
    assert s(1, None, None, None, 8, 64, FAKE, None) == PQ_ERR_NULL          # absmax criterion needs absmax
    assert s(0, FAKE, FAKE, None, 0, 64, FAKE, None) == PQ_ERR_SHAPE
    assert s(7, FAKE, FAKE, FAKE, 8, 64, FAKE, None) == PQ_ERR_FORMAT
    o = lib.pq_order_by_score
    assert o(None, FAKE, 64, 0.5, FAKE, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert o(FAKE, FAKE, 64, 1.5, FAKE, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert o(FAKE, FAKE, 64, 0.5, FAKE, FAKE, 8, None) == PQ_ERR_WORKSPACE
    r = lib.pq_order_round_robin
    assert r(FAKE, 96, 64, C.c_void_p(0x2000), None) == PQ_ERR_SHAPE         # K % group
    assert r(FAKE, 64, 16, FAKE, None) == PQ_ERR_SHAPE                       # in place
    assert lib.pq_order_random(1, 64, None, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert lib.pq_order_random(1, 1 << 20, FAKE, FAKE, 1 << 30, None) == PQ_ERR_SHAPE


def test_hadamard_validation(lib):
    f = lib.pq_hadamard_reorder
    assert f(None, None, 8, 64, 64, FAKE, 64, None) == PQ_ERR_NULL
    assert f(None, FAKE, 8, 64, 64, None, 64, None) == PQ_ERR_NULL
    assert f(None, FAKE, 8, 1152, 1152, FAKE, 1152, None) == PQ_ERR_SHAPE        # 9 * 2^7: no construction
    assert b"Hadamard" in lib.pq_last_error()
    assert f(None, FAKE, 8, 64, 56, FAKE, 64, None) == PQ_ERR_SHAPE
    assert f(C.c_void_p(0x1004), FAKE, 8, 64, 64, FAKE, 64, None) == PQ_ERR_SHAPE
    g = lib.pq_hadamard_quantize_act_packed
    assert g(None, 1, 64, FAKE, 8, 64, 64, None, None, 1 << 20, None, 0, None) == PQ_ERR_NULL
    assert g(None, 0, 16, FAKE, 8, 64, 64, None, FAKE, 1 << 20, None, 0, None) == PQ_ERR_NULL
    assert g(None, 1, 64, FAKE, 8, 24, 24, None, FAKE, 1 << 20, None, 0, None) == PQ_ERR_SHAPE    # K % group
    assert g(None, 1, 64, FAKE, 8, 64, 64, None, FAKE, 16, None, 0, None) == PQ_ERR_WORKSPACE


def test_norm_validation(lib):
    def params(kind=0, perm=None, gamma=None, eps=1e-6):
        return pq.NormParams(kind, perm, gamma, None, None, 0, eps)
    f = lib.pq_norm_reorder
    ok = params()
    assert f(None, FAKE, 8, 64, 64, FAKE, 64, None) == PQ_ERR_NULL
    assert f(C.byref(ok), None, 8, 64, 64, FAKE, 64, None) == PQ_ERR_NULL
    assert f(C.byref(ok), FAKE, 8, 64, 64, None, 64, None) == PQ_ERR_NULL
    assert f(C.byref(params(kind=5)), FAKE, 8, 64, 64, FAKE, 64, None) == PQ_ERR_FORMAT
    assert f(C.byref(ok), FAKE, 0, 64, 64, FAKE, 64, None) == PQ_ERR_SHAPE
    assert f(C.byref(ok), FAKE, 8, 60, 64, FAKE, 64, None) == PQ_ERR_SHAPE          # K % 8
    assert f(C.byref(ok), FAKE, 8, 64, 56, FAKE, 64, None) == PQ_ERR_SHAPE          # ld < K
    assert f(C.byref(ok), FAKE, 8, 64, 64, FAKE, 60, None) == PQ_ERR_SHAPE          # ldy
    assert f(C.byref(params(eps=-1.0)), FAKE, 8, 64, 64, FAKE, 64, None) == PQ_ERR_SHAPE
    assert f(C.byref(params(perm=0x1004)), FAKE, 8, 64, 64, FAKE, 64, None) == PQ_ERR_SHAPE   # alignment
    d = lib.pq_dynamic_tensor_scale
    assert d(None, 8, 64, 64, FAKE, None) == PQ_ERR_NULL and d(FAKE, 8, 64, 64, None, None) == PQ_ERR_NULL
    assert d(FAKE, 8, 60, 64, FAKE, None) == PQ_ERR_SHAPE and d(FAKE, 8, 64, 56, FAKE, None) == PQ_ERR_SHAPE
    g = lib.pq_norm_quantize_act_packed
    assert g(C.byref(ok), 1, 64, FAKE, 8, 64, 64, None, None, 1 << 20, None, 0, None) == PQ_ERR_NULL
    assert g(C.byref(ok), 0, 16, FAKE, 8, 64, 64, None, FAKE, 1 << 20, None, 0, None) == PQ_ERR_NULL   # NVFP4 scale
    assert g(C.byref(ok), 1, 48, FAKE, 8, 96, 96, None, FAKE, 1 << 20, None, 0, None) == PQ_ERR_FORMAT
    assert g(C.byref(ok), 0, 16, FAKE, 8, 48, 48, FAKE, FAKE, 1 << 20, None, 0, None) == PQ_ERR_SHAPE   # K % 32
    assert g(C.byref(ok), 1, 64, FAKE, 8, 64, 64, None, FAKE, 16, None, 0, None) == PQ_ERR_WORKSPACE
    assert b"operand buffer" in lib.pq_last_error()


def test_int3_dense_validation(lib):
    db = pq.pq_int3_dense_bytes
    assert db(12288, 3072) == 12288 * 3072 * 3 // 8
    assert db(1, 32) == 12
    assert db(0, 64) == 0 and db(4, 40) == 0 and db(4, 0) == 0 and db(-1, 64) == 0
    for f in (lib.pq_int3_pack, lib.pq_int3_unpack):
        assert f(None, 8, 64, FAKE, None) == PQ_ERR_NULL
        assert f(FAKE, 8, 64, None, None) == PQ_ERR_NULL
        assert f(FAKE, 0, 64, FAKE, None) == PQ_ERR_SHAPE
        assert f(FAKE, 8, 40, FAKE, None) == PQ_ERR_SHAPE          # K % 32
        assert f(FAKE, 8, 0, FAKE, None) == PQ_ERR_SHAPE
        assert f(FAKE, (1 << 24) + 1, 64, FAKE, None) == PQ_ERR_SHAPE
        assert f(C.c_void_p(0x1004), 8, 64, FAKE, None) == PQ_ERR_SHAPE
        assert f(FAKE, 8, 64, C.c_void_p(0x1008), None) == PQ_ERR_SHAPE
        assert "pq_int3_" in pq.pq_last_error()
    p = lib.pq_pack_operand_int3
    assert p(32, None, FAKE, 8, 64, FAKE, 1 << 20, None) == PQ_ERR_NULL
    assert p(32, FAKE, FAKE, 8, 64, None, 1 << 20, None) == PQ_ERR_NULL
    assert p(48, FAKE, FAKE, 8, 96, FAKE, 1 << 20, None) == PQ_ERR_FORMAT
    assert p(32, FAKE, FAKE, 0, 64, FAKE, 1 << 20, None) == PQ_ERR_SHAPE
    assert p(32, FAKE, FAKE, 8, 64, FAKE, 16, None) == PQ_ERR_WORKSPACE
    assert "pq_pack_operand_int3" in pq.pq_last_error()


def test_header_is_plain_c_and_links(tmp_path, lib):
    """include/permuquant.h compiles as C99 without a HIP or C++ header in sight, and a C program linked
    against the library reaches the host-side argument checks."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_pq.c"
    src.write_text(
        '#include <stdio.h>\n'
        '#include "permuquant.h"\n'
        'int main(void) {\n'
        '  int rc = pq_quantize_act(PQ_FMT_INT4, 64, NULL, 8, 64, 64, NULL, NULL, NULL, NULL, NULL);\n'
        '  printf("%d %d %s\\n", pq_version(), rc, pq_last_error());\n'
        '  return rc == PQ_ERR_NULL ? 0 : 1;\n'
        '}\n')
    exe = tmp_path / "use_pq"
    libdir = os.path.dirname(pq.lib_path())
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
           "-L", libdir, "-lpermuquant", "-Wl,-rpath," + libdir, "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "NULL" in r.stdout
