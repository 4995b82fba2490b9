"""Thin Python binding of the C-ABI library (include/permuquant.h).

Argument marshalling only: every step of the path runs inside the library's HIP kernels.
torch tensors provide device memory and the current stream; nothing is computed here and
there is no CPU fallback -- if the library cannot be loaded the first call raises.
Functions carry the names of the C entry points.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

FMT_NVFP4, FMT_INT4, FMT_INT3 = 0, 1, 2
OP_CALIB_MOMENTS, OP_SELECT_PERM, OP_QUANTIZE_WEIGHTS, OP_QUANTIZE_ACT, OP_QGEMM, OP_QUANT_ERROR, \
    OP_SELECT_PERM_OUTPUT, OP_CHANNEL_STATS, OP_ORDER = range(9)
CRIT_VARIANCE, CRIT_ABSMAX = 0, 1
MAX_ALPHAS = 15
DEFAULT_ALPHAS = (0.0, 0.2, 0.4, 0.6, 0.8, 1.0)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libpermuquant.so")
_lib = None


class PQError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("permuquant error %d: %s" % (code, msg))
        self.code = code


class _Report(C.Structure):
    _fields_ = [("accepted", C.c_int), ("alpha_index", C.c_int), ("e_orig", C.c_double),
                ("e_best", C.c_double), ("e_cand", C.c_double * MAX_ALPHAS),
                ("sum_x2", C.c_double), ("sum_w2", C.c_double)]


class NormParams(C.Structure):
    """pq_norm_params of the header."""
    _fields_ = [("kind", C.c_int), ("perm", C.c_void_p), ("gamma", C.c_void_p), ("mod_scale", C.c_void_p),
                ("mod_shift", C.c_void_p), ("rows_per_mod", C.c_int64), ("eps", C.c_float)]


NORM_RMS, NORM_ADALN = 0, 1


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libpermuquant.so (built in-tree by paper_2605_09503_amd.build). Raises if missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PQError(-100, "library not built: %s (run python -m paper_2605_09503_amd.build)" % _LIB_PATH)
    lib = C.CDLL(_LIB_PATH)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    lib.pq_last_error.restype = C.c_char_p
    lib.pq_last_error.argtypes = []
    lib.pq_version.restype = i32
    lib.pq_workspace_bytes.restype = sz
    lib.pq_workspace_bytes.argtypes = [i32, i32, i32, i64, i64, i64, i32]
    lib.pq_calib_moments.argtypes = [vp, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.pq_calib_moments_static.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    lib.pq_calib_moments_batched.argtypes = [C.POINTER(vp), i32, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.pq_tensor_scale.argtypes = [vp, vp, vp]
    lib.pq_tensor_scale.restype = i32
    lib.pq_select_perm.argtypes = [i32, i32, vp, vp, i64, C.POINTER(vp), i32, i64, vp, i64,
                                   C.c_float, C.c_float, C.POINTER(C.c_double), i32, C.c_double,
                                   vp, C.POINTER(_Report), vp, sz, vp]
    lib.pq_select_perm_output_error.argtypes = lib.pq_select_perm.argtypes
    lib.pq_select_perm_device_scales.argtypes = [i32, i32, vp, vp, i64, C.POINTER(vp), i32, i64, vp, i64,
                                                 vp, vp, C.POINTER(C.c_double), i32, C.c_double,
                                                 vp, C.POINTER(_Report), vp, sz, vp]
    lib.pq_quant_error.argtypes = [i32, i32, vp, i64, i64, vp, C.c_float, vp, vp, sz, vp]
    lib.pq_quantize_weights.argtypes = [i32, i32, vp, i64, i64, vp, vp, vp, vp, vp]
    lib.pq_quantize_act.argtypes = [i32, i32, vp, i64, i64, i64, vp, vp, vp, vp, vp]
    gemm_args = [i32, i32, vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, i64, vp, sz, vp]
    lib.pq_qgemm.argtypes = gemm_args
    lib.pq_qgemm_f32.argtypes = gemm_args
    lib.pq_qgemm_run.argtypes = gemm_args
    lib.pq_qgemm_prep.argtypes = [i32, i32, vp, vp, i64, i64, i64, vp, sz, vp]
    lib.pq_operand_bytes.restype = sz
    lib.pq_operand_bytes.argtypes = [i32, i32, i64, i64]
    lib.pq_pack_operand.argtypes = [i32, i32, vp, vp, i64, i64, vp, sz, vp]
    lib.pq_quantize_act_packed.argtypes = [i32, i32, vp, i64, i64, i64, vp, vp, sz, vp, vp, vp]
    lib.pq_int3_dense_bytes.restype = sz
    lib.pq_int3_dense_bytes.argtypes = [i64, i64]
    lib.pq_int3_pack.argtypes = [vp, i64, i64, vp, vp]
    lib.pq_int3_unpack.argtypes = [vp, i64, i64, vp, vp]
    lib.pq_pack_operand_int3.argtypes = [i32, vp, vp, i64, i64, vp, sz, vp]
    packed_args = [i32, i32, vp, vp, vp, vp, i64, i64, i64, vp, i64, vp]
    lib.pq_qgemm_packed.argtypes = packed_args
    lib.pq_qgemm_packed_f32.argtypes = packed_args
    lib.pq_qgemm_packed_bias.argtypes = [i32, i32, vp, vp, vp, vp, i64, i64, i64, vp, vp, i64, vp]
    lib.pq_calib_channel_stats.argtypes = [vp, i64, i64, i64, vp, vp, vp, sz, vp]
    lib.pq_channel_statistic.argtypes = [i32, vp, vp, vp, i64, i64, vp, vp]
    lib.pq_order_by_score.argtypes = [vp, vp, i64, C.c_double, vp, vp, sz, vp]
    lib.pq_order_round_robin.argtypes = [vp, i64, i32, vp, vp]
    lib.pq_order_random.argtypes = [C.c_uint64, i64, vp, vp, sz, vp]
    lib.pq_hadamard_reorder.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
    lib.pq_hadamard_quantize_act_packed.argtypes = [vp, i32, i32, vp, i64, i64, i64, vp, vp, sz, vp, i64, vp]
    lib.pq_dynamic_tensor_scale.argtypes = [vp, i64, i64, i64, vp, vp]
    lib.pq_norm_reorder.argtypes = [C.POINTER(NormParams), vp, i64, i64, i64, vp, i64, vp]
    lib.pq_norm_quantize_act_packed.argtypes = [C.POINTER(NormParams), i32, i32, vp, i64, i64, i64, vp, vp, sz,
                                                vp, i64, vp]
    lib.pq_probe_stream.argtypes = [vp, sz, vp, sz, vp]
    lib.pq_qgemm_check_int_scales.argtypes = [i32, i32, vp, i64, i64, C.POINTER(C.c_int64), vp, sz, vp]
    lib.pq_probe_mfma.argtypes = [i32, vp, C.POINTER(C.c_double), vp]
    lib.pq_probe_mfma_operands.argtypes = [i32, i32, vp, vp, i64, i64, i64, i32, vp, C.POINTER(C.c_double), vp]
    for name in ("pq_calib_moments", "pq_calib_moments_batched", "pq_select_perm", "pq_quant_error", "pq_quantize_weights",
                 "pq_quantize_act", "pq_qgemm", "pq_qgemm_f32", "pq_qgemm_run", "pq_qgemm_prep", "pq_probe_stream",
                 "pq_probe_mfma", "pq_pack_operand", "pq_qgemm_packed", "pq_qgemm_packed_f32",
                 "pq_quantize_act_packed"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise PQError(rc, load().pq_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def pq_last_error() -> str:
    return load().pq_last_error().decode()


def pq_version() -> int:
    return load().pq_version()


def pq_workspace_bytes(op: int, fmt: int, group: int, M: int, N: int, K: int, n_batches: int = 0) -> int:
    return int(load().pq_workspace_bytes(op, fmt, group, M, N, K, n_batches))


def _workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def pq_calib_moments(x: torch.Tensor, sumsq: torch.Tensor, absmax: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, rows: Optional[int] = None,
                     K: Optional[int] = None, ld: Optional[int] = None) -> None:
    """sumsq[K] (float64, in/out) += column sums of squares of bf16 x[rows, ld]."""
    rows = x.shape[0] if rows is None else rows
    K = x.shape[1] if K is None else K
    ld = x.stride(0) if ld is None else ld
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(OP_CALIB_MOMENTS, 0, 0, rows, 0, K, 1), x.device)
    _check(load().pq_calib_moments(_ptr(x), rows, K, ld, _ptr(sumsq), _ptr(absmax), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream()))


STATIC_SCRATCH_BYTES = 3 << 20      # PQ_STATIC_SCRATCH_BYTES of the header


def pq_calib_moments_static(x: torch.Tensor, sumsq: torch.Tensor, absmax: Optional[torch.Tensor] = None,
                            rows: Optional[int] = None, K: Optional[int] = None,
                            ld: Optional[int] = None) -> None:
    """pq_calib_moments with the partial sums in scratch memory the library holds itself: the call
    takes no workspace and allocates nothing."""
    rows = x.shape[0] if rows is None else rows
    K = x.shape[1] if K is None else K
    ld = x.stride(0) if ld is None else ld
    _check(load().pq_calib_moments_static(_ptr(x), rows, K, ld, _ptr(sumsq), _ptr(absmax), _stream()))


def pq_calib_moments_batched(xs: Sequence[torch.Tensor], sumsq: torch.Tensor,
                             absmax: Optional[torch.Tensor] = None,
                             workspace: Optional[torch.Tensor] = None) -> None:
    """sumsq[K] += column sums of squares over all batches (equal shapes), one launch."""
    rows, K = xs[0].shape
    ld = xs[0].stride(0)
    nb = len(xs)
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(OP_CALIB_MOMENTS, 0, 0, rows, 0, K, nb), xs[0].device)
    ptrs = (C.c_void_p * nb)(*[x.data_ptr() for x in xs])
    _check(load().pq_calib_moments_batched(ptrs, nb, rows, K, ld, _ptr(sumsq), _ptr(absmax), _ptr(workspace),
                                           0 if workspace is None else workspace.numel(), _stream()))


def pq_tensor_scale(absmax: torch.Tensor, tensor_scale_out: torch.Tensor) -> None:
    """NVFP4 per-tensor scale T = fl32(absmax / 2688), computed on the device."""
    _check(load().pq_tensor_scale(_ptr(absmax), _ptr(tensor_scale_out), _stream()))


@dataclass
class SelectReport:
    accepted: bool
    alpha_index: int
    e_orig: float
    e_best: float
    e_cand: List[float]
    sum_x2: float
    sum_w2: float


def _select(entry: str, op: int, fmt, group, act_sumsq, w_sumsq, x_calib, w, act_tensor_scale, w_tensor_scale,
            perm_out, alphas, tau, workspace) -> SelectReport:
    M, K = x_calib[0].shape
    N = w.shape[0]
    nb = len(x_calib)
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(op, fmt, group, M, N, K, nb), w.device)
    ptrs = (C.c_void_p * nb)(*[xb.data_ptr() for xb in x_calib])
    al = (C.c_double * len(alphas))(*[float(a) for a in alphas])
    rep = _Report()
    if entry == "pq_select_perm_device_scales":
        ta, tw = _ptr(act_tensor_scale), _ptr(w_tensor_scale)
    else:
        ta, tw = float(act_tensor_scale), float(w_tensor_scale)
    _check(getattr(load(), entry)(fmt, group, _ptr(act_sumsq), _ptr(w_sumsq), K, ptrs, nb, M, _ptr(w), N,
                                  ta, tw, al, len(alphas),
                                  float(tau), _ptr(perm_out), C.byref(rep), _ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream()))
    return SelectReport(bool(rep.accepted), rep.alpha_index, rep.e_orig, rep.e_best,
                        [rep.e_cand[j] for j in range(len(alphas))], rep.sum_x2, rep.sum_w2)


def pq_select_perm(fmt: int, group: int, act_sumsq: torch.Tensor, w_sumsq: torch.Tensor,
                   x_calib: Sequence[torch.Tensor], w: torch.Tensor, act_tensor_scale: float,
                   w_tensor_scale: float, perm_out: torch.Tensor,
                   alphas: Sequence[float] = DEFAULT_ALPHAS, tau: float = 0.0,
                   workspace: Optional[torch.Tensor] = None) -> SelectReport:
    return _select("pq_select_perm", OP_SELECT_PERM, fmt, group, act_sumsq, w_sumsq, x_calib, w,
                   act_tensor_scale, w_tensor_scale, perm_out, alphas, tau, workspace)


def pq_select_perm_device_scales(fmt: int, group: int, act_sumsq: torch.Tensor, w_sumsq: torch.Tensor,
                                 x_calib: Sequence[torch.Tensor], w: torch.Tensor,
                                 act_tensor_scale: Optional[torch.Tensor], w_tensor_scale: Optional[torch.Tensor],
                                 perm_out: torch.Tensor, alphas: Sequence[float] = DEFAULT_ALPHAS, tau: float = 0.0,
                                 workspace: Optional[torch.Tensor] = None) -> SelectReport:
    """pq_select_perm with the NVFP4 tensor scales as device floats (no host copy needed before the call)."""
    return _select("pq_select_perm_device_scales", OP_SELECT_PERM, fmt, group, act_sumsq, w_sumsq, x_calib, w,
                   act_tensor_scale, w_tensor_scale, perm_out, alphas, tau, workspace)


def pq_select_perm_output_error(fmt: int, group: int, act_sumsq: torch.Tensor, w_sumsq: torch.Tensor,
                                x_calib: Sequence[torch.Tensor], w: torch.Tensor, act_tensor_scale: float,
                                w_tensor_scale: float, perm_out: torch.Tensor,
                                alphas: Sequence[float] = DEFAULT_ALPHAS, tau: float = 0.0,
                                workspace: Optional[torch.Tensor] = None) -> SelectReport:
    """The selection with the relative error of the layer's output as the metric."""
    return _select("pq_select_perm_output_error", OP_SELECT_PERM_OUTPUT, fmt, group, act_sumsq, w_sumsq, x_calib, w,
                   act_tensor_scale, w_tensor_scale, perm_out, alphas, tau, workspace)


def pq_quant_error(fmt: int, group: int, x: torch.Tensor, perm: Optional[torch.Tensor],
                   tensor_scale: float, err_out: torch.Tensor,
                   workspace: Optional[torch.Tensor] = None) -> None:
    rows, K = x.shape
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(OP_QUANT_ERROR, fmt, group, rows, 0, K), x.device)
    _check(load().pq_quant_error(fmt, group, _ptr(x), rows, K, _ptr(perm), float(tensor_scale),
                                 _ptr(err_out), _ptr(workspace),
                                 0 if workspace is None else workspace.numel(), _stream()))


def pq_quantize_weights(fmt: int, group: int, w: torch.Tensor, perm: Optional[torch.Tensor],
                        codes: torch.Tensor, scales: torch.Tensor, tensor_scale_out: torch.Tensor) -> None:
    N, K = w.shape
    _check(load().pq_quantize_weights(fmt, group, _ptr(w), N, K, _ptr(perm), _ptr(codes), _ptr(scales),
                                      _ptr(tensor_scale_out), _stream()))


def pq_quantize_act(fmt: int, group: int, x: torch.Tensor, perm: Optional[torch.Tensor],
                    tensor_scale: Optional[torch.Tensor], codes: torch.Tensor, scales: torch.Tensor,
                    M: Optional[int] = None, K: Optional[int] = None, ld: Optional[int] = None) -> None:
    M = x.shape[0] if M is None else M
    K = x.shape[1] if K is None else K
    ld = x.stride(0) if ld is None else ld
    _check(load().pq_quantize_act(fmt, group, _ptr(x), M, K, ld, _ptr(perm), _ptr(tensor_scale),
                                  _ptr(codes), _ptr(scales), _stream()))


def _gemm(fn, fmt, group, a_codes, a_scales, a_ts, w_codes, w_scales, w_ts, y, workspace, M, N, K, ldy):
    M = a_codes.shape[0] if M is None else M
    K = a_codes.shape[1] * 2 if K is None else K
    N = w_codes.shape[0] if N is None else N
    ldy = y.stride(0) if ldy is None else ldy
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(OP_QGEMM, fmt, group, M, N, K), a_codes.device)
    _check(fn(fmt, group, _ptr(a_codes), _ptr(a_scales), _ptr(a_ts), _ptr(w_codes), _ptr(w_scales),
              _ptr(w_ts), M, N, K, _ptr(y), ldy, _ptr(workspace),
              0 if workspace is None else workspace.numel(), _stream()))


def pq_qgemm(fmt: int, group: int, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
             w_tensor_scale, y: torch.Tensor, workspace: Optional[torch.Tensor] = None,
             M=None, N=None, K=None, ldy=None) -> None:
    """y[M, N] (bf16) = dequant(A) @ dequant(W)^T."""
    _gemm(load().pq_qgemm, fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
          w_tensor_scale, y, workspace, M, N, K, ldy)


def pq_qgemm_prep(fmt: int, group: int, a_scales, w_scales, M: int, N: int, K: int,
                  workspace: Optional[torch.Tensor]) -> None:
    """Scale preparation half of pq_qgemm (INT formats; no-op for NVFP4)."""
    _check(load().pq_qgemm_prep(fmt, group, _ptr(a_scales), _ptr(w_scales), M, N, K, _ptr(workspace),
                                0 if workspace is None else workspace.numel(), _stream()))


def pq_qgemm_run(fmt: int, group: int, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                 w_tensor_scale, y: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                 M=None, N=None, K=None, ldy=None) -> None:
    """Product half of pq_qgemm: the workspace must have been filled by pq_qgemm_prep."""
    _gemm(load().pq_qgemm_run, fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
          w_tensor_scale, y, workspace, M, N, K, ldy)


def pq_qgemm_f32(fmt: int, group: int, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                 w_tensor_scale, y: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                 M=None, N=None, K=None, ldy=None) -> None:
    """Same product, fp32 output (accumulator before the bf16 rounding)."""
    _gemm(load().pq_qgemm_f32, fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
          w_tensor_scale, y, workspace, M, N, K, ldy)


def pq_operand_bytes(fmt: int, group: int, rows: int, K: int) -> int:
    return int(load().pq_operand_bytes(fmt, group, rows, K))


def pq_pack_operand(fmt: int, group: int, codes: torch.Tensor, scales: torch.Tensor,
                    operand: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Stored quantizer output -> the GEMM's panel layout (allocates the buffer unless given)."""
    rows, K = codes.shape[0], codes.shape[1] * 2
    if operand is None:
        operand = torch.empty(max(pq_operand_bytes(fmt, group, rows, K), 16), dtype=torch.uint8, device=codes.device)
    _check(load().pq_pack_operand(fmt, group, _ptr(codes), _ptr(scales), rows, K, _ptr(operand),
                                  operand.numel(), _stream()))
    return operand


def pq_int3_dense_bytes(rows: int, K: int) -> int:
    return int(load().pq_int3_dense_bytes(rows, K))


def pq_int3_pack(codes: torch.Tensor, dense: Optional[torch.Tensor] = None) -> torch.Tensor:
    """INT3 codes in nibbles [rows, K/2] -> dense 3-bit storage [rows, 3K/8] (allocates unless given)."""
    rows, K = codes.shape[0], codes.shape[1] * 2
    if dense is None:
        dense = torch.empty((rows, K // 8 * 3), dtype=torch.uint8, device=codes.device)
    _check(load().pq_int3_pack(_ptr(codes), rows, K, _ptr(dense), _stream()))
    return dense


def pq_int3_unpack(dense: torch.Tensor, K: int, codes: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Dense 3-bit storage [rows, 3K/8] -> nibbles [rows, K/2] (allocates unless given)."""
    rows = dense.shape[0]
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=dense.device)
    _check(load().pq_int3_unpack(_ptr(dense), rows, K, _ptr(codes), _stream()))
    return codes


def pq_pack_operand_int3(group: int, dense: torch.Tensor, scales: torch.Tensor, K: int,
                         operand: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Dense 3-bit codes + scales -> the GEMM's panel layout (allocates the buffer unless given)."""
    rows = dense.shape[0]
    if operand is None:
        operand = torch.empty(max(pq_operand_bytes(FMT_INT3, group, rows, K), 16), dtype=torch.uint8,
                              device=dense.device)
    _check(load().pq_pack_operand_int3(group, _ptr(dense), _ptr(scales), rows, K, _ptr(operand),
                                       operand.numel(), _stream()))
    return operand


def pq_quantize_act_packed(fmt: int, group: int, x: torch.Tensor, tensor_scale: Optional[torch.Tensor],
                           operand: Optional[torch.Tensor] = None, codes: Optional[torch.Tensor] = None,
                           scales: Optional[torch.Tensor] = None, K: Optional[int] = None) -> torch.Tensor:
    """Dynamic activation quantization straight into the GEMM's panel layout."""
    M = x.shape[0]
    K = x.shape[1] if K is None else K
    if operand is None:
        operand = torch.empty(max(pq_operand_bytes(fmt, group, M, K), 16), dtype=torch.uint8, device=x.device)
    _check(load().pq_quantize_act_packed(fmt, group, _ptr(x), M, K, x.stride(0), _ptr(tensor_scale),
                                         _ptr(operand), operand.numel(), _ptr(codes), _ptr(scales), _stream()))
    return operand


def pq_calib_channel_stats(x: torch.Tensor, total: Optional[torch.Tensor], absmax: Optional[torch.Tensor],
                           K: Optional[int] = None, workspace: Optional[torch.Tensor] = None) -> None:
    """Per channel: sum (fp64, accumulated into `total`) and largest magnitude (fp32, max into `absmax`)."""
    rows = x.shape[0]
    K = x.shape[1] if K is None else K
    if workspace is None:
        workspace = _workspace(pq_workspace_bytes(OP_CHANNEL_STATS, 0, 0, rows, 0, K), x.device)
    _check(load().pq_calib_channel_stats(_ptr(x), rows, K, x.stride(0), _ptr(total), _ptr(absmax), _ptr(workspace),
                                         workspace.numel(), _stream()))


def pq_channel_statistic(kind: int, total, sumsq, absmax, n_rows: int, out: torch.Tensor) -> torch.Tensor:
    _check(load().pq_channel_statistic(kind, _ptr(total), _ptr(sumsq), _ptr(absmax), n_rows, out.numel(), _ptr(out),
                                       _stream()))
    return out


def _order_ws(K: int, device, workspace):
    return workspace if workspace is not None else _workspace(pq_workspace_bytes(OP_ORDER, 0, 0, 0, 0, K), device)


def pq_order_by_score(act_stat: torch.Tensor, w_stat: torch.Tensor, alpha: float, perm_out: torch.Tensor,
                      workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    K = act_stat.numel()
    ws = _order_ws(K, act_stat.device, workspace)
    _check(load().pq_order_by_score(_ptr(act_stat), _ptr(w_stat), K, float(alpha), _ptr(perm_out), _ptr(ws),
                                    ws.numel(), _stream()))
    return perm_out


def pq_order_round_robin(order: torch.Tensor, group: int, perm_out: torch.Tensor) -> torch.Tensor:
    _check(load().pq_order_round_robin(_ptr(order), order.numel(), group, _ptr(perm_out), _stream()))
    return perm_out


def pq_order_random(seed: int, perm_out: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    K = perm_out.numel()
    ws = _order_ws(K, perm_out.device, workspace)
    _check(load().pq_order_random(int(seed), K, _ptr(perm_out), _ptr(ws), ws.numel(), _stream()))
    return perm_out


def pq_dynamic_tensor_scale(x: torch.Tensor, tensor_scale_out: Optional[torch.Tensor] = None,
                            K: Optional[int] = None) -> torch.Tensor:
    """T = max|x| / 2688 of the live tensor, left on the device (first pass of a dynamic NVFP4 scale)."""
    if tensor_scale_out is None:
        tensor_scale_out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(load().pq_dynamic_tensor_scale(_ptr(x), x.shape[0], x.shape[1] if K is None else K, x.stride(0),
                                          _ptr(tensor_scale_out), _stream()))
    return tensor_scale_out


def _norm_params(kind, perm, gamma, mod_scale, mod_shift, rows_per_mod, eps) -> "NormParams":
    raw = [None if t is None else t.data_ptr() for t in (perm, gamma, mod_scale, mod_shift)]
    return NormParams(int(kind), raw[0], raw[1], raw[2], raw[3], int(rows_per_mod), float(eps))


def pq_norm_reorder(kind: int, x: torch.Tensor, eps: float, perm: Optional[torch.Tensor] = None,
                    gamma: Optional[torch.Tensor] = None, mod_scale: Optional[torch.Tensor] = None,
                    mod_shift: Optional[torch.Tensor] = None, rows_per_mod: int = 0,
                    y: Optional[torch.Tensor] = None, K: Optional[int] = None) -> torch.Tensor:
    """RMSNorm / modulated LayerNorm whose output comes out in the channel order `perm` (bf16 [M, K])."""
    M = x.shape[0]
    K = x.shape[1] if K is None else K
    if y is None:
        y = torch.empty((M, K), dtype=torch.bfloat16, device=x.device)
    p = _norm_params(kind, perm, gamma, mod_scale, mod_shift, rows_per_mod, eps)
    _check(load().pq_norm_reorder(C.byref(p), _ptr(x), M, K, x.stride(0), _ptr(y), y.stride(0), _stream()))
    return y


def pq_norm_quantize_act_packed(kind: int, fmt: int, group: int, x: torch.Tensor, eps: float,
                                tensor_scale: Optional[torch.Tensor], perm: Optional[torch.Tensor] = None,
                                gamma: Optional[torch.Tensor] = None, mod_scale: Optional[torch.Tensor] = None,
                                mod_shift: Optional[torch.Tensor] = None, rows_per_mod: int = 0,
                                operand: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None,
                                K: Optional[int] = None) -> torch.Tensor:
    """The same layer feeding the activation quantizer directly: returns the GEMM operand."""
    M = x.shape[0]
    K = x.shape[1] if K is None else K
    if operand is None:
        operand = torch.empty(max(pq_operand_bytes(fmt, group, M, K), 16), dtype=torch.uint8, device=x.device)
    p = _norm_params(kind, perm, gamma, mod_scale, mod_shift, rows_per_mod, eps)
    _check(load().pq_norm_quantize_act_packed(C.byref(p), fmt, group, _ptr(x), M, K, x.stride(0),
                                              _ptr(tensor_scale), _ptr(operand), operand.numel(), _ptr(y),
                                              0 if y is None else y.stride(0), _stream()))
    return operand


def pq_hadamard_reorder(x: torch.Tensor, perm: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None,
                        K: Optional[int] = None) -> torch.Tensor:
    """x H with the columns of the result in the order `perm` (bf16 [M, K])."""
    M = x.shape[0]
    K = x.shape[1] if K is None else K
    if y is None:
        y = torch.empty((M, K), dtype=torch.bfloat16, device=x.device)
    _check(load().pq_hadamard_reorder(_ptr(perm), _ptr(x), M, K, x.stride(0), _ptr(y), y.stride(0), _stream()))
    return y


def pq_hadamard_quantize_act_packed(fmt: int, group: int, x: torch.Tensor, tensor_scale: Optional[torch.Tensor],
                                    perm: Optional[torch.Tensor] = None, operand: Optional[torch.Tensor] = None,
                                    y: Optional[torch.Tensor] = None, K: Optional[int] = None) -> torch.Tensor:
    """The rotation feeding the activation quantizer directly: returns the GEMM operand."""
    M = x.shape[0]
    K = x.shape[1] if K is None else K
    if operand is None:
        operand = torch.empty(max(pq_operand_bytes(fmt, group, M, K), 16), dtype=torch.uint8, device=x.device)
    _check(load().pq_hadamard_quantize_act_packed(_ptr(perm), fmt, group, _ptr(x), M, K, x.stride(0),
                                                  _ptr(tensor_scale), _ptr(operand), operand.numel(), _ptr(y),
                                                  0 if y is None else y.stride(0), _stream()))
    return operand


def _gemm_packed(fn, fmt, group, a_operand, a_ts, w_operand, w_ts, y, M, N, K, ldy):
    _check(fn(fmt, group, _ptr(a_operand), _ptr(a_ts), _ptr(w_operand), _ptr(w_ts), M, N, K, _ptr(y),
              y.stride(0) if ldy is None else ldy, _stream()))


def pq_qgemm_packed(fmt: int, group: int, a_operand, a_tensor_scale, w_operand, w_tensor_scale,
                    y: torch.Tensor, M: int, N: int, K: int, ldy=None) -> None:
    _gemm_packed(load().pq_qgemm_packed, fmt, group, a_operand, a_tensor_scale, w_operand, w_tensor_scale,
                 y, M, N, K, ldy)


def pq_qgemm_packed_bias(fmt: int, group: int, a_operand, a_tensor_scale, w_operand, w_tensor_scale,
                         bias: torch.Tensor, y: torch.Tensor, M: int, N: int, K: int, ldy=None) -> None:
    """The packed product plus the layer's bias (bf16 [N]), added before the rounding to bf16."""
    _check(load().pq_qgemm_packed_bias(fmt, group, _ptr(a_operand), _ptr(a_tensor_scale), _ptr(w_operand),
                                       _ptr(w_tensor_scale), M, N, K, _ptr(bias), _ptr(y),
                                       y.stride(0) if ldy is None else ldy, _stream()))


def pq_qgemm_packed_f32(fmt: int, group: int, a_operand, a_tensor_scale, w_operand, w_tensor_scale,
                        y: torch.Tensor, M: int, N: int, K: int, ldy=None) -> None:
    _gemm_packed(load().pq_qgemm_packed_f32, fmt, group, a_operand, a_tensor_scale, w_operand,
                 w_tensor_scale, y, M, N, K, ldy)


def pq_probe_stream(src: torch.Tensor, read_bytes: int, dst: torch.Tensor, write_bytes: int) -> None:
    """Plain streaming kernel: reads read_bytes of src, writes write_bytes of dst."""
    _check(load().pq_probe_stream(_ptr(src), read_bytes, _ptr(dst), write_bytes, _stream()))


def pq_probe_mfma(iters: int, sink: torch.Tensor) -> float:
    """Matrix-pipe-only loop on every compute unit; returns the floating-point operations issued."""
    flops = C.c_double(0.0)
    _check(load().pq_probe_mfma(iters, _ptr(sink), C.byref(flops), _stream()))
    return flops.value


def pq_qgemm_check_int_scales(fmt: int, group: int, scales: torch.Tensor, rows: int, K: int) -> int:
    """Number of INT group scales the product kernel would not reproduce exactly (synchronises)."""
    ws = torch.empty(256, dtype=torch.uint8, device=scales.device)
    bad = C.c_int64(-1)
    _check(load().pq_qgemm_check_int_scales(fmt, group, _ptr(scales), rows, K, C.byref(bad), _ptr(ws), ws.numel(),
                                            _stream()))
    return bad.value


def pq_probe_mfma_operands(fmt: int, group: int, a_operand: torch.Tensor, w_operand: torch.Tensor, M: int, N: int,
                           K: int, iters: int, sink: torch.Tensor) -> float:
    """Matrix-pipe-only loop on fragments of the two packed operands; returns the operations issued."""
    flops = C.c_double(0.0)
    _check(load().pq_probe_mfma_operands(fmt, group, _ptr(a_operand), _ptr(w_operand), M, N, K, iters, _ptr(sink),
                                         C.byref(flops), _stream()))
    return flops.value


# ------------------------------------------------------------------------ allocation helpers
def scale_dtype(fmt: int):
    return torch.uint8 if fmt == FMT_NVFP4 else torch.float32


def alloc_quantized(fmt: int, group: int, rows: int, K: int, device="cuda"):
    """(codes, scales) buffers in the stored layout."""
    codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=device)
    scales = torch.empty((rows, K // group), dtype=scale_dtype(fmt), device=device)
    return codes, scales


def bf16_from_bits(bits_u16, device="cuda") -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 tensor on the device (no value conversion)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16))
    return t.to(device).view(torch.bfloat16)
