#!/usr/bin/env python3
"""Benchmark of the per-group-quantized linear layer on one MI355X.

A step is one pass of the whole hot path over one synthetic layer:
  calibration moments of every calibration batch and of W -> permutation selection ->
  weight quantization in the selected order (+ packing into the GEMM's operand layout) ->
  dynamic activation quantization of one token batch (straight into that layout) ->
  low-bit GEMM with bf16 output.
Inputs are generated once (seeded, synthetic, FLUX-DiT-shaped) and are resident in HBM before
the timed region.  One JSON line goes to stdout; everything else goes to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config all|c0|c1|c2|c3|c3up|c3down|c4]

Without --config every FLUX-shaped configuration runs in one process: the headline workload is
the NVFP4 MLP pair (c3: up and down projection, a step covers both layers), and the JSON line
carries a `configs` object with the figures of c1, c2, c3up, c3down and c4 each measured the
same way.  --config <name> runs that workload alone, with every auxiliary timing.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

import numpy as np


def log(*a):
    print(*a, file=sys.stderr, flush=True)


HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16/bf16 matrix peak

WORKLOADS = {
    "c0": "tiny NVFP4 g16 linear X[256,512] W[512,512]",
    "c1": "INT4 g64 FLUX-DiT attention-out linear X[4608,3072] W[3072,3072], 8 calibration batches",
    "c2": "NVFP4 g16 FLUX-DiT fused QKV X[4608,3072] W[9216,3072], 8 calibration batches",
    "c3up": "NVFP4 g16 FLUX-DiT MLP up X[4608,3072] W[12288,3072], 8 calibration batches",
    "c3down": "NVFP4 g16 FLUX-DiT MLP down X[4608,12288] W[3072,12288], 8 calibration batches",
    "c4": "INT3 g32 stress X[8192,3072] W[12288,3072], 8 calibration batches",
    "c3": "NVFP4 g16 FLUX-DiT MLP pair: up X[4608,3072] W[12288,3072] and down X[4608,12288] W[3072,12288], "
          "8 calibration batches each, one permutation per layer",
}
FMT_NAMES = ["nvfp4", "int4", "int3"]


def quant_bytes_per_elem(fmt, g):
    return 2.0 + 0.5 + (1.0 / 16 if fmt == 0 else 4.0 / g)


def qbytes_out(fmt, g, M, K):
    return (0.5 + (1.0 / 16 if fmt == 0 else 4.0 / g)) * M * K


def blas_threads():
    """Threads the oracle's matmul actually runs on (its elementwise steps run on one)."""
    try:
        from threadpoolctl import threadpool_info
        n = [int(p.get("num_threads", 0)) for p in threadpool_info() if p.get("user_api") in ("blas", "openmp")]
        if n and max(n) > 0:
            return max(n)
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", 0)) or os.cpu_count()


class Layer:
    """One linear layer of a configuration: its synthetic tensors on the device, every buffer the
    path needs (allocated once; the timed region allocates nothing) and the calls of one step."""

    def __init__(self, name, torch, pq, synth, dev):
        self.name, self.torch, self.pq, self.dev = name, torch, pq, dev
        cfg = self.cfg = synth.CONFIGS[name]
        fmt, g, M, N, K, nb = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K, cfg.n_calib
        self.flops = 2.0 * M * N * K
        t0 = time.perf_counter()
        self.st = synth.make_struct(cfg)
        with cf.ThreadPoolExecutor(max_workers=min(9, os.cpu_count() or 1)) as ex:   # numpy releases the GIL
            bits = list(ex.map(lambda b: synth.make_batch(self.st, b), range(nb + 1)))
        self.calib_bits, self.test_bits = bits[:nb], bits[nb]
        log("%s: synthetic inputs generated in %.1f s" % (name, time.perf_counter() - t0))
        self.xs = [pq.bf16_from_bits(b, dev) for b in self.calib_bits]
        self.w = pq.bf16_from_bits(self.st.w_bits, dev)
        x_test = pq.bf16_from_bits(self.test_bits, dev)
        self.sa = torch.zeros(K, dtype=torch.float64, device=dev)
        self.sw = torch.zeros(K, dtype=torch.float64, device=dev)
        self.amax_a = torch.zeros(1, dtype=torch.float32, device=dev)
        self.amax_w = torch.zeros(1, dtype=torch.float32, device=dev)
        self.ts_a = torch.ones(1, dtype=torch.float32, device=dev)
        self.ts_w = torch.ones(1, dtype=torch.float32, device=dev)
        self.perm = torch.empty(K, dtype=torch.int32, device=dev)
        self.a_codes, self.a_scales = pq.alloc_quantized(fmt, g, M, K, dev)
        self.w_codes, self.w_scales = pq.alloc_quantized(fmt, g, N, K, dev)
        self.y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        u8 = dict(dtype=torch.uint8, device=dev)
        self.ws_mom = torch.empty(max(pq.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, fmt, g, M, 0, K, nb),
                                      pq.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, fmt, g, N, 0, K, 1), 16), **u8)
        self.ws_sel = torch.empty(pq.pq_workspace_bytes(pq.OP_SELECT_PERM, fmt, g, M, N, K, nb), **u8)
        self.a_op = torch.empty(max(pq.pq_operand_bytes(fmt, g, M, K), 16), **u8)       # GEMM operands
        self.w_op = torch.empty(max(pq.pq_operand_bytes(fmt, g, N, K), 16), **u8)
        # the producer of the activations emits them in the selected order (the permutation is
        # folded into the previous module offline); build that input once, outside the timing
        self.rep = self.calibrate()
        torch.cuda.synchronize()
        self.x_run = x_test.index_select(1, self.perm.long()).contiguous()
        del x_test
        log("%s: selection accepted=%s alpha_index=%d E_orig=%.6g E_best=%.6g" %
            (name, self.rep.accepted, self.rep.alpha_index, self.rep.e_orig, self.rep.e_best))

    def calibrate(self):
        pq, cfg = self.pq, self.cfg
        self.sa.zero_(); self.sw.zero_(); self.amax_a.zero_(); self.amax_w.zero_()
        pq.pq_calib_moments_batched(self.xs, self.sa, self.amax_a, self.ws_mom)
        pq.pq_calib_moments(self.w, self.sw, self.amax_w, self.ws_mom)
        if cfg.fmt == pq.FMT_NVFP4:
            pq.pq_tensor_scale(self.amax_a, self.ts_a)
            pq.pq_tensor_scale(self.amax_w, self.ts_w)
        # the tensor scales stay on the device: nothing synchronises before the selection's own read-back
        return pq.pq_select_perm_device_scales(cfg.fmt, cfg.group, self.sa, self.sw, self.xs, self.w, self.ts_a,
                                               self.ts_w, self.perm, workspace=self.ws_sel)

    def prepare_weights(self):
        pq, cfg = self.pq, self.cfg
        pq.pq_quantize_weights(cfg.fmt, cfg.group, self.w, self.perm, self.w_codes, self.w_scales, self.ts_w)
        pq.pq_pack_operand(cfg.fmt, cfg.group, self.w_codes, self.w_scales, self.w_op)

    def forward(self):
        # the activation quantizer writes the GEMM's panel layout directly; the weights were packed offline
        pq, cfg = self.pq, self.cfg
        pq.pq_quantize_act_packed(cfg.fmt, cfg.group, self.x_run, self.ts_a, self.a_op)
        pq.pq_qgemm_packed(cfg.fmt, cfg.group, self.a_op, self.ts_a, self.w_op, self.ts_w, self.y, cfg.M, cfg.N, cfg.K)

    def step(self):
        self.calibrate()
        self.prepare_weights()
        self.forward()


def make_timer(torch):
    # The launches of a timing loop are captured into a graph and replayed: a Python loop issues one
    # launch per ~8 us, which would hide every kernel shorter than that behind the host.  Events are
    # recorded on the stream the graph is replayed on (torch's current stream, which is also the stream
    # the binding hands to the library).  Calls that synchronise cannot be captured and are timed eagerly.
    def time_calls(fn, iters, graph=True, warm_replays=2):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if graph:
            g_ = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_):
                for i in range(iters):
                    fn(i)
            for _ in range(warm_replays):    # untimed: first touch, and the clocks settle
                g_.replay()
            torch.cuda.synchronize()
            e0.record()
            g_.replay()
            e1.record()
        else:
            e0.record()
            for i in range(iters):
                fn(i)
            e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters            # seconds per call
    return time_calls


def timed_steps(torch, layers, steps, warmup):
    for _ in range(warmup):
        for L in layers:
            L.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for L in layers:
            L.step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def hbm(nbytes, t):
    return {"us": t * 1e6, "gbs": nbytes / t / 1e9, "frac_hbm_peak": nbytes / t / 1e9 / HBM_PEAK_GBS}


def core_kernels(L, it, time_calls):
    """Every kernel of the path on its own, with the references measured on the same inputs."""
    torch, pq, cfg, dev = L.torch, L.pq, L.cfg, L.dev
    fmt, g, M, N, K, nb = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K, cfg.n_calib
    L.prepare_weights()
    L.forward()
    # the product kernel on packed operands (what the forward path runs).  The chip lowers its clock
    # under matrix load within some 20 ms: several untimed replays first.
    t_gemm = time_calls(lambda i: pq.pq_qgemm_packed(fmt, g, L.a_op, L.ts_a, L.w_op, L.ts_w, L.y, M, N, K), it,
                        warm_replays=6)
    # what the matrix pipes sustain without any other work: on one constant pair of fragments, and on
    # fragments of these very operands (both inputs change from one instruction to the next)
    # (launches of several ms and untimed replays in front, like the product's: the clock has settled)
    sink = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    mfma_iters = 20000
    fl_c = pq.pq_probe_mfma(mfma_iters, sink)
    t_mfma_c = time_calls(lambda i: pq.pq_probe_mfma(mfma_iters, sink), 3, warm_replays=3)
    fl_o = pq.pq_probe_mfma_operands(fmt, g, L.a_op, L.w_op, M, N, K, mfma_iters, sink)
    t_mfma_o = time_calls(lambda i: pq.pq_probe_mfma_operands(fmt, g, L.a_op, L.w_op, M, N, K, mfma_iters, sink), 3,
                          warm_replays=3)
    t_fwd = time_calls(lambda i: L.forward(), it, warm_replays=4)
    # two more views: the same kernel on all-zero operands at the full shape (no switching activity in the
    # operands: what the kernel's structure allows when the chip is not held back by its power limit); and,
    # for scale, the vendor library's dense bf16 GEMM (torch.matmul) of the unquantized tensors at the same
    # shape -- neither is part of the path
    a_zero, w_zero = torch.zeros_like(L.a_op), torch.zeros_like(L.w_op)
    y_zero = torch.empty_like(L.y)
    t_gemm_zero = time_calls(lambda i: pq.pq_qgemm_packed(fmt, g, a_zero, L.ts_a, w_zero, L.ts_w, y_zero, M, N, K), it,
                             warm_replays=6)
    del a_zero, w_zero, y_zero
    t_blas = time_calls(lambda i: torch.matmul(L.x_run, L.w.t(), out=L.y), it, warm_replays=6)
    L.forward()

    t_qa_warm = time_calls(lambda i: pq.pq_quantize_act_packed(fmt, g, L.x_run, L.ts_a, L.a_op), it)
    # cold: rotate through > 1 GB of distinct inputs so that no input is cache-resident
    n_rot = min(64, max(2, int(1.2e9 // (M * K * 2)) + 1))
    pool = [L.x_run] + [torch.empty_like(L.x_run).copy_(L.x_run) for _ in range(n_rot - 1)]
    nit = max(it, n_rot)
    t_qa_cold = time_calls(lambda i: pq.pq_quantize_act_packed(fmt, g, pool[i % n_rot], L.ts_a, L.a_op), nit)
    L.forward()                       # leave a_op / y as the forward path produces them
    t_mom_cold = time_calls(lambda i: pq.pq_calib_moments(pool[i % n_rot], L.sa, None, L.ws_mom), nit)
    t_mom_warm = time_calls(lambda i: pq.pq_calib_moments(L.x_run, L.sa, None, L.ws_mom), it)
    # references: a plain streaming kernel with the footprint of the quantizer (reads the bf16 tensor,
    # writes codes + scales) and of the moments pass (reads only), on the same rotating inputs
    qout = torch.empty(int(qbytes_out(fmt, g, M, K)) // 16 * 16 + 16, dtype=torch.uint8, device=dev)
    in_bytes = M * K * 2
    t_floor_q = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], in_bytes, qout, qout.numel() - 16), nit)
    t_floor_m = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], in_bytes, qout, 0), nit)
    del pool
    t_mom_all = time_calls(lambda i: pq.pq_calib_moments_batched(L.xs, L.sa, L.amax_a, L.ws_mom), 10)
    # cold: rotate through whole sets of batches (> 1 GB together, beyond the 256 MB Infinity Cache)
    n_sets = min(64, max(2, int(1.2e9 // (nb * M * K * 2)) + 1))
    sets = [L.xs] + [[torch.empty_like(b).copy_(b) for b in L.xs] for _ in range(n_sets - 1)]
    t_mom_all_cold = time_calls(lambda i: pq.pq_calib_moments_batched(sets[i % n_sets], L.sa, L.amax_a, L.ws_mom),
                                2 * n_sets)
    del sets
    # the calibration set as one buffer, rotating over enough copies to stay out of the caches
    xcats = [torch.cat([b.reshape(-1) for b in L.xs]) for _ in range(n_sets)]
    t_floor_mall = time_calls(lambda i: pq.pq_probe_stream(xcats[i % n_sets], xcats[0].numel() * 2, qout, 0),
                              2 * n_sets)
    del xcats, qout
    t_qw = time_calls(lambda i: L.prepare_weights(), 5)
    t_cal = time_calls(lambda i: L.calibrate(), 3, graph=False)
    ta_h = L.ts_a.item() if fmt == pq.FMT_NVFP4 else 1.0
    tw_h = L.ts_w.item() if fmt == pq.FMT_NVFP4 else 1.0
    t_sel = time_calls(lambda i: pq.pq_select_perm(fmt, g, L.sa, L.sw, L.xs, L.w, ta_h, tw_h, L.perm,
                                                   workspace=L.ws_sel), 3, graph=False)
    qbytes = quant_bytes_per_elem(fmt, g) * M * K
    mbytes = 2.0 * M * K
    gemm_tflops = L.flops / t_gemm / 1e12
    mfma_c, mfma_o = fl_c / t_mfma_c / 1e12, fl_o / t_mfma_o / 1e12
    return {
        "qgemm_kernel": {"us": t_gemm * 1e6, "tflops": gemm_tflops, "frac_mfma_f16_peak": gemm_tflops / MFMA_F16_PEAK_TFLOPS,
                         "frac_of_mfma_only_loop_on_these_operands": gemm_tflops / mfma_o},
        "forward_quantize_act_plus_qgemm": {"us": t_fwd * 1e6, "tflops": L.flops / t_fwd / 1e12},
        "qgemm_kernel_all_zero_operands": {"us": t_gemm_zero * 1e6, "tflops": L.flops / t_gemm_zero / 1e12,
                                           "frac_mfma_f16_peak": L.flops / t_gemm_zero / 1e12 / MFMA_F16_PEAK_TFLOPS},
        "reference_vendor_bf16_gemm_same_shape": {"us": t_blas * 1e6, "tflops": L.flops / t_blas / 1e12,
                                                  "frac_mfma_f16_peak": L.flops / t_blas / 1e12 / MFMA_F16_PEAK_TFLOPS},
        "quantize_act_warm": hbm(qbytes, t_qa_warm),
        "quantize_act_cold": hbm(qbytes, t_qa_cold),
        "calib_moments_warm": hbm(mbytes, t_mom_warm),
        "calib_moments_cold": hbm(mbytes, t_mom_cold),
        "calib_moments_all_batches_warm": hbm(nb * mbytes, t_mom_all),
        "calib_moments_all_batches_cold": hbm(nb * mbytes, t_mom_all_cold),
        "quantize_weights_and_pack": {"us": t_qw * 1e6},
        "calibrate_moments_plus_select": {"us": t_cal * 1e6},
        "select_perm": {"us": t_sel * 1e6, "element_evaluations_per_s": 7.0 * (nb * M + N) * K / t_sel},
        # same-run references (not part of the path)
        "reference_stream_quantizer_footprint_cold": {"us": t_floor_q * 1e6, "gbs": qbytes / t_floor_q / 1e9},
        "reference_stream_read_one_batch_cold": {"us": t_floor_m * 1e6, "gbs": mbytes / t_floor_m / 1e9},
        "reference_stream_read_all_batches_cold": {"us": t_floor_mall * 1e6, "gbs": nb * mbytes / t_floor_mall / 1e9},
        "reference_mfma_only_loop_constant_operands": {"tflops": mfma_c, "frac_mfma_f16_peak": mfma_c / MFMA_F16_PEAK_TFLOPS},
        "reference_mfma_only_loop_these_operands": {"tflops": mfma_o, "frac_mfma_f16_peak": mfma_o / MFMA_F16_PEAK_TFLOPS},
    }


def detail_kernels(L, it, time_calls):
    """Auxiliary timings: the row-major operand path, the steps in front of the path (normalisation,
    Hadamard rotation), the selection under the layer-output metric, 3-bit storage."""
    torch, pq, cfg, dev = L.torch, L.pq, L.cfg, L.dev
    import paper_2605_09503_amd.synth as synth
    fmt, g, M, N, K, nb = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K, cfg.n_calib
    out = {}
    ws_gemm = torch.empty(max(pq.pq_workspace_bytes(pq.OP_QGEMM, fmt, g, M, N, K), 16), dtype=torch.uint8, device=dev)
    pq.pq_quantize_act(fmt, g, L.x_run, None, L.ts_a, L.a_codes, L.a_scales)
    pq.pq_qgemm_prep(fmt, g, L.a_scales, L.w_scales, M, N, K, ws_gemm)
    t = time_calls(lambda i: pq.pq_qgemm_run(fmt, g, L.a_codes, L.a_scales, L.ts_a, L.w_codes, L.w_scales, L.ts_w,
                                             L.y, workspace=ws_gemm), it, warm_replays=3)
    out["qgemm_kernel_row_major_operands"] = {"us": t * 1e6, "tflops": L.flops / t / 1e12}
    t = time_calls(lambda i: pq.pq_qgemm(fmt, g, L.a_codes, L.a_scales, L.ts_a, L.w_codes, L.w_scales, L.ts_w, L.y,
                                         workspace=ws_gemm), it)
    out["qgemm_call_row_major_with_scale_prep"] = {"us": t * 1e6, "tflops": L.flops / t / 1e12}
    t = time_calls(lambda i: pq.pq_pack_operand(fmt, g, L.a_codes, L.a_scales, L.a_op), it)
    out["pack_operand_activations"] = {"us": t * 1e6}
    qbytes = quant_bytes_per_elem(fmt, g) * M * K
    mbytes = 2.0 * M * K
    t = time_calls(lambda i: pq.pq_quantize_act(fmt, g, L.x_run, None, L.ts_a, L.a_codes, L.a_scales), it)
    out["quantize_act_row_major_warm"] = hbm(qbytes, t)
    n_rot = min(64, max(2, int(1.2e9 // (M * K * 2)) + 1))
    pool = [L.x_run] + [torch.empty_like(L.x_run).copy_(L.x_run) for _ in range(n_rot - 1)]
    nit = max(it, n_rot)
    t = time_calls(lambda i: pq.pq_quantize_act(fmt, g, pool[i % n_rot], None, L.ts_a, L.a_codes, L.a_scales), nit)
    out["quantize_act_row_major_cold"] = hbm(qbytes, t)
    L.forward()
    # the layer in front of the quantizer (RMSNorm / modulated LayerNorm) with the reorder absorbed
    # into its row load: as a bf16 tensor and feeding the quantizer directly, on the same rotating inputs
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED_BASE + 77)
    n_mod = 4
    gamma = (1.0 + 0.3 * torch.randn(K, device=dev, generator=gen)).to(torch.bfloat16)
    mod_s = (0.5 * torch.randn((n_mod, K), device=dev, generator=gen)).to(torch.bfloat16)
    mod_b = (0.5 * torch.randn((n_mod, K), device=dev, generator=gen)).to(torch.bfloat16)
    per_mod = -(-M // n_mod)
    y_norm = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    norm_op = torch.empty_like(L.a_op)
    ts_n = torch.full((1,), 0.004, dtype=torch.float32, device=dev)     # a static tensor scale for |y| < ~10
    perm = L.perm
    t = time_calls(lambda i: pq.pq_norm_reorder(pq.NORM_RMS, pool[i % n_rot], 1e-6, perm, gamma, y=y_norm), nit)
    out["norm_reorder_rms_cold"] = hbm(2 * mbytes, t)
    t = time_calls(lambda i: pq.pq_norm_reorder(pq.NORM_ADALN, pool[i % n_rot], 1e-6, perm, None, mod_s, mod_b,
                                                per_mod, y=y_norm), nit)
    out["norm_reorder_adaln_cold"] = hbm(2 * mbytes, t)
    t = time_calls(lambda i: pq.pq_norm_quantize_act_packed(pq.NORM_RMS, fmt, g, pool[i % n_rot], 1e-6, ts_n,
                                                            perm, gamma, operand=norm_op), nit)
    out["norm_quantize_act_rms_cold"] = hbm(qbytes, t)
    t = time_calls(lambda i: pq.pq_norm_quantize_act_packed(pq.NORM_ADALN, fmt, g, pool[i % n_rot], 1e-6, ts_n,
                                                            perm, None, mod_s, mod_b, per_mod, operand=norm_op), nit)
    out["norm_quantize_act_adaln_cold"] = hbm(qbytes, t)
    # the Hadamard variant (x H P) where the width has a construction
    if K in (2 ** (K.bit_length() - 1), 12 * 2 ** max(0, (K // 12).bit_length() - 1),
             20 * 2 ** max(0, (K // 20).bit_length() - 1)):
        t = time_calls(lambda i: pq.pq_hadamard_reorder(pool[i % n_rot], perm, y=y_norm), nit)
        out["hadamard_reorder_cold"] = hbm(2 * mbytes, t)
        t = time_calls(lambda i: pq.pq_hadamard_quantize_act_packed(fmt, g, pool[i % n_rot], ts_n, perm,
                                                                    operand=norm_op), nit)
        out["hadamard_quantize_act_cold"] = hbm(qbytes, t)
    t = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], M * K * 2, y_norm, M * K * 2), nit)
    out["reference_stream_norm_footprint_cold"] = {"us": t * 1e6, "gbs": 2 * mbytes / t / 1e9}
    del pool, y_norm, norm_op
    # the selection under the other metric (relative error of the layer's output): the forward path run
    # once per candidate and batch, plus the unquantized products; not part of the timed step
    ws_out = torch.empty(pq.pq_workspace_bytes(pq.OP_SELECT_PERM_OUTPUT, fmt, g, M, N, K, nb), dtype=torch.uint8,
                         device=dev)
    perm_o = torch.empty_like(L.perm)
    ta_h = L.ts_a.item() if fmt == pq.FMT_NVFP4 else 1.0
    tw_h = L.ts_w.item() if fmt == pq.FMT_NVFP4 else 1.0
    t = time_calls(lambda i: pq.pq_select_perm_output_error(fmt, g, L.sa, L.sw, L.xs, L.w, ta_h, tw_h, perm_o,
                                                            workspace=ws_out), 2, graph=False)
    out["select_perm_output_error"] = {"us": t * 1e6}
    del ws_out, perm_o
    if fmt == pq.FMT_INT3:
        # weights at rest in three bits per code: to and from the nibble form, and straight to the GEMM's
        dense = pq.pq_int3_pack(L.w_codes)
        t_p3 = time_calls(lambda i: pq.pq_int3_pack(L.w_codes, dense), it)
        t_u3 = time_calls(lambda i: pq.pq_int3_unpack(dense, K, L.w_codes), it)
        t_o3 = time_calls(lambda i: pq.pq_pack_operand_int3(g, dense, L.w_scales, K, L.w_op), it)
        b3 = 0.875 * N * K
        out["int3_pack_weights_warm"] = {"us": t_p3 * 1e6, "gbs": b3 / t_p3 / 1e9}
        out["int3_unpack_weights_warm"] = {"us": t_u3 * 1e6, "gbs": b3 / t_u3 / 1e9}
        out["pack_operand_int3_weights_warm"] = {"us": t_o3 * 1e6}
    L.prepare_weights()
    L.forward()
    return out


def cpu_baseline(layers, ms_gpu_step):
    """The oracle as it stands (numpy fp64) on a bounded sample of the same workload, extrapolated in
    the row counts (every step of the path is linear in the rows of X and of W).  Also spot-checks the
    timed GPU output against the oracle on the sampled outputs."""
    from oracle import calib as OC, formats as OF, gemm as OG, quantize as OQ
    t_total, parts = 0.0, []
    t_wall = time.perf_counter()
    for L in layers:
        cfg, torch = L.cfg, L.torch
        fmt, g, M, N, K, nb = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K, cfg.n_calib
        perm_h = L.perm.cpu().numpy()
        ta = np.float32(L.ts_a.item()) if fmt == 0 else None
        tw = np.float32(L.ts_w.item()) if fmt == 0 else None
        # about 6 M elements per sampled tensor: a second of the oracle's quantizer each
        rows_w = int(min(N, max(64, (6 << 20) // K)))
        rows_x = int(min(M, max(64, (6 << 20) // K)))
        w64 = OF.bf16_bits_to_f64(L.st.w_bits[:rows_w])
        x64 = OF.bf16_bits_to_f64(L.calib_bits[0][:rows_x])
        # calibration half: moments, the alpha grid's sorts, error of the original and six candidate orders
        t0 = time.perf_counter()
        sw_ref = OC.column_sumsq(w64)
        t_mom_w = time.perf_counter() - t0
        t0 = time.perf_counter()
        sa_ref = OC.column_sumsq(x64)
        t_mom_x = time.perf_counter() - t0
        t0 = time.perf_counter()
        orders = [None] + [OC.sort_descending(OC.joint_key(sa_ref, sw_ref, a)) for a in OC.DEFAULT_ALPHAS]
        t_sort = time.perf_counter() - t0
        t0 = time.perf_counter()
        for p_ in orders:
            OC.squared_error(fmt, g, w64, p_, tw)
        t_err_w = time.perf_counter() - t0
        t0 = time.perf_counter()
        for p_ in orders:
            OC.squared_error(fmt, g, x64, p_, ta)
        t_err_x = time.perf_counter() - t0
        # offline weight quantization in the selected order, then the forward half on sampled rows / columns
        t0 = time.perf_counter()
        qw = OQ.quantize(fmt, g, w64[:, perm_h], tw)
        t_qw = time.perf_counter() - t0
        x_bits_run = L.x_run[:rows_x].view(torch.int16).cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        qa = OQ.quantize(fmt, g, OF.bf16_bits_to_f64(x_bits_run), ta)
        y_ref = OG.dequant_product(fmt, g, qa, qw)
        t_fwd = time.perf_counter() - t0
        fx, fw = M / rows_x, N / rows_w
        t_layer = t_mom_w * fw + t_mom_x * fx * nb + t_sort + t_err_w * fw + t_err_x * fx * nb + t_qw * fw + t_fwd * fx * fw
        t_total += t_layer
        parts.append("%s: %d of %d rows of W and %d of %d rows of one calibration batch / the test batch "
                     "(moments %.2f s, sorts %.2f s, error of 7 orders %.2f + %.2f s, weight quantization %.2f s, "
                     "quantize_act + dequantized product %.2f s; extrapolated layer step %.0f s)"
                     % (L.name, rows_w, N, rows_x, M, t_mom_w + t_mom_x, t_sort, t_err_w, t_err_x, t_qw, t_fwd, t_layer))
        # spot check of the timed GPU result against the oracle on the same outputs
        got = L.y[:rows_x, :rows_w].float().cpu().numpy().astype(np.float64)
        big = np.abs(y_ref) > 1e-2
        rel = np.abs(got[big] - y_ref[big]) / np.abs(y_ref[big])
        log("  %s: spot check vs oracle on %dx%d outputs: max rel err %.3e (bf16 output)" % (L.name, rows_x, rows_w, rel.max()))
        assert rel.max() <= 2.0 ** -8 + 1e-3
    flops = sum(L.flops for L in layers)
    return {"value": flops / t_total / 1e12, "unit": "TFLOP/s", "cores": blas_threads(), "host_cores": os.cpu_count(),
            "kind": "oracle",
            "sample": "the oracle (numpy fp64) on row samples of the same tensors, %.0f s of CPU work, every part scaled "
                      "linearly to the full row counts and all calibration batches -- %s; value = 2*M*N*K / extrapolated "
                      "step time %.0f s; elementwise steps run on one thread, the matmul on `cores` BLAS threads"
                      % (time.perf_counter() - t_wall, "; ".join(parts), t_total)}


def config_summary(L, ms_step, kernels):
    cfg, rep = L.cfg, L.rep
    s = {
        "workload": WORKLOADS[L.name], "format": FMT_NAMES[cfg.fmt], "group": cfg.group,
        "M": cfg.M, "N": cfg.N, "K": cfg.K, "calib_batches": cfg.n_calib,
        "ms_per_step": ms_step, "tflops_per_step": L.flops / (ms_step * 1e-3) / 1e12,
        "qgemm_us": kernels["qgemm_kernel"]["us"], "qgemm_tflops": kernels["qgemm_kernel"]["tflops"],
        "qgemm_frac_mfma_f16_peak": kernels["qgemm_kernel"]["frac_mfma_f16_peak"],
        "qgemm_frac_of_mfma_only_loop_on_these_operands": kernels["qgemm_kernel"]["frac_of_mfma_only_loop_on_these_operands"],
        "quantize_act_cold_frac_hbm_peak": kernels["quantize_act_cold"]["frac_hbm_peak"],
        "quantize_act_warm_frac_hbm_peak": kernels["quantize_act_warm"]["frac_hbm_peak"],
        "calib_moments_cold_frac_hbm_peak": kernels["calib_moments_cold"]["frac_hbm_peak"],
        "calib_moments_all_batches_cold_frac_hbm_peak": kernels["calib_moments_all_batches_cold"]["frac_hbm_peak"],
        "select_perm_us": kernels["select_perm"]["us"],
        "forward_pair_us": kernels["forward_quantize_act_plus_qgemm"]["us"],
        # calibration error (sum of the two tensors' relative squared quantization errors) without and
        # with the selected permutation, and the decision of the acceptance rule
        "accepted": bool(rep.accepted), "alpha_index": int(rep.alpha_index),
        "e_orig": rep.e_orig, "e_best": rep.e_best,
        "kernels": kernels,
    }
    return s


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="all", choices=["all"] + sorted(WORKLOADS))
    ap.add_argument("--kernel-iters", type=int, default=50, help="launches per kernel timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true",
                    help="skip the auxiliary timings (keeps a profile of the path's kernels pure)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on one GPU only (every step of the path shards over token "
            "rows without communication). Run with --gpus 1.")
        sys.exit(2)

    import torch
    from paper_2605_09503_amd import pq, synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    pq.load()                      # fail loudly if the HIP library is missing
    dev = "cuda"
    time_calls = make_timer(torch)
    it = args.kernel_iters

    headline = "c3" if args.config == "all" else args.config
    head_names = ["c3up", "c3down"] if headline == "c3" else [headline]
    others = [n for n in ("c1", "c2", "c4") if args.config == "all"]
    # auxiliary timings: for a single named workload, and for the smallest FLUX-shaped one in the full run
    detail_for = set() if args.no_detail else ({"c1"} if args.config == "all" else set(head_names))
    log("workload %s: %s" % (headline, WORKLOADS[headline]))

    head_layers = [Layer(n, torch, pq, synth, dev) for n in head_names]
    ms_per_step = timed_steps(torch, head_layers, args.steps, args.warmup)
    flops = sum(L.flops for L in head_layers)
    configs = {}
    for L in head_layers:
        ms_l = timed_steps(torch, [L], args.steps, args.warmup) if len(head_layers) > 1 else ms_per_step
        k = core_kernels(L, it, time_calls)
        if L.name in detail_for:
            k.update(detail_kernels(L, it, time_calls))
        configs[L.name] = config_summary(L, ms_l, k)
    # a plain copy of known size, outside every timing: gives the byte counters of a counter
    # run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) a reference to be scaled by
    probe_src = torch.empty(64 << 20, dtype=torch.float32, device=dev).fill_(1.0)
    probe_dst = torch.empty_like(probe_src)
    probe_dst.copy_(probe_src)
    torch.cuda.synchronize()
    del probe_src, probe_dst

    cpu = None if args.no_cpu_baseline else cpu_baseline(head_layers, ms_per_step)
    t_gemm_head = sum(configs[n]["qgemm_us"] for n in head_names) * 1e-6
    gemm_tflops = flops / t_gemm_head / 1e12
    mfma_o = [configs[n]["kernels"]["reference_mfma_only_loop_these_operands"]["tflops"] for n in head_names]
    head_cfg = {n: {key: configs[n][key] for key in ("format", "group", "M", "N", "K", "calib_batches", "accepted")}
                for n in head_names}
    del head_layers
    torch.cuda.empty_cache()

    for n in others:
        L = Layer(n, torch, pq, synth, dev)
        ms_l = timed_steps(torch, [L], args.steps, args.warmup)
        k = core_kernels(L, it, time_calls)
        if n in detail_for:
            k.update(detail_kernels(L, it, time_calls))
        configs[n] = config_summary(L, ms_l, k)
        del L
        torch.cuda.empty_cache()

    for n, c in configs.items():
        log("%s: %.3f ms per step, qgemm %.1f us = %.1f %% of the fp16 MFMA peak (%.0f %% of an MFMA-only loop on the "
            "same operands), quantize_act cold %.1f %%, moments cold %.1f %% / %.1f %% (all batches) of HBM peak, "
            "select_perm %.0f us, E %.5g -> %.5g accepted=%s"
            % (n, c["ms_per_step"], c["qgemm_us"], 100 * c["qgemm_frac_mfma_f16_peak"],
               100 * c["qgemm_frac_of_mfma_only_loop_on_these_operands"], 100 * c["quantize_act_cold_frac_hbm_peak"],
               100 * c["calib_moments_cold_frac_hbm_peak"], 100 * c["calib_moments_all_batches_cold_frac_hbm_peak"],
               c["select_perm_us"], c["e_orig"], c["e_best"], c["accepted"]))
        for kn, v in c["kernels"].items():
            log("  %-46s %s" % (kn, json.dumps({a: round(b, 4) for a, b in v.items()})))

    out = {
        "metric": "qgemm TFLOP/s + % of MFMA-dtype peak on FLUX-shaped W4A4 linears; quantizer GB/s",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "%s: %s" % (headline, WORKLOADS[headline]),
                   "step": "per layer: moments of all calibration batches and W, select_perm, quantize_weights + "
                           "pack_operand, quantize_act_packed, qgemm_packed; value = sum of 2*M*N*K / step time",
                   "layers": head_cfg},
        # the product kernel of the headline workload: flops of its launches (one per layer) over the sum of
        # their event-timed durations
        "roofline": {"bound": "mfma", "kernel": "qgemm_kernel", "achieved": gemm_tflops,
                     "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None,
                     "algorithmic_flops_per_launch": flops / len(head_names),
                     "launches": {n: {"us": configs[n]["qgemm_us"], "frac": configs[n]["qgemm_frac_mfma_f16_peak"]}
                                  for n in head_names},
                     "mfma_only_loop_on_the_same_operands_tflops": sum(mfma_o) / len(mfma_o)},
        "cpu_baseline": cpu,
        "configs": configs,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
