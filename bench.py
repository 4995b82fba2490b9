#!/usr/bin/env python3
"""Benchmark of the per-group-quantized linear layer on one MI355X.

A step is one pass of the whole hot path over one synthetic layer:
  calibration moments of every calibration batch and of W -> permutation selection ->
  weight quantization in the selected order (+ packing into the GEMM's operand layout) ->
  dynamic activation quantization of one token batch (straight into that layout) ->
  low-bit GEMM with bf16 output.
Inputs are generated once (seeded, synthetic, FLUX-DiT-shaped) and are resident in HBM before
the timed region.  One JSON line goes to stdout; everything else goes to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c1]
"""
from __future__ import annotations

import argparse
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
}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c1", choices=sorted(WORKLOADS))
    ap.add_argument("--kernel-iters", type=int, default=50, help="launches per kernel timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-row-major-comparison", action="store_true",
                    help="skip the timings of the row-major operand path (keeps a profile of qgemm_kernel pure)")
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
    cfg = synth.CONFIGS[args.config]
    fmt, g, M, N, K, nb = cfg.fmt, cfg.group, cfg.M, cfg.N, cfg.K, cfg.n_calib
    log("workload %s: %s" % (args.config, WORKLOADS[args.config]))

    t0 = time.perf_counter()
    st, calib_bits, test_bits = synth.make_layer(cfg)
    log("synthetic inputs generated in %.1f s" % (time.perf_counter() - t0))
    xs = [pq.bf16_from_bits(b, dev) for b in calib_bits]
    w = pq.bf16_from_bits(st.w_bits, dev)
    x_test = pq.bf16_from_bits(test_bits, dev)

    # ---- persistent buffers (allocated once; the timed region allocates nothing) ----------
    sa = torch.zeros(K, dtype=torch.float64, device=dev)
    sw = torch.zeros(K, dtype=torch.float64, device=dev)
    amax_a = torch.zeros(1, dtype=torch.float32, device=dev)
    amax_w = torch.zeros(1, dtype=torch.float32, device=dev)
    ts_a = torch.ones(1, dtype=torch.float32, device=dev)
    ts_w = torch.ones(1, dtype=torch.float32, device=dev)
    perm = torch.empty(K, dtype=torch.int32, device=dev)
    a_codes, a_scales = pq.alloc_quantized(fmt, g, M, K, dev)
    w_codes, w_scales = pq.alloc_quantized(fmt, g, N, K, dev)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    ws_mom = torch.empty(max(max(pq.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, fmt, g, M, 0, K, nb),
                             pq.pq_workspace_bytes(pq.OP_CALIB_MOMENTS, fmt, g, N, 0, K, 1)), 16),
                         dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(pq.pq_workspace_bytes(pq.OP_SELECT_PERM, fmt, g, M, N, K, nb), dtype=torch.uint8, device=dev)
    ws_gemm = torch.empty(max(pq.pq_workspace_bytes(pq.OP_QGEMM, fmt, g, M, N, K), 16), dtype=torch.uint8, device=dev)
    a_op = torch.empty(max(pq.pq_operand_bytes(fmt, g, M, K), 16), dtype=torch.uint8, device=dev)   # GEMM operands
    w_op = torch.empty(max(pq.pq_operand_bytes(fmt, g, N, K), 16), dtype=torch.uint8, device=dev)

    def calibrate():
        sa.zero_(); sw.zero_(); amax_a.zero_(); amax_w.zero_()
        pq.pq_calib_moments_batched(xs, sa, amax_a, ws_mom)
        pq.pq_calib_moments(w, sw, amax_w, ws_mom)
        ta = tw = 1.0
        if fmt == pq.FMT_NVFP4:
            pq.pq_tensor_scale(amax_a, ts_a)
            pq.pq_tensor_scale(amax_w, ts_w)
            ta, tw = ts_a.item(), ts_w.item()      # host copies for the selection call
        return pq.pq_select_perm(fmt, g, sa, sw, xs, w, ta, tw, perm, workspace=ws_sel)

    # the producer of the activations emits them in the selected order (the permutation is
    # folded into the previous module offline); build that input once, outside the timing
    rep = calibrate()
    torch.cuda.synchronize()
    x_run = x_test.index_select(1, perm.long()).contiguous()
    log("selection: accepted=%s alpha_index=%d E_orig=%.6g E_best=%.6g" %
        (rep.accepted, rep.alpha_index, rep.e_orig, rep.e_best))

    # forward path: the activation quantizer writes the GEMM's panel layout directly, the
    # weights were packed into it offline
    def forward():
        pq.pq_quantize_act_packed(fmt, g, x_run, ts_a, a_op)
        pq.pq_qgemm_packed(fmt, g, a_op, ts_a, w_op, ts_w, y, M, N, K)

    def prepare_weights():
        pq.pq_quantize_weights(fmt, g, w, perm, w_codes, w_scales, ts_w)
        pq.pq_pack_operand(fmt, g, w_codes, w_scales, w_op)

    def step():
        calibrate()
        prepare_weights()
        forward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    flops = 2.0 * M * N * K

    # ---- per-kernel timings with events on the launch stream ------------------------------
    # The launches of a timing loop are captured into a graph and replayed: a Python loop issues
    # one launch per ~8 us, which would hide every kernel shorter than that behind the host.
    # (Calls that synchronise -- pq_select_perm -- cannot be captured and are timed eagerly.)
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

    it = args.kernel_iters
    # the product kernel on packed operands (what the forward path runs); for comparison the same
    # kernel on the quantizers' row-major layout, alone and with its INT scale preparation
    # (the matrix clock takes some 20 ms of this load to settle: several untimed replays first)
    t_gemm = time_calls(lambda i: pq.pq_qgemm_packed(fmt, g, a_op, ts_a, w_op, ts_w, y, M, N, K), it, warm_replays=6)
    pq.pq_quantize_act(fmt, g, x_run, None, ts_a, a_codes, a_scales)
    t_gemm_rm = t_gemm_call = float("nan")
    if not args.no_row_major_comparison:
        pq.pq_qgemm_prep(fmt, g, a_scales, w_scales, M, N, K, ws_gemm)
        t_gemm_rm = time_calls(lambda i: pq.pq_qgemm_run(fmt, g, a_codes, a_scales, ts_a, w_codes, w_scales, ts_w, y,
                                                         workspace=ws_gemm), it, warm_replays=3)
        t_gemm_call = time_calls(lambda i: pq.pq_qgemm(fmt, g, a_codes, a_scales, ts_a, w_codes, w_scales, ts_w, y,
                                                       workspace=ws_gemm), it)
    t_pack_a = time_calls(lambda i: pq.pq_pack_operand(fmt, g, a_codes, a_scales, a_op), it)
    t_qa_warm = time_calls(lambda i: pq.pq_quantize_act_packed(fmt, g, x_run, ts_a, a_op), it)
    t_qa_rm_warm = time_calls(lambda i: pq.pq_quantize_act(fmt, g, x_run, None, ts_a, a_codes, a_scales), it)
    # cold: rotate through > 1 GB of distinct inputs so that no input is cache-resident
    n_rot = max(2, int(1.2e9 // (M * K * 2)) + 1)
    pool = [x_run] + [torch.empty_like(x_run).copy_(x_run) for _ in range(n_rot - 1)]
    t_qa_cold = time_calls(lambda i: pq.pq_quantize_act_packed(fmt, g, pool[i % n_rot], ts_a, a_op), max(it, n_rot))
    t_qa_rm_cold = time_calls(lambda i: pq.pq_quantize_act(fmt, g, pool[i % n_rot], None, ts_a, a_codes, a_scales),
                              max(it, n_rot))
    forward()                       # leave a_op / y as the forward path produces them
    t_mom_cold = time_calls(lambda i: pq.pq_calib_moments(pool[i % n_rot], sa, None, ws_mom), max(it, n_rot))
    t_mom_warm = time_calls(lambda i: pq.pq_calib_moments(x_run, sa, None, ws_mom), it)
    del pool
    t_mom_all = time_calls(lambda i: pq.pq_calib_moments_batched(xs, sa, amax_a, ws_mom), 10)
    # cold: rotate through whole sets of batches (> 1 GB together, beyond the 256 MB Infinity Cache)
    n_sets = max(2, int(1.2e9 // (nb * M * K * 2)) + 1)
    sets = [xs] + [[torch.empty_like(b).copy_(b) for b in xs] for _ in range(n_sets - 1)]
    t_mom_all_cold = time_calls(lambda i: pq.pq_calib_moments_batched(sets[i % n_sets], sa, amax_a, ws_mom),
                                2 * n_sets)
    del sets
    t_fwd = time_calls(lambda i: forward(), it, warm_replays=4)
    t_qw = time_calls(lambda i: prepare_weights(), 5)
    t_cal = time_calls(lambda i: calibrate(), 3, graph=False)
    ta_h = ts_a.item() if fmt == pq.FMT_NVFP4 else 1.0
    tw_h = ts_w.item() if fmt == pq.FMT_NVFP4 else 1.0
    t_sel = time_calls(lambda i: pq.pq_select_perm(fmt, g, sa, sw, xs, w, ta_h, tw_h, perm, workspace=ws_sel), 3,
                       graph=False)
    # the selection under the other metric (relative error of the layer's output): the forward path run
    # once per candidate and batch, plus the unquantized products; not part of the timed step
    ws_out = torch.empty(pq.pq_workspace_bytes(pq.OP_SELECT_PERM_OUTPUT, fmt, g, M, N, K, nb), dtype=torch.uint8,
                         device=dev)
    perm_o = torch.empty_like(perm)
    t_sel_out = time_calls(lambda i: pq.pq_select_perm_output_error(fmt, g, sa, sw, xs, w, ta_h, tw_h, perm_o,
                                                                    workspace=ws_out), 2, graph=False)
    del ws_out, perm_o

    # references measured in the same run: a plain streaming kernel with the footprint of the
    # quantizer (reads the bf16 tensor, writes codes + scales) and of the moments pass (reads
    # only), on the same rotating inputs; and the matrix rate the device sustains on an
    # MFMA-only loop at the clock it holds under that load
    qout = torch.empty(int(qbytes_out(fmt, g, M, K)) // 16 * 16 + 16, dtype=torch.uint8, device=dev)
    in_bytes = M * K * 2
    pool = [x_run] + [torch.empty_like(x_run).copy_(x_run) for _ in range(n_rot - 1)]
    t_floor_q = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], in_bytes, qout, qout.numel() - 16),
                           max(it, n_rot))
    t_floor_m = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], in_bytes, qout, 0), max(it, n_rot))
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
    norm_op = torch.empty_like(a_op)
    ts_n = torch.full((1,), 0.004, dtype=torch.float32, device=dev)     # a static tensor scale for |y| < ~10
    nit = max(it, n_rot)
    t_rms = time_calls(lambda i: pq.pq_norm_reorder(pq.NORM_RMS, pool[i % n_rot], 1e-6, perm, gamma, y=y_norm), nit)
    t_aln = time_calls(lambda i: pq.pq_norm_reorder(pq.NORM_ADALN, pool[i % n_rot], 1e-6, perm, None, mod_s, mod_b,
                                                    per_mod, y=y_norm), nit)
    t_rms_q = time_calls(lambda i: pq.pq_norm_quantize_act_packed(pq.NORM_RMS, fmt, g, pool[i % n_rot], 1e-6, ts_n,
                                                                  perm, gamma, operand=norm_op), nit)
    t_aln_q = time_calls(lambda i: pq.pq_norm_quantize_act_packed(pq.NORM_ADALN, fmt, g, pool[i % n_rot], 1e-6, ts_n,
                                                                  perm, None, mod_s, mod_b, per_mod, operand=norm_op), nit)
    # the Hadamard variant (x H P) where the width has a construction
    t_had = t_had_q = float("nan")
    if K in (2 ** (K.bit_length() - 1), 12 * 2 ** max(0, (K // 12).bit_length() - 1), 20 * 2 ** max(0, (K // 20).bit_length() - 1)):
        t_had = time_calls(lambda i: pq.pq_hadamard_reorder(pool[i % n_rot], perm, y=y_norm), nit)
        t_had_q = time_calls(lambda i: pq.pq_hadamard_quantize_act_packed(fmt, g, pool[i % n_rot], ts_n, perm,
                                                                          operand=norm_op), nit)
    t_floor_n = time_calls(lambda i: pq.pq_probe_stream(pool[i % n_rot], in_bytes, y_norm, in_bytes), nit)
    del pool, y_norm, norm_op
    # the calibration set as one buffer, rotating over enough copies to stay out of the caches
    xcats = [torch.cat([b.reshape(-1) for b in xs]) for _ in range(n_sets)]
    t_floor_mall = time_calls(lambda i: pq.pq_probe_stream(xcats[i % n_sets], xcats[0].numel() * 2, qout, 0),
                              2 * n_sets)
    del xcats
    sink = torch.empty(256 * 512, dtype=torch.float32, device=dev)
    mfma_iters = 4000
    mfma_flops = pq.pq_probe_mfma(mfma_iters, sink)
    t_mfma = time_calls(lambda i: pq.pq_probe_mfma(mfma_iters, sink), 5)
    mfma_sustained = mfma_flops / t_mfma / 1e12

    qbytes = quant_bytes_per_elem(fmt, g) * M * K
    mbytes = 2.0 * M * K
    gemm_tflops = flops / t_gemm / 1e12
    kernels = {
        "qgemm_kernel": {"us": t_gemm * 1e6, "tflops": gemm_tflops, "frac_mfma_f16_peak": gemm_tflops / MFMA_F16_PEAK_TFLOPS},
        "qgemm_kernel_row_major_operands": {"us": t_gemm_rm * 1e6, "tflops": flops / t_gemm_rm / 1e12},
        "qgemm_call_row_major_with_scale_prep": {"us": t_gemm_call * 1e6, "tflops": flops / t_gemm_call / 1e12},
        "pack_operand_activations": {"us": t_pack_a * 1e6},
        "quantize_act_warm": {"us": t_qa_warm * 1e6, "gbs": qbytes / t_qa_warm / 1e9,
                              "frac_hbm_peak": qbytes / t_qa_warm / 1e9 / HBM_PEAK_GBS},
        "quantize_act_cold": {"us": t_qa_cold * 1e6, "gbs": qbytes / t_qa_cold / 1e9,
                              "frac_hbm_peak": qbytes / t_qa_cold / 1e9 / HBM_PEAK_GBS},
        "quantize_act_row_major_warm": {"us": t_qa_rm_warm * 1e6, "gbs": qbytes / t_qa_rm_warm / 1e9,
                                        "frac_hbm_peak": qbytes / t_qa_rm_warm / 1e9 / HBM_PEAK_GBS},
        "quantize_act_row_major_cold": {"us": t_qa_rm_cold * 1e6, "gbs": qbytes / t_qa_rm_cold / 1e9,
                                        "frac_hbm_peak": qbytes / t_qa_rm_cold / 1e9 / HBM_PEAK_GBS},
        "calib_moments_warm": {"us": t_mom_warm * 1e6, "gbs": mbytes / t_mom_warm / 1e9,
                               "frac_hbm_peak": mbytes / t_mom_warm / 1e9 / HBM_PEAK_GBS},
        "calib_moments_cold": {"us": t_mom_cold * 1e6, "gbs": mbytes / t_mom_cold / 1e9,
                               "frac_hbm_peak": mbytes / t_mom_cold / 1e9 / HBM_PEAK_GBS},
        "calib_moments_all_batches_warm": {"us": t_mom_all * 1e6, "gbs": nb * mbytes / t_mom_all / 1e9,
                                           "frac_hbm_peak": nb * mbytes / t_mom_all / 1e9 / HBM_PEAK_GBS},
        "calib_moments_all_batches_cold": {"us": t_mom_all_cold * 1e6, "gbs": nb * mbytes / t_mom_all_cold / 1e9,
                                           "frac_hbm_peak": nb * mbytes / t_mom_all_cold / 1e9 / HBM_PEAK_GBS},
        "forward_quantize_act_plus_qgemm": {"us": t_fwd * 1e6, "tflops": flops / t_fwd / 1e12},
        "quantize_weights_and_pack": {"us": t_qw * 1e6},
        "calibrate_moments_plus_select": {"us": t_cal * 1e6},
        "select_perm": {"us": t_sel * 1e6,
                        "element_evaluations_per_s": 7.0 * (nb * M + N) * K / t_sel},
        "select_perm_output_error": {"us": t_sel_out * 1e6},
        # the step in front of the path (normalisation with the reorder absorbed), cold inputs
        "norm_reorder_rms_cold": {"us": t_rms * 1e6, "gbs": 2 * mbytes / t_rms / 1e9,
                                  "frac_hbm_peak": 2 * mbytes / t_rms / 1e9 / HBM_PEAK_GBS},
        "norm_reorder_adaln_cold": {"us": t_aln * 1e6, "gbs": 2 * mbytes / t_aln / 1e9,
                                    "frac_hbm_peak": 2 * mbytes / t_aln / 1e9 / HBM_PEAK_GBS},
        "norm_quantize_act_rms_cold": {"us": t_rms_q * 1e6, "gbs": qbytes / t_rms_q / 1e9,
                                       "frac_hbm_peak": qbytes / t_rms_q / 1e9 / HBM_PEAK_GBS},
        "norm_quantize_act_adaln_cold": {"us": t_aln_q * 1e6, "gbs": qbytes / t_aln_q / 1e9,
                                         "frac_hbm_peak": qbytes / t_aln_q / 1e9 / HBM_PEAK_GBS},
        "hadamard_reorder_cold": {"us": t_had * 1e6, "gbs": 2 * mbytes / t_had / 1e9,
                                  "frac_hbm_peak": 2 * mbytes / t_had / 1e9 / HBM_PEAK_GBS},
        "hadamard_quantize_act_cold": {"us": t_had_q * 1e6, "gbs": qbytes / t_had_q / 1e9,
                                       "frac_hbm_peak": qbytes / t_had_q / 1e9 / HBM_PEAK_GBS},
        # same-run references (not part of the path)
        "reference_stream_norm_footprint_cold": {"us": t_floor_n * 1e6, "gbs": 2 * mbytes / t_floor_n / 1e9},
        "reference_stream_quantizer_footprint_cold": {"us": t_floor_q * 1e6, "gbs": qbytes / t_floor_q / 1e9},
        "reference_stream_read_one_batch_cold": {"us": t_floor_m * 1e6, "gbs": mbytes / t_floor_m / 1e9},
        "reference_stream_read_all_batches_cold": {"us": t_floor_mall * 1e6, "gbs": nb * mbytes / t_floor_mall / 1e9},
        "reference_mfma_only_loop": {"tflops": mfma_sustained, "frac_mfma_f16_peak": mfma_sustained / MFMA_F16_PEAK_TFLOPS},
    }
    if fmt == pq.FMT_INT3:
        # weights at rest in three bits per code: to and from the nibble form, and straight to the GEMM's
        dense = pq.pq_int3_pack(w_codes)
        t_p3 = time_calls(lambda i: pq.pq_int3_pack(w_codes, dense), it)
        t_u3 = time_calls(lambda i: pq.pq_int3_unpack(dense, K, w_codes), it)
        t_o3 = time_calls(lambda i: pq.pq_pack_operand_int3(g, dense, w_scales, K, w_op), it)
        b3 = 0.875 * N * K
        kernels["int3_pack_weights_warm"] = {"us": t_p3 * 1e6, "gbs": b3 / t_p3 / 1e9}
        kernels["int3_unpack_weights_warm"] = {"us": t_u3 * 1e6, "gbs": b3 / t_u3 / 1e9}
        kernels["pack_operand_int3_weights_warm"] = {"us": t_o3 * 1e6}
    if args.no_row_major_comparison:
        del kernels["qgemm_kernel_row_major_operands"], kernels["qgemm_call_row_major_with_scale_prep"]
    for k, v in kernels.items():
        log("  %-34s %s" % (k, json.dumps({a: round(b, 4) for a, b in v.items()})))

    # a plain copy of known size, outside every timing: gives the byte counters of a counter
    # run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) a reference to be scaled by
    probe_src = torch.empty(64 << 20, dtype=torch.float32, device=dev).fill_(1.0)
    probe_dst = torch.empty_like(probe_src)
    probe_dst.copy_(probe_src)
    torch.cuda.synchronize()
    del probe_src, probe_dst

    # ---- CPU baseline: the oracle as it stands, on a bounded sample -------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import formats as OF, quantize as OQ, gemm as OG
        perm_h = perm.cpu().numpy()
        ta = np.float32(ts_a.item()) if fmt == 0 else None
        tw = np.float32(ts_w.item()) if fmt == 0 else None
        x_bits_run = x_run.view(torch.int16).cpu().numpy().view(np.uint16)
        cols = min(N, 3072)
        qw = OQ.quantize(fmt, g, OF.bf16_bits_to_f64(st.w_bits[:cols])[:, perm_h], tw)   # offline, not timed

        def cpu_forward(rows):
            t0 = time.perf_counter()
            qa = OQ.quantize(fmt, g, OF.bf16_bits_to_f64(x_bits_run[:rows]), ta)
            yr = OG.dequant_product(fmt, g, qa, qw)
            return time.perf_counter() - t0, yr

        t_probe, _ = cpu_forward(128)
        rows = int(min(M, max(128, 128 * 5.0 / max(t_probe, 1e-3))))       # a few seconds at most
        t_fwd_cpu, y_ref = cpu_forward(rows)
        t_fwd_full = t_fwd_cpu * (M / rows) * (N / cols)
        # calibration half of the step: moments, the alpha grid's sorts, and the error of the
        # original and the six candidate orders -- on as many calibration batches as fit ~10 s
        from oracle import calib as OC
        w64 = OF.bf16_bits_to_f64(st.w_bits)
        t0 = time.perf_counter()
        sw_ref = OC.column_sumsq(w64)
        sa_ref = OC.column_sumsq(OF.bf16_bits_to_f64(calib_bits[0])) * nb     # stand-in for the sort keys
        orders = [None] + [OC.sort_descending(OC.joint_key(sa_ref, sw_ref, a)) for a in OC.DEFAULT_ALPHAS]
        for p_ in orders:
            OC.squared_error(fmt, g, w64, p_, tw)
        t_w_cpu = time.perf_counter() - t0
        used, t_act_cpu = 0, 0.0
        while used < nb and t_act_cpu < 10.0:
            t0 = time.perf_counter()
            xb = OF.bf16_bits_to_f64(calib_bits[used])
            OC.column_sumsq(xb)
            for p_ in orders:
                OC.squared_error(fmt, g, xb, p_, ta)
            t_act_cpu += time.perf_counter() - t0
            used += 1
        t_step_cpu = t_w_cpu + t_act_cpu * nb / used + t_fwd_full
        cpu = {"value": flops / t_step_cpu / 1e12, "unit": "TFLOP/s",
               "cores": blas_threads(), "kind": "oracle",
               "sample": "the oracle (numpy fp64) on the same workload: calibration half (moments, sorts, error of "
                         "the original and six candidate orders) measured on W and on %d of %d calibration batches "
                         "(%.1f s + %.1f s, scaled to all batches), forward half (quantize_act + dequantized "
                         "product) on %d of %d token rows (%.1f s, scaled); value = 2*M*N*K / extrapolated step "
                         "time %.1f s; elementwise steps run on one thread, the matmul on the BLAS threads"
                         % (used, nb, t_w_cpu, t_act_cpu, rows, M, t_fwd_cpu, t_step_cpu)}
        # spot check of the timed GPU result against the oracle on the same outputs
        got = y[:rows, :cols].float().cpu().numpy().astype(np.float64)
        big = np.abs(y_ref) > 1e-2
        rel = np.abs(got[big] - y_ref[big]) / np.abs(y_ref[big])
        log("  spot check vs oracle on %dx%d outputs: max rel err %.3e (bf16 output)" % (rows, cols, rel.max()))
        assert rel.max() <= 2.0 ** -8 + 1e-3

    # HBM bytes per qgemm launch from the committed counter summary, if there is one for this workload
    traffic = None
    prof = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "qgemm_%s_hbm_traffic.md" % args.config)
    if os.path.exists(prof):
        for line in open(prof):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                traffic = float(line.split("=")[1])

    out = {
        "metric": "qgemm TFLOP/s + % of MFMA-dtype peak on FLUX-shaped W4A4 linears; quantizer GB/s",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "%s: %s" % (args.config, WORKLOADS[args.config]),
                   "step": "moments of all calibration batches and W, select_perm, quantize_weights + pack_operand, "
                           "quantize_act_packed, qgemm_packed; value = 2*M*N*K / step time",
                   "format": ["nvfp4", "int4", "int3"][fmt], "group": g, "M": M, "N": N, "K": K,
                   "calib_batches": nb, "accepted": bool(rep.accepted)},
        "roofline": {"bound": "mfma", "kernel": "qgemm_kernel", "achieved": gemm_tflops,
                     "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / MFMA_F16_PEAK_TFLOPS, "traffic": traffic,
                     "algorithmic_flops_per_launch": flops},
        "cpu_baseline": cpu,
        "kernels": kernels,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
