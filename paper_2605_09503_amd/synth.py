"""Seeded synthetic inputs for the per-group-quantized linear layer.

This module only draws random tensors and rounds them to bf16.  It holds none of
the method's arithmetic (no quantizer, no moments, no sort, no GEMM), so both the
CPU oracle's tests and the HIP path's tests can take their inputs from it.

The tensors stand in for the calibration activations and the weights of the
FLUX.1-dev linears the paper measures on (Sec. 4.4): the real model weights and
calibration prompts are not available, so shapes, outlier structure and value
distributions are synthetic.  Values are formed in fp64, rounded once
(round-to-nearest-even) to bf16, and handed out as uint16 bit patterns, so the
same bits reach every consumer.

Layout: X is [M, K] row-major (tokens x input channels); W is [N, K] row-major
(output x input channels), i.e. Y = X @ W.T (Eq. 8 with the paper's W transposed).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

FMT_NVFP4 = 0
FMT_INT4 = 1
FMT_INT3 = 2

SEED_BASE = 950300


@dataclass(frozen=True)
class LayerCfg:
    """One linear layer of a configuration."""
    name: str
    cfg_id: int
    fmt: int
    group: int
    M: int
    N: int
    K: int
    n_calib: int
    act_kind: str            # "gauss", "student_t3", "gelu"
    act_sigma: float         # sigma of the log-normal channel scales
    n_outlier: int           # outlier channels
    outlier_lo: float
    outlier_hi: float
    row_boost_frac: float = 0.0   # fraction of rows scaled by row_boost
    row_boost: float = 1.0
    seed_offset: int = 0     # distinguishes the layers of one configuration


CONFIGS: Dict[str, LayerCfg] = {
    # Tiny NVFP4 layer
    "c0": LayerCfg("c0", 0, FMT_NVFP4, 16, 256, 512, 512, 4, "gauss", 0.5, 8, 30.0, 30.0),
    # INT4 g64, attention-out projection (4096 image + 512 text tokens)
    "c1": LayerCfg("c1", 1, FMT_INT4, 64, 4608, 3072, 3072, 8, "gauss", 0.5, 32, 20.0, 50.0),
    # NVFP4 g16, fused QKV projection, heavy-tailed activations
    "c2": LayerCfg("c2", 2, FMT_NVFP4, 16, 4608, 9216, 3072, 8, "student_t3", 0.7, 0, 1.0, 1.0),
    # NVFP4 g16, MLP up / down pair
    "c3up": LayerCfg("c3up", 3, FMT_NVFP4, 16, 4608, 12288, 3072, 8, "gauss", 0.5, 8, 30.0, 30.0),
    "c3down": LayerCfg("c3down", 3, FMT_NVFP4, 16, 4608, 3072, 12288, 8, "gelu", 0.5, 0, 1.0, 1.0,
                       seed_offset=5),
    # INT3 g32 stress case
    "c4": LayerCfg("c4", 4, FMT_INT3, 32, 8192, 12288, 3072, 8, "gauss", 0.5, 64, 50.0, 50.0,
                   row_boost_frac=0.05, row_boost=4.0),
}


def scaled(cfg: LayerCfg, M: int | None = None, N: int | None = None, K: int | None = None,
           n_calib: int | None = None, n_outlier: int | None = None, name: str | None = None
           ) -> LayerCfg:
    """A copy of cfg with smaller shapes (for parity cases the oracle finishes quickly)."""
    import dataclasses
    return dataclasses.replace(
        cfg,
        M=cfg.M if M is None else M, N=cfg.N if N is None else N, K=cfg.K if K is None else K,
        n_calib=cfg.n_calib if n_calib is None else n_calib,
        n_outlier=cfg.n_outlier if n_outlier is None else n_outlier,
        name=name or (cfg.name + "_scaled"))


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round fp64 values to bf16 (round-to-nearest-even, one rounding) -> uint16 bits.

    The fp64 -> bf16 rounding is done directly on the fp64 value (not via fp32),
    so there is no double rounding.
    """
    v = np.ascontiguousarray(v, dtype=np.float64)
    f = v.astype(np.float32)                      # candidate (may be double-rounded)
    b = f.view(np.uint32)
    # candidate bf16 neighbours around v: truncate fp32 bits, then pick nearest to v in fp64
    lo = (b & np.uint32(0xFFFF0000))
    hi = lo + np.uint32(0x00010000)
    lo_f = lo.view(np.float32).astype(np.float64)
    hi_f = hi.view(np.float32).astype(np.float64)
    # lo_f and hi_f bracket f in magnitude; f itself may sit one fp32 ulp off v, so compare to v
    d_lo = np.abs(v - lo_f)
    d_hi = np.abs(hi_f - v)
    lo_even = ((lo >> np.uint32(16)) & np.uint32(1)) == 0
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~lo_even)
    out = np.where(take_hi, hi, lo) >> np.uint32(16)
    return out.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class LayerStruct:
    """What stays fixed over the calibration batches of one layer."""
    cfg: LayerCfg
    chan_scale: np.ndarray        # [K] fp64, outliers included
    w_bits: np.ndarray            # [N, K] uint16 bf16 bits


def _struct_rng(cfg: LayerCfg) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED_BASE + 10 * cfg.cfg_id + cfg.seed_offset))


def _batch_rng(cfg: LayerCfg, b: int) -> np.random.Generator:
    # batches 0..n_calib-1 calibrate; batch n_calib is the test / timed batch
    return np.random.Generator(
        np.random.PCG64(SEED_BASE + 10 * cfg.cfg_id + cfg.seed_offset + 1000 * (1 + b)))


def make_struct(cfg: LayerCfg) -> LayerStruct:
    rng = _struct_rng(cfg)
    chan = np.exp(cfg.act_sigma * rng.standard_normal(cfg.K))
    if cfg.n_outlier > 0:
        idx = rng.choice(cfg.K, size=cfg.n_outlier, replace=False)
        chan[idx] *= rng.uniform(cfg.outlier_lo, cfg.outlier_hi, size=cfg.n_outlier)
    w_chan = np.exp(0.3 * rng.standard_normal(cfg.K))
    w_bits = np.empty((cfg.N, cfg.K), dtype=np.uint16)
    step = max(1, (1 << 22) // cfg.K)
    for r0 in range(0, cfg.N, step):
        r1 = min(cfg.N, r0 + step)
        w = 0.02 * rng.standard_normal((r1 - r0, cfg.K)) * w_chan[None, :]
        w_bits[r0:r1] = f64_to_bf16_bits(w)
    return LayerStruct(cfg, chan, w_bits)


def make_batch(st: LayerStruct, b: int, M: int | None = None) -> np.ndarray:
    """Activation batch b as bf16 bits [M, K]."""
    cfg = st.cfg
    M = cfg.M if M is None else M
    rng = _batch_rng(cfg, b)
    out = np.empty((M, cfg.K), dtype=np.uint16)
    if cfg.row_boost_frac > 0.0:
        n_boost = int(cfg.row_boost_frac * M)
        boost_rows = rng.choice(M, size=n_boost, replace=False)
        row_mul = np.ones(M)
        row_mul[boost_rows] = cfg.row_boost
    else:
        row_mul = None
    step = max(1, (1 << 22) // cfg.K)
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        if cfg.act_kind == "student_t3":
            base = rng.standard_t(3.0, size=(r1 - r0, cfg.K))
        else:
            base = rng.standard_normal((r1 - r0, cfg.K))
        v = base * st.chan_scale[None, :]
        if cfg.act_kind == "gelu":
            from scipy.special import erf
            v = 0.5 * v * (1.0 + erf(v / np.sqrt(2.0)))
        if row_mul is not None:
            v = v * row_mul[r0:r1, None]
        out[r0:r1] = f64_to_bf16_bits(v)
    return out


def make_layer(cfg: LayerCfg) -> Tuple[LayerStruct, List[np.ndarray], np.ndarray]:
    """(struct, calibration batches, test batch) for one layer."""
    st = make_struct(cfg)
    calib = [make_batch(st, b) for b in range(cfg.n_calib)]
    test = make_batch(st, cfg.n_calib)
    return st, calib, test
