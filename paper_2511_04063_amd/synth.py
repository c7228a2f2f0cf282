"""Seeded synthetic inputs for the QR-Orth calibration step.

This module only draws numbers.  It contains none of the method's arithmetic (no QR,
no loss, no gradients) so that the GPU library's tests and the independent CPU
checker can both take their inputs from it.

The paper calibrates on LLM activations (128 sequences x 2048 tokens, about 10 % of
the tokens kept, batch 64; Sec. 5 and the appendix on sample size) whose statistics it
reports as zero-mean, unit-variance, very heavy-tailed (kurtosis 37-245, appendix on
activation statistics) with a few massive-outlier channels.  Neither the models nor the
datasets are available here; the generators below stand in for them with the same
shapes (hidden sizes 4096 / 5120 / 8192 and 128x128 head rotations), token counts and
value structure.

All draws come from NumPy's counter-based Philox generator, so a (config, seed) pair
always gives the same bytes on every machine.
"""

from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20251104


@dataclass(frozen=True)
class CalibConfig:
    """Shape and value recipe of one workload."""

    name: str
    b: int            # independent problems
    n: int            # channels (rotation is n x n)
    T: int            # token rows per problem
    x_dtype: str      # "f32" or "bf16": storage type of X
    dist: str         # "normal" or "student_t3"
    outlier_frac: float   # fraction of channels scaled (ceil), or 0 when outlier_count is used
    outlier_count: int    # explicit number of outlier channels (0 -> use outlier_frac)
    outlier_scale: float
    token_lognormal_sigma: float  # 0 -> no per-token scale
    steps: int
    lr: float
    index: int        # used to derive the seeds


CONFIGS = {
    # n=256, T=2048, fp32; N(0,1) with 4 seeded channels x50; 10 steps, lr 1e-2
    "tiny": CalibConfig("tiny", 1, 256, 2048, "f32", "normal", 0.0, 4, 50.0, 0.0, 10, 1e-2, 0),
    # 7B-shaped residual rotation
    "7b": CalibConfig("7b", 1, 4096, 8192, "bf16", "student_t3", 0.01, 0, 30.0, 0.5, 100, 1e-2, 1),
    # 13B-shaped
    "13b": CalibConfig("13b", 1, 5120, 8192, "bf16", "student_t3", 0.01, 0, 30.0, 0.5, 100, 1e-2, 2),
    # 70B-shaped
    "70b": CalibConfig("70b", 1, 8192, 16384, "bf16", "student_t3", 0.005, 0, 100.0, 0.5, 100, 1e-3, 3),
    # 64 independent head-dim rotations
    "heads": CalibConfig("heads", 64, 128, 16384, "bf16", "normal", 0.0, 2, 40.0, 0.0, 200, 1e-3, 4),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32.

    bfloat16 keeps the top 16 bits of the IEEE-754 binary32 pattern.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    rounded &= np.uint32(0xFFFF0000)
    out = rounded.view(np.float32).copy()
    # keep NaN/Inf patterns untouched (the generators never produce them)
    bad = ~np.isfinite(a)
    if bad.any():
        out[bad] = a[bad]
    return out


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of float32 values that are exactly bfloat16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


def scaled_config(base: str, *, n: int | None = None, T: int | None = None,
                  b: int | None = None, x_dtype: str | None = None) -> CalibConfig:
    """A config with the value recipe of ``base`` but other sizes (for small parity cases)."""
    c = CONFIGS[base]
    return CalibConfig(
        name=f"{c.name}-like", b=c.b if b is None else b, n=c.n if n is None else n,
        T=c.T if T is None else T, x_dtype=c.x_dtype if x_dtype is None else x_dtype,
        dist=c.dist, outlier_frac=c.outlier_frac, outlier_count=c.outlier_count,
        outlier_scale=c.outlier_scale, token_lognormal_sigma=c.token_lognormal_sigma,
        steps=c.steps, lr=c.lr, index=c.index)


def make_inputs(cfg: CalibConfig | str, seed: int | None = None, row_chunk: int = 1024):
    """Draw X (b, T, n) and Z0 (b, n, n) for a config.

    Returns a dict with
      X    float32 array (b, T, n); when cfg.x_dtype == "bf16" every value is exactly
           representable in bfloat16 (rounded once here, ties to even);
      Z0   float32 array (b, n, n), N(0,1);
      outlier_channels  int array (b, k);
      cfg  the config.
    Seeds: BASE_SEED*10 + cfg.index (+ user seed * 1000) for X, +5 for Z0, +7 for the
    outlier-channel permutation.
    """
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    s0 = BASE_SEED * 10 + cfg.index + (0 if seed is None else 1000 * int(seed))
    rx, rz, rp = _rng(s0), _rng(s0 + 5), _rng(s0 + 7)
    b, n, T = cfg.b, cfg.n, cfg.T
    k_out = cfg.outlier_count if cfg.outlier_count > 0 else int(math.ceil(cfg.outlier_frac * n))
    k_out = min(k_out, n)
    X = np.empty((b, T, n), dtype=np.float32)
    chans = np.empty((b, k_out), dtype=np.int64)
    for ib in range(b):
        ch = rp.permutation(n)[:k_out]
        chans[ib] = ch
        col_scale = np.ones(n, dtype=np.float64)
        col_scale[ch] = cfg.outlier_scale
        for r0 in range(0, T, row_chunk):
            r1 = min(T, r0 + row_chunk)
            if cfg.dist == "normal":
                blk = rx.standard_normal((r1 - r0, n))
            elif cfg.dist == "student_t3":
                blk = rx.standard_t(3.0, size=(r1 - r0, n))
            else:
                raise ValueError(cfg.dist)
            blk *= col_scale[None, :]
            if cfg.token_lognormal_sigma > 0.0:
                g = rx.standard_normal(r1 - r0)
                blk *= np.exp(cfg.token_lognormal_sigma * g)[:, None]
            X[ib, r0:r1] = blk.astype(np.float32)
    if cfg.x_dtype == "bf16":
        X = round_to_bf16(X.reshape(-1)).reshape(b, T, n)
    Z0 = rz.standard_normal((b, n, n)).astype(np.float32)
    return {"X": X, "Z0": Z0, "outlier_channels": chans, "cfg": cfg}
