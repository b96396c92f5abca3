"""Seeded synthetic inputs for the SERQ linear layer.

This module only draws random tensors and moves data around (casts, channel
gathers).  It holds none of the method's arithmetic: no quantisation, no
saliency metric, no matmul.  Both the CPU oracle's tests and the HIP path's
tests / bench take their inputs from here, so the two sides see identical
bits without sharing any code that computes.

The shapes follow the LLaMA-style layer sizes of the paper's per-layer latency
table (appendix, Table 10) and the activation structure the paper describes
(a few channels carry outliers that are one to two orders of magnitude larger
than the rest; Sec. 2.1 and Sec. 3.2).  No dataset or trained weight is used.

Recipe (every tensor has its own PCG64 stream, seed = 1000*config + index):
  X  [M,K]  ~ N(0,1); a seeded subset of channels ("outliers") is multiplied
            by a per-channel factor drawn from U(lo,hi) (or a constant).
  s  [K]    ~ U(0.5,2); on outlier channels additionally * sqrt(factor), so
            the static flattening moves part of the outlier into the weights.
  W  [N,K]  ~ N(0,0.02).
  R  [r,N]  ~ N(0,0.01)   (a stand-in compensation matrix; tests also use the
            residual the offline pack step extracts).
X, W, R are rounded to the layer's storage dtype (fp16 or bf16); s stays fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np
import torch

_DT = {"fp16": torch.float16, "bf16": torch.bfloat16, "fp32": torch.float32}


@dataclass(frozen=True)
class LayerSpec:
    name: str
    cfg: int            # which of the five benchmark configurations this belongs to
    abits: int          # 4 (W4A4) or 8 (W4A8)
    M: int
    K: int
    N: int
    r: int
    in_dtype: str       # storage dtype of X, W, R
    out_dtype: str      # dtype of Y
    n_outlier: int      # number of outlier channels
    mult_lo: float      # outlier multiplier range
    mult_hi: float
    seed_index: int = 0

    @property
    def seed(self) -> int:
        return 1000 * self.cfg + self.seed_index

    def with_(self, **kw) -> "LayerSpec":
        return replace(self, **kw)


def _pct(K: int, frac: float) -> int:
    return max(1, int(round(K * frac)))


def config1() -> LayerSpec:
    return LayerSpec("cfg1_tiny", 1, 4, 8, 256, 256, 16, "fp16", "fp32", 4, 20.0, 20.0)


def config2() -> LayerSpec:
    return LayerSpec("cfg2_attn_proj", 2, 4, 2048, 4096, 4096, 64, "bf16", "bf16",
                     _pct(4096, 0.01), 30.0, 100.0)


def config3(which: str, M: int) -> LayerSpec:
    if which == "up":
        K, N, idx = 4096, 11008, 0
    elif which == "down":
        K, N, idx = 11008, 4096, 1
    else:
        raise ValueError(which)
    return LayerSpec(f"cfg3_{which}_M{M}", 3, 8, M, K, N, 128, "bf16", "bf16",
                     _pct(K, 0.01), 30.0, 100.0, seed_index=10 * idx)


def config4(M: int) -> LayerSpec:
    return LayerSpec(f"cfg4_wide_M{M}", 4, 4, M, 8192, 28672, 128, "bf16", "bf16",
                     _pct(8192, 0.005), 50.0, 50.0)


_CFG5 = {"qkv": (4096, 6144, 0), "o": (4096, 4096, 1),
         "gate_up": (4096, 28672, 2), "down": (14336, 4096, 3)}


def config5(layer: str, r: int) -> LayerSpec:
    K, N, idx = _CFG5[layer]
    return LayerSpec(f"cfg5_{layer}_r{r}", 5, 4, 4096, K, N, r, "bf16", "bf16",
                     _pct(K, 0.01), 30.0, 100.0, seed_index=10 * idx)


def config5_layers() -> Tuple[str, ...]:
    return tuple(_CFG5)


def _rng(spec: LayerSpec, k: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(spec.seed * 16 + k))


def _normal_to(rng: np.random.Generator, shape, std: float, dtype: torch.dtype,
               rows_per_block: int = 1024) -> torch.Tensor:
    """N(0,std) drawn block-wise in fp32 and rounded to `dtype` (keeps host memory low)."""
    out = torch.empty(shape, dtype=dtype)
    rows = shape[0]
    for r0 in range(0, rows, rows_per_block):
        r1 = min(rows, r0 + rows_per_block)
        blk = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        out[r0:r1] = torch.from_numpy(blk).to(dtype)
    return out


def make_layer(spec: LayerSpec, want=("X", "s", "W", "R")) -> Dict[str, object]:
    """Draw the layer's tensors (original channel order).

    Returns a dict with torch CPU tensors X [M,K], W [N,K], R [r,N] in the
    storage dtype, s [K] fp32, and `outliers` (int64 channel indices) /
    `mult` (their factors).  Pieces not named in `want` are skipped.
    """
    dt = _DT[spec.in_dtype]
    out: Dict[str, object] = {"spec": spec}

    r_ch = _rng(spec, 0)
    outliers = np.sort(r_ch.choice(spec.K, size=spec.n_outlier, replace=False)).astype(np.int64)
    if spec.mult_lo == spec.mult_hi:
        mult = np.full(spec.n_outlier, spec.mult_lo, dtype=np.float32)
    else:
        mult = r_ch.uniform(spec.mult_lo, spec.mult_hi, size=spec.n_outlier).astype(np.float32)
    out["outliers"] = outliers
    out["mult"] = mult

    if "X" in want:
        rng = _rng(spec, 1)
        X = np.empty((spec.M, spec.K), dtype=np.float32)
        for r0 in range(0, spec.M, 1024):
            r1 = min(spec.M, r0 + 1024)
            X[r0:r1] = rng.standard_normal((r1 - r0, spec.K), dtype=np.float32)
        X[:, outliers] *= mult[None, :]
        out["X"] = torch.from_numpy(X).to(dt)
    if "s" in want:
        rng = _rng(spec, 2)
        s = rng.uniform(0.5, 2.0, size=spec.K).astype(np.float32)
        s[outliers] *= np.sqrt(mult).astype(np.float32)
        out["s"] = torch.from_numpy(s)
    if "W" in want:
        out["W"] = _normal_to(_rng(spec, 3), (spec.N, spec.K), 0.02, dt)
    if "R" in want and spec.r > 0:
        out["R"] = _normal_to(_rng(spec, 4), (spec.r, spec.N), 0.01, dt)
    return out


def permute_channels(X: torch.Tensor, perm) -> torch.Tensor:
    """X_hat[:, kp] = X[:, perm[kp]] -- the channel order the permuted weights expect."""
    idx = torch.as_tensor(np.asarray(perm), dtype=torch.int64)
    return X.index_select(1, idx).contiguous()


def integer_layer(M: int, K: int, N: int, qx: int, seed: int):
    """Integer-valued X in [-qx,qx] and W in [-7,7], every row containing its extreme value.

    With s = 1 every quantisation scale is exactly 1, so the whole layer must
    reduce to a textbook integer matrix product.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.integers(-qx, qx + 1, size=(M, K)).astype(np.float32)
    W = rng.integers(-7, 8, size=(N, K)).astype(np.float32)
    X[np.arange(M), rng.integers(0, K, size=M)] = np.where(rng.random(M) < 0.5, -qx, qx)
    W[np.arange(N), rng.integers(0, K, size=N)] = np.where(rng.random(N) < 0.5, -7, 7)
    return X, W
