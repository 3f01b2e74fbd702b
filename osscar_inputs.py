"""Seeded synthetic layer generator shared by the oracle tests, the GPU tests and bench.py.

This module holds NONE of the pruning method's arithmetic: it only manufactures the problem data
(calibration activations X, dense weights W, the ridge recipe, group size, k, swap budget) of the five
synthetic layers that stand in for the paper's ResNet50 / OPT workloads (Section 5 "Models and
datasets", Appendix B.1), whose real calibration data and trained weights are not available.

Every element is a pure function of (seed, tensor id, row, column): a 32-bit integer hash picks one of
65536 standard-normal quantiles from a table, so any sub-block of any tensor can be produced on its
own, on the CPU or on the GPU, with identical bits (integer ops, one table lookup, IEEE mul / max /
round-to-nearest-even casts only -- no transcendental is evaluated per element).
"""
from __future__ import annotations

import dataclasses
import functools
from typing import Optional

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_GOLD = 0x9E3779B9

# tensor ids
_T_X, _T_W, _T_XSCALE, _T_HEAVY = 1, 2, 3, 4


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    n: int            # calibration rows (tokens / patches)
    p: int            # number of groups
    q: int            # rows per group
    m: int            # output columns of W
    k: int            # groups to keep
    swaps: int        # local-search swap budget
    x_dtype: str      # "f32" | "bf16"
    w_dtype: str
    lam_abs: float
    lam_rel: float    # lambda = lam_abs + lam_rel * mean(diag(X^T X))
    recipe: str       # "ar1" | "relu_channel" | "relu_col" | "head"
    w_std: float
    scale_sigma: float = 0.0   # sigma of the log-normal per-column / per-group scale
    heavy_cols: int = 0        # number of columns whose scale is multiplied by 20
    mix: float = 0.0           # correlated variant: x_j += mix * x_{j+1 mod d1} before rounding
    seed: int = 0

    @property
    def d1(self) -> int:
        return self.p * self.q

    def replace(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)


_BASE_SEED = 0x05CA0000

CONFIGS = {
    # tiny dense layer, fp32, AR(1)-correlated rows
    "cfg1": LayerConfig("cfg1", n=512, p=64, q=1, m=32, k=32, swaps=50, x_dtype="f32", w_dtype="f32",
                        lam_abs=1e-3, lam_rel=0.0, recipe="ar1", w_std=(1.0 / 64) ** 0.5, seed=_BASE_SEED + 1),
    # exhaustive sub-case of cfg1 (all C(16,8) supports can be enumerated)
    "cfg1x": LayerConfig("cfg1x", n=512, p=16, q=1, m=32, k=8, swaps=50, x_dtype="f32", w_dtype="f32",
                         lam_abs=1e-3, lam_rel=0.0, recipe="ar1", w_std=(1.0 / 16) ** 0.5, seed=_BASE_SEED + 11),
    # ResNet50-style 3x3 conv as im2col least squares
    "cfg2": LayerConfig("cfg2", n=12544, p=256, q=9, m=256, k=128, swaps=500, x_dtype="f32", w_dtype="f32",
                        lam_abs=0.0, lam_rel=1e-2, recipe="relu_channel", w_std=(2.0 / 2304) ** 0.5,
                        scale_sigma=0.5, seed=_BASE_SEED + 2),
    # OPT-1.3B-shaped fc2
    "cfg3": LayerConfig("cfg3", n=262144, p=8192, q=1, m=2048, k=4096, swaps=2000, x_dtype="bf16", w_dtype="bf16",
                        lam_abs=0.0, lam_rel=1e-2, recipe="relu_col", w_std=0.02, scale_sigma=1.0, heavy_cols=8,
                        seed=_BASE_SEED + 3),
    # OPT-1.3B-shaped attention out_proj, heads of 64 rows
    "cfg4": LayerConfig("cfg4", n=262144, p=32, q=64, m=2048, k=24, swaps=200, x_dtype="bf16", w_dtype="bf16",
                        lam_abs=0.0, lam_rel=1e-2, recipe="head", w_std=0.02, scale_sigma=0.7, seed=_BASE_SEED + 4),
    # OPT-30B-shaped fc2
    "cfg5": LayerConfig("cfg5", n=262144, p=28672, q=1, m=7168, k=14336, swaps=5000, x_dtype="bf16", w_dtype="bf16",
                        lam_abs=0.0, lam_rel=1e-2, recipe="relu_col", w_std=0.015, scale_sigma=1.0,
                        seed=_BASE_SEED + 5),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


@functools.lru_cache(maxsize=None)
def _quantile_table_np() -> np.ndarray:
    """65536 standard-normal quantiles at the bin mid-points, as float32."""
    from scipy.special import ndtri
    u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(u).astype(np.float32)


@functools.lru_cache(maxsize=None)
def _quantile_table(device: str) -> torch.Tensor:
    return torch.from_numpy(_quantile_table_np()).to(device)


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """A 32-bit avalanche mixer on int64 tensors holding values in [0, 2^32)."""
    x = ((x ^ (x >> 16)) * 0x7FEB352D) & _M32
    x = ((x ^ (x >> 15)) * 0x846CA68B) & _M32
    return x ^ (x >> 16)


def _mix32_int(x: int) -> int:
    x &= _M32
    x = ((x ^ (x >> 16)) * 0x7FEB352D) & _M32
    x = ((x ^ (x >> 15)) * 0x846CA68B) & _M32
    return x ^ (x >> 16)


def hash_u32(seed: int, tensor_id: int, rows: torch.Tensor, cols: torch.Tensor) -> torch.Tensor:
    """hash(seed, tensor_id, row, col) in [0, 2^32) for the outer grid rows x cols (int64 tensors)."""
    base = _mix32_int(seed ^ _mix32_int(tensor_id * _GOLD))
    hr = _mix32((rows + base) & _M32)                       # per row
    hc = (cols * _GOLD) & _M32                              # per column
    return _mix32(hr[:, None] ^ hc[None, :])


def std_normal(seed: int, tensor_id: int, rows: torch.Tensor, cols: torch.Tensor) -> torch.Tensor:
    """float32 standard-normal variates (16-bit quantile resolution, |z| <= 4.3) on the rows x cols grid."""
    h = hash_u32(seed, tensor_id, rows, cols)
    return _quantile_table(str(rows.device))[h >> 16]


def _arange(n: int, device) -> torch.Tensor:
    return torch.arange(n, dtype=torch.int64, device=device)


def column_scales(cfg: LayerConfig) -> np.ndarray:
    """Per-column multiplicative scale of X (float32), always computed on the CPU."""
    d1 = cfg.d1
    if cfg.recipe == "ar1":
        return np.ones(d1, dtype=np.float32)
    ngrp = cfg.p if cfg.recipe in ("relu_channel", "head") else d1
    z = std_normal(cfg.seed, _T_XSCALE, _arange(1, "cpu"), _arange(ngrp, "cpu"))[0].numpy().astype(np.float64)
    s = np.exp(cfg.scale_sigma * z)
    if cfg.recipe in ("relu_channel", "head"):
        s = np.repeat(s, cfg.q)
    if cfg.heavy_cols:
        h = hash_u32(cfg.seed, _T_HEAVY, _arange(1, "cpu"), _arange(4 * cfg.heavy_cols, "cpu"))[0].numpy()
        picked = []
        for v in h:
            c = int(v) % d1
            if c not in picked:
                picked.append(c)
            if len(picked) == cfg.heavy_cols:
                break
        s[np.array(picked)] *= 20.0
    return s.astype(np.float32)


def gen_X(cfg: LayerConfig, row0: int = 0, nrows: Optional[int] = None, cols: Optional[torch.Tensor] = None,
          device="cpu") -> torch.Tensor:
    """Rows [row0, row0+nrows) of X restricted to columns `cols` (int64 tensor; default all), in cfg.x_dtype."""
    device = torch.device(device)
    nrows = cfg.n - row0 if nrows is None else nrows
    d1 = cfg.d1
    rows = _arange(nrows, device) + row0
    allcols = cols is None
    cols = _arange(d1, device) if allcols else cols.to(device=device, dtype=torch.int64)
    scales = torch.from_numpy(column_scales(cfg)).to(device)

    def raw(cc: torch.Tensor) -> torch.Tensor:
        z = std_normal(cfg.seed, _T_X, rows, cc)
        if cfg.recipe == "ar1":
            return z
        if cfg.recipe in ("relu_channel", "relu_col"):
            return torch.clamp_min(z * scales[cc][None, :], 0.0)
        if cfg.recipe == "head":
            return z * scales[cc][None, :]
        raise ValueError(cfg.recipe)

    if cfg.recipe == "ar1":
        # x_0 = z_0, x_i = 0.6 x_{i-1} + 0.8 z_i : stationary AR(1), Sigma_ij = 0.6^|i-j|
        z = raw(_arange(d1, device))
        x = torch.empty_like(z)
        x[:, 0] = z[:, 0]
        for i in range(1, d1):
            x[:, i] = x[:, i - 1] * 0.6 + z[:, i] * 0.8
        if cfg.mix:
            x = x + cfg.mix * torch.roll(x, -1, dims=1)
        x = x[:, cols]
    else:
        x = raw(cols)
        if cfg.mix:
            x = x + cfg.mix * raw((cols + 1) % d1)
    return x.to(torch_dtype(cfg.x_dtype)).contiguous()


def gen_W(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """Dense weights W (d1 x m) in cfg.w_dtype."""
    device = torch.device(device)
    z = std_normal(cfg.seed, _T_W, _arange(cfg.d1, device), _arange(cfg.m, device))
    return (z * np.float32(cfg.w_std)).to(torch_dtype(cfg.w_dtype)).contiguous()


def scaled(cfg: LayerConfig, p: int, m: int, n: int, k: Optional[int] = None, swaps: Optional[int] = None,
           **kw) -> LayerConfig:
    """A smaller layer with the same recipe (for parity tests that the CPU oracle finishes in seconds)."""
    return cfg.replace(name=f"{cfg.name}_p{p}_m{m}_n{n}", p=p, m=m, n=n, k=(p // 2 if k is None else k),
                       swaps=(cfg.swaps if swaps is None else swaps), **kw)
