"""Seeded synthetic inputs for the sparse-linear attention path (numpy only).

This module holds no arithmetic of the method itself: it only draws the tensors
that both the HIP path and the CPU oracle are fed with.  The inputs stand in for
the attention activations of a video diffusion transformer (Section 6.1 of the
paper uses Wan2.1-1.3B: 12 heads of 128, about 32K tokens, 64x64 blocks,
k_h=5%, k_l=10%; the appendix's image experiment has N = 1024 on a 2-D grid): tokens live on a (t, h, w) grid in raster order, and Q/K/V are
smooth random Fourier features of the grid position plus white noise, so that
neighbouring query blocks prefer overlapping key blocks the way real video
attention does.

Recipe (per batch b and head h, generator PCG64([seed, b, h])):
  omega  [8,3] ~ N(0,1)        cycles per grid extent
  beta   [8]   ~ U[0, 2pi)
  G_Q, G_K, G_V [8,d] ~ N(0, 1/8)
  F[n,m] = sqrt(2) cos(2pi omega_m . p_n + beta_m),  p_n = (t/Tg, y/Hg, x/Wg)
  X = F G_X + 0.3 N(0,1)       for X in Q, K (and V unless v_white)
  V ~ N(0,1)                   when v_white (the tiny fp32 case)
  unit_var: X /= sqrt(1.09);   bf16: values rounded once to bf16 (RNE)
Proj ~ N(0, 0.02^2) from PCG64([seed, 1000003]); dO ~ N(0,1) from
PCG64([seed, b, h, 7]).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Iterable, Optional, Tuple

import numpy as np

BASE_SEED = 250924006


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d: int
    grid: Tuple[int, int, int]
    dtype: str            # "fp32" | "bf16": storage type of Q,K,V,Proj,dO
    k_h: float
    k_l: float
    phi: str = "softmax"
    block: int = 64
    v_white: bool = False
    unit_var: bool = True
    seed: int = BASE_SEED

    @property
    def N(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def T(self) -> int:
        return -(-self.N // self.block)


WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 case: forward and backward, the oracle finishes in well under a second
    "tiny": Workload("tiny", 1, 2, 64, (4, 16, 16), "fp32", 0.10, 0.10,
                     v_white=True, unit_var=False, seed=BASE_SEED + 1),
    # Wan-1.3B-shaped layer (forward only / forward+backward use the same tensors)
    "wan": Workload("wan", 1, 12, 128, (21, 30, 52), "bf16", 0.05, 0.10, seed=BASE_SEED + 2),
    # long-sequence layer
    "long": Workload("long", 1, 40, 128, (21, 45, 80), "bf16", 0.05, 0.10, seed=BASE_SEED + 5),
    # image-shaped layer (Appendix, image generation: 512 x 512 images -> a 32 x 32 latent grid,
    # N = 1024, 87.5 % sparsity i.e. k_h = 12.5 %): short sequences, many (batch x head) problems
    "image": Workload("image", 16, 16, 64, (1, 32, 32), "bf16", 0.125, 0.10, seed=BASE_SEED + 6),
    # reduced-size relatives used by the parity tests (ragged tails, several tiles)
    "small_bf16": Workload("small_bf16", 1, 2, 128, (3, 10, 37), "bf16", 0.10, 0.10,
                           seed=BASE_SEED + 11),
    "small_bf16_d64": Workload("small_bf16_d64", 1, 3, 64, (2, 11, 41), "bf16", 0.12, 0.15,
                               seed=BASE_SEED + 13),
    "small_fp32": Workload("small_fp32", 2, 2, 64, (2, 9, 29), "fp32", 0.15, 0.20,
                           v_white=True, unit_var=False, seed=BASE_SEED + 12),
}

SWEEP_KH = (0.025, 0.05, 0.10, 0.20, 1.0)


def sweep(k_h: float) -> Workload:
    """Sparsity-sweep member on the Wan-shaped layer (k_l = 10 %, 0 when dense)."""
    return replace(WORKLOADS["wan"], name=f"wan_kh{k_h:g}", k_h=k_h,
                   k_l=0.0 if k_h >= 1.0 else 0.10)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def _positions(grid: Tuple[int, int, int]) -> np.ndarray:
    tg, hg, wg = grid
    t, y, x = np.meshgrid(np.arange(tg), np.arange(hg), np.arange(wg), indexing="ij")
    p = np.stack([t.ravel() / tg, y.ravel() / hg, x.ravel() / wg], axis=1)
    return p.astype(np.float64)


def make_head(w: Workload, b: int, h: int, with_dO: bool = True) -> Dict[str, np.ndarray]:
    """Q, K, V (and dO) of one (batch, head): float32 arrays of shape [N, d]."""
    rng = np.random.Generator(np.random.PCG64([w.seed, b, h]))
    N, d = w.N, w.d
    omega = rng.standard_normal((8, 3))
    beta = rng.uniform(0.0, 2.0 * math.pi, size=8)
    G = {k: rng.standard_normal((8, d)) * math.sqrt(1.0 / 8.0) for k in ("Q", "K", "V")}
    p = _positions(w.grid)
    F = (math.sqrt(2.0) * np.cos(2.0 * math.pi * (p @ omega.T) + beta)).astype(np.float32)
    out: Dict[str, np.ndarray] = {}
    for k in ("Q", "K", "V"):
        noise = rng.standard_normal((N, d), dtype=np.float32)
        if k == "V" and w.v_white:
            x = noise
        else:
            x = F @ G[k].astype(np.float32) + np.float32(0.3) * noise
            if w.unit_var:
                x = x * np.float32(1.0 / math.sqrt(1.09))
        out[k] = round_to_bf16(x) if w.dtype == "bf16" else np.ascontiguousarray(x, np.float32)
    if with_dO:
        r2 = np.random.Generator(np.random.PCG64([w.seed, b, h, 7]))
        g = r2.standard_normal((N, d), dtype=np.float32)
        out["dO"] = round_to_bf16(g) if w.dtype == "bf16" else g
    return out


def make_proj(w: Workload) -> np.ndarray:
    """Proj [d, d] float32 (bf16-representable when the workload is bf16)."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 1000003]))
    W = (rng.standard_normal((w.d, w.d)) * 0.02).astype(np.float32)
    return round_to_bf16(W) if w.dtype == "bf16" else W


def make_inputs(w: Workload, heads: Optional[Iterable[int]] = None,
                with_dO: bool = True) -> Dict[str, np.ndarray]:
    """All tensors of a workload as float32 arrays [B, H', N, d] (H' = selected heads).
    Every (batch, head) has its own generator, so the heads are drawn by a few threads."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    hs = list(range(w.H)) if heads is None else list(heads)
    names = ("Q", "K", "V") + (("dO",) if with_dO else ())
    out = {k: np.empty((w.B, len(hs), w.N, w.d), np.float32) for k in names}

    def one(bh):
        b, hi = bh
        t = make_head(w, b, hs[hi], with_dO)
        for k in names:
            out[k][b, hi] = t[k]

    jobs = [(b, hi) for b in range(w.B) for hi in range(len(hs))]
    nthr = max(1, min(8, len(jobs), os.cpu_count() or 1))
    if nthr == 1 or w.N * w.d < (1 << 20):
        for j in jobs:
            one(j)
    else:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(one, jobs))
    out["Proj"] = make_proj(w)
    return out
