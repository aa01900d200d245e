"""Seeded synthetic inputs for the linear-attention operator.

This module only draws random numbers and packs them into the stored dtype
(fp32 arrays, or bf16 bit patterns held as uint16).  It contains none of the
operator's arithmetic, so the CPU oracle and the HIP path can both consume the
very same bits without sharing any code of the method itself.

The shapes follow the video-token counts of the paper's two model sizes
(21 latent frames; 832x480 and 1280x720 frames patchified to 30x52 and 45x80
tokens, Sec. 5.1 / App. A); head count and head width are those of the public
Wan architectures.  Values are synthetic: N(0,1)/sqrt(d) activations with a
per-head scale drawn from U(0.5, 2) and, for the large shapes, 0.1 % outlier
tokens at 20x magnitude.  The feature-map matrices W~_q, W~_k (Eq. 5) are
N(0,1) because trained ones are not available.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

__all__ = [
    "CONFIGS", "Inputs", "generate", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "stored_to_f32",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (round-to-nearest-even), return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def stored_to_f32(a: np.ndarray) -> np.ndarray:
    """fp32 view of a stored tensor (uint16 = bf16 bits, float32 = itself)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a)
    return np.asarray(a, dtype=np.float32)


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    H: int
    n: int
    d: int
    dtype: str                 # "f32" or "bf16": storage type of q, k, v, out and W~
    seeds: tuple               # one seed per batch item
    head_scale: bool           # per-head, per-tensor scale ~ U(0.5, 2)
    outlier_frac: float        # fraction of token rows multiplied by 20
    with_dout: bool = False    # also draw an upstream gradient ~ N(0, 0.1^2)


CONFIGS: Dict[str, Config] = {
    # tiny case a brute-force O(n^2) evaluation finishes in seconds
    "C1": Config("C1", 1, 2, 1024, 64, "f32", (1001,), False, 0.0),
    # Wan-1.3B layer at 480p: 21 x 30 x 52 tokens
    "C2": Config("C2", 1, 12, 32760, 128, "bf16", (1002,), True, 0.0),
    # Wan-14B layer at 720p: 21 x 45 x 80 tokens, plus outlier tokens
    "C3": Config("C3", 1, 40, 75600, 128, "bf16", (1003,), True, 0.001),
    # classifier-free-guidance pair, each item seeded on its own
    "C4": Config("C4", 2, 40, 75600, 128, "bf16", (1004, 1005), True, 0.001),
    # post-training step (forward + backward) at the 1.3B shape
    "C5": Config("C5", 1, 12, 32760, 128, "bf16", (1006,), True, 0.0, True),
    # second architecture (the paper's App. on CogVideoX-2B: 30 heads of width 64; 49 frames at
    # 480 x 720 -> 13 x 30 x 45 latent patches): exercises the d = 64 kernels at a real shape
    "C6": Config("C6", 1, 30, 17550, 64, "bf16", (1007,), True, 0.0),
}


@dataclass
class Inputs:
    cfg: Config
    B: int
    H: int
    n: int
    d: int
    dtype: str
    q: np.ndarray              # [B, H, n, d] stored dtype
    k: np.ndarray
    v: np.ndarray
    wq: np.ndarray             # [H, d, d/2] stored dtype
    wk: np.ndarray
    dout: Optional[np.ndarray] = None
    outlier_rows: List[np.ndarray] = field(default_factory=list)


def _pack(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    return np.ascontiguousarray(x32, dtype=np.float32)


def generate(name: str, *, n: Optional[int] = None, H: Optional[int] = None,
             B: Optional[int] = None, d: Optional[int] = None,
             dtype: Optional[str] = None, with_dout: Optional[bool] = None) -> Inputs:
    """Draw the inputs of configuration `name`.

    The keyword overrides shrink (or re-type) a configuration while keeping its
    value recipe; a shrunk tensor is NOT a prefix of the full one.
    """
    cfg = CONFIGS[name]
    B_ = cfg.B if B is None else B
    H_ = cfg.H if H is None else H
    n_ = cfg.n if n is None else n
    d_ = cfg.d if d is None else d
    dt = cfg.dtype if dtype is None else dtype
    want_dout = cfg.with_dout if with_dout is None else with_dout
    assert dt in ("f32", "bf16") and d_ % 2 == 0
    seeds = list(cfg.seeds) + [cfg.seeds[-1] + 7919 * (i + 1) for i in range(max(0, B_ - len(cfg.seeds)))]

    store = np.uint16 if dt == "bf16" else np.float32
    q = np.empty((B_, H_, n_, d_), store)
    k = np.empty_like(q)
    v = np.empty_like(q)
    dout = np.empty_like(q) if want_dout else None
    outlier_rows: List[np.ndarray] = []
    inv_sqrt_d = np.float32(1.0 / np.sqrt(d_))

    # W~ belongs to the layer, not to a batch item: drawn from the first seed.
    root0 = np.random.Generator(np.random.Philox(seeds[0]))
    g_q, g_k, g_v, g_wq, g_wk, g_scale, g_out, g_do = root0.spawn(8)
    wq = _pack(g_wq.standard_normal((H_, d_, d_ // 2), dtype=np.float32), dt)
    wk = _pack(g_wk.standard_normal((H_, d_, d_ // 2), dtype=np.float32), dt)

    for b in range(B_):
        if b > 0:
            root = np.random.Generator(np.random.Philox(seeds[b]))
            g_q, g_k, g_v, _, _, g_scale, g_out, g_do = root.spawn(8)
        if cfg.head_scale:
            scales = g_scale.uniform(0.5, 2.0, size=(3, H_)).astype(np.float32)
        else:
            scales = np.ones((3, H_), np.float32)
        n_out = int(np.ceil(cfg.outlier_frac * n_)) if cfg.outlier_frac > 0 else 0
        rows = np.sort(g_out.choice(n_, size=n_out, replace=False)) if n_out else np.zeros(0, np.int64)
        outlier_rows.append(rows)
        # one child stream per (tensor, head): heads can be drawn in parallel and a head's
        # values do not depend on how many heads are generated
        jobs = []
        for ti, (gen, dst) in enumerate(((g_q, q), (g_k, k), (g_v, v))):
            for h, child in enumerate(gen.spawn(H_)):
                jobs.append((child, dst, h, inv_sqrt_d * scales[ti, h], True))
        if want_dout:
            for h, child in enumerate(g_do.spawn(H_)):
                jobs.append((child, dout, h, np.float32(0.1), False))

        def draw(job, b=b, rows=rows, n_out=n_out):
            child, dst, h, mul, outliers = job
            x = child.standard_normal((n_, d_), dtype=np.float32)
            x *= mul
            if outliers and n_out:
                x[rows] *= np.float32(20.0)
            dst[b, h] = _pack(x, dt)

        if len(jobs) * n_ * d_ > (1 << 22):
            with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
                list(ex.map(draw, jobs))
        else:
            for j in jobs:
                draw(j)

    return Inputs(cfg, B_, H_, n_, d_, dt, q, k, v, wq, wk, dout, outlier_rows)
