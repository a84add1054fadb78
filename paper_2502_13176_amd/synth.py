"""Seeded synthetic workloads: shapes, importance scores, K/V/Q payloads.

This module is the one piece shared by the CPU oracle's tests and the GPU
path's tests/bench.  It holds no arithmetic of the method itself: no
attention, no eviction, no budget rounding.  Budget allocators are passed in
as callables so each side plugs in its own.

The workloads stand in for the paper's evaluation setting (LLaMA-3-8B at
context 8192 and Qwen2.5-7B at context 32768, Results section): only the
cache *shapes* matter to the hot path, so K/V/Q are N(0,1) draws rounded to
bf16 and importance scores are drawn from heavy-tailed distributions that
give the ragged per-head budgets the paper's allocation produces.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Callable, List, Optional, Sequence

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    Hq: int
    Hkv: int
    D: int
    batch: int
    ctx: int
    dtype: str                      # "bf16" | "f32"
    seed: int
    keep_pct: int                   # percent of L*Hkv*ctx tokens kept globally
    lo: int
    hi: int
    importance: str                 # "fixed" | "lognormal" | "pareto"
    sigma: float = 1.0
    alpha: float = 1.2
    fixed_budgets: Optional[Sequence[int]] = None
    floor_frac: float = 0.0         # fraction of heads pinned to `lo` (lowest importance)
    sink: int = 4
    recent: int = 64
    interval: int = 64              # decode steps between compactions
    slack: int = 64                 # capacity beyond budget per cache
    scores: str = "uniform"         # "uniform" | "kernel"
    steps: int = 128

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def m(self) -> int:
        return self.L * self.Hkv

    @property
    def n_caches(self) -> int:
        return self.L * self.batch * self.Hkv

    @property
    def global_budget(self) -> int:
        return (self.m * self.ctx * self.keep_pct) // 100

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def token_bytes(self) -> int:
        """K row + V row of one cached token of one KV head."""
        return 2 * self.D * self.elem_bytes


# The five workloads named by the benchmark definition.  "compression X%" is
# read as X% of tokens evicted, i.e. keep_pct = 100 - X.
WORKLOADS = {
    "tiny": Workload("tiny", L=1, Hq=4, Hkv=2, D=64, batch=1, ctx=256, dtype="f32", seed=1000,
                     keep_pct=50, lo=64, hi=192, importance="fixed", fixed_budgets=(64, 192),
                     sink=4, recent=16, interval=1, slack=256, steps=1),
    "llama1": Workload("llama1", L=1, Hq=32, Hkv=8, D=128, batch=1, ctx=8192, dtype="bf16",
                       seed=1001, keep_pct=50, lo=256, hi=8192, importance="lognormal", sigma=1.0,
                       steps=1),
    "llama32": Workload("llama32", L=32, Hq=32, Hkv=8, D=128, batch=8, ctx=32768, dtype="bf16",
                        seed=1002, keep_pct=30, lo=128, hi=32768, importance="lognormal",
                        sigma=1.5, interval=64, slack=64, steps=128),
    "qwen": Workload("qwen", L=28, Hq=28, Hkv=4, D=128, batch=16, ctx=32768, dtype="bf16",
                     seed=1003, keep_pct=50, lo=128, hi=32768, importance="lognormal", sigma=1.0,
                     floor_frac=0.10, interval=64, slack=64, steps=128),
    "long": Workload("long", L=32, Hq=32, Hkv=8, D=128, batch=4, ctx=131072, dtype="bf16",
                     seed=1004, keep_pct=15, lo=256, hi=131072, importance="pareto", alpha=1.2,
                     interval=32, slack=32, scores="kernel", steps=256),
}
WORKLOAD_ORDER = ["tiny", "llama1", "llama32", "qwen", "long"]


def shrink(w: Workload, **kw) -> Workload:
    """A smaller replica of a workload (fewer layers / sequences / shorter context)."""
    return replace(w, **kw)


def importance_scores(w: Workload) -> np.ndarray:
    """One positive fp64 importance score per (layer, KV head), layer-major."""
    rng = np.random.Generator(np.random.PCG64(w.seed))
    if w.importance == "lognormal":
        return rng.lognormal(0.0, w.sigma, w.m)
    if w.importance == "pareto":
        return 1.0 + rng.pareto(w.alpha, w.m)
    if w.importance == "fixed":
        return np.asarray(w.fixed_budgets, dtype=np.float64)
    raise ValueError(w.importance)


AllocFn = Callable[[Sequence[float], int, int, int], List[int]]


def budgets_for(w: Workload, alloc_proportional: AllocFn) -> List[int]:
    """Per-(layer, KV head) token budgets for a workload, using the caller's allocator.

    When `floor_frac` > 0 the round(floor_frac*m) lowest-importance heads are
    set to `lo` and the remaining heads share what is left.
    """
    if w.importance == "fixed":
        reps = w.m // len(w.fixed_budgets)
        return [int(b) for b in w.fixed_budgets] * reps
    imp = importance_scores(w)
    m = w.m
    n_floor = int(round(w.floor_frac * m))
    if n_floor == 0:
        return list(alloc_proportional(imp, w.global_budget, w.lo, w.hi))
    order = sorted(range(m), key=lambda i: (imp[i], i))
    pinned = set(order[:n_floor])
    rest = [i for i in range(m) if i not in pinned]
    sub = alloc_proportional(imp[rest], w.global_budget - n_floor * w.lo, w.lo, w.hi)
    out = [w.lo] * m
    for i, b in zip(rest, sub):
        out[i] = int(b)
    return out


# ---------------------------------------------------------------------------
# bf16 bit patterns (round-to-nearest-even), as the payload generator emits them
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def payload(rng: np.random.Generator, shape, dtype: str, peaked: bool = False) -> np.ndarray:
    """N(0,1) draws in storage format: fp32 array for "f32", uint16 bf16 bits for "bf16".

    `peaked` scales about 1% of the rows by 8 so a few logits dominate.
    """
    x = rng.standard_normal(shape, dtype=np.float32)
    if peaked and x.ndim >= 2:
        rows = rng.random(x.shape[:-1]) < 0.01
        x[rows] *= 8.0
    if dtype == "f32":
        return x
    return f32_to_bf16_bits(x)


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage-format array to fp64."""
    if dtype == "f32":
        return a.astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


def uniform_scores(rng: np.random.Generator, n: int) -> np.ndarray:
    return rng.random(n, dtype=np.float32)


def fill_arena_on_device(arena, w: Workload):
    """Fills the K/V/score/pos planes of a device arena (an object with torch tensors k, v, score,
    pos and numpy tables off_host, cap_host) with the seeded payload, generated on the device in
    slabs: N(0,1) rounded to the storage type, scores U(0,1) or zero, pos = row index inside its
    cache.  Returns the torch generator so that further inputs continue the same stream."""
    import torch
    g = torch.Generator(device=arena.device)
    g.manual_seed(w.seed)
    slab = 1 << 22  # rows
    for plane in (arena.k, arena.v):
        for r0 in range(0, arena.total_tokens, slab):
            r1 = min(arena.total_tokens, r0 + slab)
            x = torch.randn((r1 - r0, w.D), generator=g, device=arena.device, dtype=torch.float32)
            plane[r0:r1].copy_(x)
            del x
    if w.scores == "uniform":
        arena.score.copy_(torch.rand((arena.total_tokens,), generator=g, device=arena.device, dtype=torch.float32))
    else:
        arena.score.zero_()
    off = torch.from_numpy(arena.off_host).to(arena.device)
    cap = torch.from_numpy(arena.cap_host).to(arena.device).to(torch.int64)
    starts = torch.repeat_interleave(off, cap)
    arena.pos.copy_((torch.arange(arena.total_tokens, device=arena.device) - starts).to(torch.int32))
    return g
