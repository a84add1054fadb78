"""Helpers for the GPU parity tests: build an arena through the binding, fill it with the seeded
payload, and mirror it into oracle caches.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

ATTN_TOL = 2e-3      # max-abs error of attention outputs: bf16 in, fp32 accumulate (benchmark definition)


def to_device_storage(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).to(device).view(torch.bfloat16)


def from_device_storage(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def make_arena(w: synth.Workload, budgets: Optional[Sequence[int]] = None, track: bool = False,
               policy: int = B.POLICY_SCORE, slack: Optional[int] = None) -> B.Arena:
    if budgets is None:
        budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = B.Arena(w.L, w.Hq, w.Hkv, w.D, w.batch, w.dtype, budgets, w.slack if slack is None else slack,
                    w.sink, w.recent, policy, track, workspace_fill=0xFF)
    # Rows beyond a cache's live length must never reach a result, and the library must not count on
    # a zeroed workspace: everything starts out as NaN (K, V, scores), -1 (positions) and 0xFF bytes.
    arena.k.fill_(float("nan"))
    arena.v.fill_(float("nan"))
    arena.score.fill_(float("nan"))
    arena.pos.fill_(-1)
    return arena


class HostState:
    """Host copy of an arena's live rows in storage format, per cache."""

    def __init__(self, n_caches: int):
        self.K: List[np.ndarray] = [None] * n_caches
        self.V: List[np.ndarray] = [None] * n_caches
        self.score: List[np.ndarray] = [None] * n_caches
        self.pos: List[np.ndarray] = [None] * n_caches

    def lens(self) -> List[int]:
        return [k.shape[0] for k in self.K]


def fill_from_host(arena: B.Arena, w: synth.Workload, lens: Sequence[int], rng: np.random.Generator,
                   scores: str = "zero", peaked: bool = False, scale: float = 1.0) -> HostState:
    """Seeded payload for every cache, uploaded in one copy per plane.  Small arenas only."""
    st = HostState(arena.n_caches)
    sdt = np.float32 if w.dtype == "f32" else np.uint16
    nan = np.float32(np.nan) if w.dtype == "f32" else np.uint16(0x7FC0)      # rows past the live length stay NaN
    Kh = np.full((arena.total_tokens, w.D), nan, dtype=sdt)
    Vh = np.full((arena.total_tokens, w.D), nan, dtype=sdt)
    Sh = np.full((arena.total_tokens,), np.nan, dtype=np.float32)
    Ph = np.full((arena.total_tokens,), -1, dtype=np.int32)
    for c in range(arena.n_caches):
        n = int(lens[c])
        assert n <= arena.cap_host[c]
        if scale == 1.0:
            k = synth.payload(rng, (n, w.D), w.dtype, peaked)
        else:
            x = (rng.standard_normal((n, w.D)) * scale).astype(np.float32)
            k = x if w.dtype == "f32" else synth.f32_to_bf16_bits(x)
        v = synth.payload(rng, (n, w.D), w.dtype)
        s = synth.uniform_scores(rng, n) if scores == "uniform" else np.zeros(n, dtype=np.float32)
        ps = np.arange(n, dtype=np.int32)
        o = int(arena.off_host[c])
        Kh[o:o + n], Vh[o:o + n], Sh[o:o + n], Ph[o:o + n] = k, v, s, ps
        st.K[c], st.V[c], st.score[c], st.pos[c] = k, v, s, ps
    arena.k.copy_(to_device_storage(Kh, w.dtype, arena.device))
    arena.v.copy_(to_device_storage(Vh, w.dtype, arena.device))
    arena.score.copy_(torch.from_numpy(Sh).to(arena.device))
    arena.pos.copy_(torch.from_numpy(Ph).to(arena.device))
    torch.cuda.synchronize()
    arena.set_lengths(lens)
    return st


def download(arena: B.Arena, w: synth.Workload, caches: Optional[Sequence[int]] = None, flush: bool = True) -> HostState:
    """Live rows of the given caches as the device holds them now.  With score tracking the weights of
    the latest attention call may still be owed to the score plane: baklava_flush_scores adds them first
    (flush=False reads the plane as it stands)."""
    if flush:
        arena.flush_scores(0, arena.L)
    torch.cuda.synchronize()
    lens = arena.len.cpu().numpy()
    st = HostState(arena.n_caches)
    for c in (range(arena.n_caches) if caches is None else caches):
        o, n = int(arena.off_host[c]), int(lens[c])
        st.K[c] = from_device_storage(arena.k[o:o + n], w.dtype)
        st.V[c] = from_device_storage(arena.v[o:o + n], w.dtype)
        st.score[c] = arena.score[o:o + n].cpu().numpy()
        st.pos[c] = arena.pos[o:o + n].cpu().numpy()
    return st


def oracle_cache(w: synth.Workload, st: HostState, c: int) -> O.Cache:
    oc = O.Cache(w.D)
    oc.load(synth.storage_to_f64(st.K[c], w.dtype), synth.storage_to_f64(st.V[c], w.dtype),
            st.score[c].astype(np.float64), st.pos[c])
    return oc


def make_q(w: synth.Workload, rng: np.random.Generator, layers: int, scale: float = 1.0):
    """Query block [layers, batch, Hq, D] in storage format and as fp64."""
    shape = (layers, w.batch, w.Hq, w.D)
    if scale == 1.0:
        q = synth.payload(rng, shape, w.dtype)
    else:
        x = (rng.standard_normal(shape) * scale).astype(np.float32)
        q = x if w.dtype == "f32" else synth.f32_to_bf16_bits(x)
    return q, synth.storage_to_f64(q, w.dtype)


def q_rows_of_cache(w: synth.Workload, c: int, layer_begin: int = 0):
    """Index (layer_rel, b, slice of query heads) of the G query rows that read cache c."""
    cpl = w.batch * w.Hkv
    l, rem = divmod(c, cpl)
    b, h = divmod(rem, w.Hkv)
    return l - layer_begin, b, slice(h * w.G, (h + 1) * w.G)


def gpu_decode(arena: B.Arena, w: synth.Workload, q_storage: np.ndarray, layer_begin: int = 0,
               layer_count: Optional[int] = None) -> np.ndarray:
    layer_count = w.L if layer_count is None else layer_count
    qd = to_device_storage(q_storage, w.dtype, arena.device)
    out = torch.full((layer_count, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
    arena.decode_attn(layer_begin, layer_count, qd, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def check_decode_against_oracle(arena, w, st: HostState, q64: np.ndarray, out_gpu: np.ndarray,
                                caches: Optional[Sequence[int]] = None, layer_begin: int = 0,
                                tol: float = ATTN_TOL) -> float:
    worst = 0.0
    for c in (range(arena.n_caches) if caches is None else caches):
        l, b, hs = q_rows_of_cache(w, c, layer_begin)
        ref, _ = O.decode_attn(q64[l, b, hs], synth.storage_to_f64(st.K[c], w.dtype),
                               synth.storage_to_f64(st.V[c], w.dtype))
        err = float(np.max(np.abs(out_gpu[l, b, hs] - ref)))
        assert np.all(np.isfinite(out_gpu[l, b, hs])), f"cache {c}: non-finite output"
        assert err <= tol, f"cache {c} (n={st.K[c].shape[0]}): max-abs error {err:.3e} > {tol}"
        worst = max(worst, err)
    return worst


def set_chunk(arena: B.Arena, chunk: int) -> None:
    """Rows per split-K work item, for both kinds of launch (layer sub-range and whole model)."""
    arena.set_option(B.OPT_CHUNK_TOKENS, chunk)
    arena.set_option(B.OPT_CHUNK_TOKENS_WHOLE, chunk)


def check_step_against_oracle(arena, w, pre: HostState, post: HostState, out: np.ndarray, q64: np.ndarray,
                              k64: np.ndarray, v64: np.ndarray, token_pos: int, t: int, caches: Sequence[int],
                              score_tol: float = 2e-3):
    """Step-local check of one decode step (append, attention, score update) on the given caches: the
    oracle starts from the device's own pre-step state, recomputes the step in fp64, and the device's
    outputs, appended rows and post-step scores must agree.  Returns (worst output error, worst score error)."""
    worst_out = worst_score = 0.0
    for c in caches:
        l, b, hs = q_rows_of_cache(w, c)
        h = c % w.Hkv
        oc = oracle_cache(w, pre, c)
        ref, _, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, h], v64[l, b, h], token_pos, t,
                                  budget=0, sink=0, recent=0, interval=0, track_scores=True)
        assert post.K[c].shape[0] == pre.K[c].shape[0] + 1 and post.pos[c][-1] == token_pos, f"step {t} cache {c}"
        err = float(np.max(np.abs(out[l, b, hs] - ref)))
        assert err <= ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
        serr = np.abs(post.score[c].astype(np.float64) - oc.score)
        assert np.all((serr <= score_tol) | (serr <= score_tol * np.abs(oc.score))), \
            f"step {t} cache {c}: score error {serr.max():.3e}"
        worst_out, worst_score = max(worst_out, err), max(worst_score, float(serr.max()))
    return worst_out, worst_score


def check_eviction_against_oracle(arena, w, budgets, post: HostState, after: HostState, kept_dev, caches: Sequence[int]):
    """The oracle's selection on the device's own fp32 post-step scores must give the device's kept
    list, and the surviving rows must be the selected ones, bit for bit."""
    cpl = w.batch * w.Hkv
    for c in caches:
        bud = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
        kept = O.compact_select(post.score[c], post.K[c].shape[0], bud, w.sink, w.recent)
        o = int(arena.off_host[c])
        assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32)), f"cache {c}: kept list"
        idx = np.asarray(kept)
        assert after.K[c].shape[0] == len(kept) == min(post.K[c].shape[0], bud)
        assert np.array_equal(after.K[c], post.K[c][idx]) and np.array_equal(after.V[c], post.V[c][idx])
        assert np.array_equal(after.score[c].view(np.uint32), post.score[c][idx].view(np.uint32))
        assert np.array_equal(after.pos[c], post.pos[c][idx])
