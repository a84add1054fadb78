"""CPU oracle for the ragged per-head KV-cache decode path (BaKlaVa, arXiv 2502.13176).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 statement of what
the hot path computes.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product (the HIP library and its Python
binding) never does, and this file imports nothing from the product.

Each function cites the passage of the paper it follows.  Where the paper is
silent the reading taken is stated in the docstring.

Pins (see tests/test_oracle_*.py):
  decode_attn            pure-Python brute force, closed forms, torch fp64 SDPA,
                         shift/permutation invariances
  score_accumulate       closed form sum = G per step
  compact_select/apply   brute-force full sort, structural invariants
  alloc_proportional     exact-rational water-filling, invariants
  alloc_threshold        conservation + structure only: the paper prints no
                         worked example of Algorithm 2 -> beyond those
                         invariants PARITY UNPINNED
  head_similarity        pure-Python brute force, closed forms (one token, two
                         tokens, uniform attention = prefix means, identity
                         attention), scale invariance, torch fp64 causal SDPA
  kv_importance          hand-computed values, range and monotonicity
  layer_similarity       closed forms (identical, opposite, orthogonal rows), brute
                         force, torch fp64 cosine_similarity, scale invariance
  alloc_two_level        conservation per layer and overall, reduction to its two
                         building blocks; the paper does not say how layer scores
                         become layer budgets -> the composition is a reading,
                         PARITY UNPINNED beyond those invariants
  prefill_scores         pure-Python brute force, total mass G*T, harmonic closed
                         form for uniform attention, torch fp64 softmax of the
                         masked logits, consistency with decode_attn's weights
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

FRAC_BITS = 40  # fixed-point fraction bits of the proportional allocator's weights


# ---------------------------------------------------------------------------
# Budget allocation (host step, once per model)
# ---------------------------------------------------------------------------

def alloc_proportional(importance: Sequence[float], global_budget: int, lo: int, hi: int) -> List[int]:
    """Budgets proportional to importance, clipped to [lo, hi], summing exactly to global_budget.

    The paper assigns larger caches to more important KV heads (Methods,
    "Assigning Memory Budgets to KV-Caches") but prints no proportional rule;
    the benchmark workloads ask for one.  Reading taken, chosen so that integer
    arithmetic alone decides every rounding:

      w_i = max(1, floor(I_i / max(I) * 2^40))
      x_i(lam) = floor(lam * w_i / 2^40),  f(lam) = sum_i clip(x_i, lo, hi)
      lam* = largest integer lam with f(lam) <= B
      b_i = clip(x_i(lam*), lo, hi); the B - sum(b) leftover tokens go, one
      each, to the heads with lo <= x_i < hi having the largest
      (lam*·w_i mod 2^40, w_i, -i).
    """
    imp = [float(v) for v in importance]
    m = len(imp)
    B = int(global_budget)
    if m == 0 or lo < 0 or hi < lo:
        raise ValueError("bad arguments")
    if any((not math.isfinite(v)) or v <= 0.0 for v in imp):
        raise ValueError("importance must be finite and positive")
    if m * lo > B or m * hi < B:
        raise ValueError("infeasible budget")
    one = 1 << FRAC_BITS
    top = max(imp)
    w = [max(1, int(math.floor((v / top) * float(one)))) for v in imp]

    def clip(x: int) -> int:
        return lo if x < lo else (hi if x > hi else x)

    def f(lam: int) -> int:
        return sum(clip((lam * wi) >> FRAC_BITS) for wi in w)

    lam_hi = ((hi << FRAC_BITS) // min(w)) + 1      # every x_i >= hi here
    if f(lam_hi) <= B:
        lam = lam_hi
    else:
        a, z = 0, lam_hi                            # f(a) <= B < f(z)
        while z - a > 1:
            mid = (a + z) // 2
            if f(mid) <= B:
                a = mid
            else:
                z = mid
        lam = a
    x = [(lam * wi) >> FRAC_BITS for wi in w]
    b = [clip(xi) for xi in x]
    left = B - sum(b)
    elig = [i for i in range(m) if lo <= x[i] < hi]
    assert 0 <= left <= len(elig)
    elig.sort(key=lambda i: ((lam * w[i]) & (one - 1), w[i], -i), reverse=True)
    for i in elig[:left]:
        b[i] += 1
    return b


def alloc_threshold(importance: Sequence[float], size_in: Sequence[int], t: float, r: float) -> List[int]:
    """Algorithm 2 (KV-cache memory reallocation by attention-head importance).

    Caches whose importance is below t give up a fraction r of their current
    size; what they free is shared by the k = min(n, m - n) most important of
    the remaining caches (n = number of reduced caches).

    Readings where the listing is ambiguous: the "all low" guard |L| > m-1
    means |L| = m; an empty low set also returns the input unchanged (the
    listing would divide 0 by 0); r is a fraction of the cache's size and the
    reduction is floor(r*size); the top-k set is drawn from the caches that
    were not reduced, ties to the lower index; the freed total F is split as
    floor(F/k) each with the remainder going one token apiece to the most
    important first; increased caches are not clipped to the context length.
    """
    imp = [float(v) for v in importance]
    size = [int(s) for s in size_in]
    m = len(imp)
    if len(size) != m:
        raise ValueError("length mismatch")
    if not (0.0 <= r <= 1.0):
        raise ValueError("r must be in [0,1]")
    if not math.isfinite(t) or not all(math.isfinite(v) for v in imp):
        raise ValueError("importances and threshold must be finite: the algorithm orders and compares them")
    low = [i for i in range(m) if imp[i] < t]
    n = len(low)
    if n == m or n == 0:
        return size
    freed = 0
    for i in low:
        d = int(math.floor(r * size[i]))
        size[i] -= d
        freed += d
    k = min(n, m - n)
    lowset = set(low)
    high = [i for i in range(m) if i not in lowset]
    high.sort(key=lambda i: (-imp[i], i))
    chosen = high[:k]
    base, rem = divmod(freed, k)
    for rank, j in enumerate(chosen):
        size[j] += base + (1 if rank < rem else 0)
    return size


def layout(budget: Sequence[int], L: int, Hkv: int, batch: int, slack: int) -> Tuple[List[int], List[int], int]:
    """Capacity and start offset (in tokens) of every cache, cache id c = (l*batch + b)*Hkv + h.

    A cache of budget b_c has room for b_c + slack rows (the rows appended
    between two compactions); offsets are the exclusive prefix sum.  Budgets
    depend on (layer, head) only: they are a property of the model (Methods,
    first paragraphs), so every sequence of the batch uses the same ones.
    """
    off, cap, total = [], [], 0
    for l in range(L):
        for b in range(batch):
            for h in range(Hkv):
                c = int(budget[l * Hkv + h]) + slack
                off.append(total)
                cap.append(c)
                total += c
    return off, cap, total


# ---------------------------------------------------------------------------
# Decode attention over one cache (Eq. 1 scaled dot-product attention, applied
# to the single query row of Eq. 4 / Eq. 7 over the reduced cache)
# ---------------------------------------------------------------------------

def decode_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """softmax(q K^T / sqrt(D)) V for the G query heads sharing one KV head.

    q [G, D], K [n, D], V [n, D], all fp64 holding the exact values of the
    stored inputs.  The cache already contains the current token's row (the
    concatenation [K'; K_t] of Eq. 7), and a decode query sees every row: no
    mask.  Returns (out [G, D], p [G, n]).
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    G, D = q.shape
    n = K.shape[0]
    if n == 0:
        raise ValueError("attention over an empty cache")
    out = np.zeros((G, D), dtype=np.float64)
    p = np.zeros((G, n), dtype=np.float64)
    for g in range(G):
        s = (K @ q[g]) / math.sqrt(D)       # s_j = q_g . k_j / sqrt(D_h)
        e = np.exp(s - np.max(s))
        p[g] = e / np.sum(e)
        out[g] = p[g] @ V
    return out, p


def score_accumulate(score: np.ndarray, p: np.ndarray) -> np.ndarray:
    """Cumulative attention per cached token (the heavy-hitter statistic, Related Work:
    eviction by cumulative attention).  For grouped-query attention the weights of the G
    query heads sharing the cache are summed: score_j += sum_g p[g, j]."""
    return np.asarray(score, dtype=np.float64) + np.sum(p, axis=0)


# ---------------------------------------------------------------------------
# Budget-enforcing eviction (f_evict, Eqs. 5-6: removed tokens vanish, the
# survivors keep their order)
# ---------------------------------------------------------------------------

POLICY_SCORE = 0       # sink + recent + top-scored middle tokens
POLICY_STREAMING = 1   # sink + most recent tokens only (the policy the paper evaluated with)


def compact_select(score: np.ndarray, n: int, budget: int, sink: int, recent: int,
                   policy: int = POLICY_SCORE) -> List[int]:
    """Ascending list of the row indices that survive eviction down to `budget`.

    n <= budget: nothing is evicted.  Otherwise the first `sink` rows and the
    last `recent` rows always survive and the remaining budget - sink - recent
    places go to the middle rows with the largest accumulated score; equal
    scores: the older row (lower index) wins.  Scores are compared as fp32
    values, the precision the kernel stores them in.  Streaming policy: sink
    rows plus the budget - sink most recent rows.
    """
    if n <= budget:
        return list(range(n))
    if policy == POLICY_STREAMING:
        if budget < sink:
            raise ValueError("budget < sink")
        recent = budget - sink
    if budget < sink + recent:
        raise ValueError("budget < sink + recent")
    k = budget - sink - recent
    mid = list(range(sink, n - recent))
    s32 = np.asarray(score[:n], dtype=np.float32)
    if np.any(np.isnan(s32)):
        raise ValueError("NaN score")
    mid.sort(key=lambda j: (-float(s32[j]), j))
    kept = list(range(sink)) + mid[:k] + list(range(n - recent, n))
    kept.sort()
    return kept


class Cache:
    """One (sequence, layer, KV head) cache: rows in arrival order after eviction."""

    def __init__(self, D: int):
        self.K = np.zeros((0, D), dtype=np.float64)
        self.V = np.zeros((0, D), dtype=np.float64)
        self.score = np.zeros((0,), dtype=np.float64)
        self.pos = np.zeros((0,), dtype=np.int64)

    @property
    def n(self) -> int:
        return self.K.shape[0]

    def append(self, k_row: np.ndarray, v_row: np.ndarray, token_pos: int) -> None:
        """[K'; K_t], [V'; V_t] of Eq. 7: the new token's row goes last, its score starts at 0."""
        self.K = np.vstack([self.K, np.asarray(k_row, dtype=np.float64)[None, :]])
        self.V = np.vstack([self.V, np.asarray(v_row, dtype=np.float64)[None, :]])
        self.score = np.append(self.score, 0.0)
        self.pos = np.append(self.pos, np.int64(token_pos))

    def load(self, K: np.ndarray, V: np.ndarray, score: np.ndarray, pos: np.ndarray) -> None:
        self.K = np.array(K, dtype=np.float64)
        self.V = np.array(V, dtype=np.float64)
        self.score = np.array(score, dtype=np.float64)
        self.pos = np.array(pos, dtype=np.int64)

    def compact(self, budget: int, sink: int, recent: int, policy: int = POLICY_SCORE) -> List[int]:
        """Apply f_evict for every row not selected; returns the kept indices."""
        kept = compact_select(self.score, self.n, budget, sink, recent, policy)
        self.K = self.K[kept]
        self.V = self.V[kept]
        self.score = self.score[kept]
        self.pos = self.pos[kept]
        return kept


def decode_step(cache: Cache, q: np.ndarray, k_new, v_new, token_pos: int, step_index: int,
                budget: int, sink: int, recent: int, interval: int, track_scores: bool,
                policy: int = POLICY_SCORE):
    """One decode step on one cache: append -> attention -> score update -> compaction when
    step_index is a multiple of `interval`.  Returns (out [G,D], p [G,n], kept or None)."""
    if k_new is not None:
        cache.append(k_new, v_new, token_pos)
    out, p = decode_attn(q, cache.K, cache.V)
    if track_scores:
        cache.score = score_accumulate(cache.score, p)
    kept = None
    if interval > 0 and step_index % interval == 0:
        kept = cache.compact(budget, sink, recent, policy)
    return out, p, kept


# ---------------------------------------------------------------------------
# One-time profiling (Algorithm 1)
# ---------------------------------------------------------------------------

COS_EPS = 1e-8  # the product of the two norms is clamped from below by this value


def head_similarity(Q: np.ndarray, K: np.ndarray, V: np.ndarray) -> Tuple[float, np.ndarray]:
    """Algorithm 1, step 1, for one attention head and one prompt.

    Q, K, V: [T, D] (the head's query rows and the key / value rows of the KV
    head it reads).  For every prompt token t the head's output row is
    out_t = sum_{j<=t} softmax_j(q_t . k_j / sqrt(D)) v_j (Eq. 1 with the causal
    mask of autoregressive inference) and the token's similarity is the cosine
    between the head's input row v_t and out_t.  Returns (mean over tokens,
    per-token cosines).

    Readings: the mask is causal (the algorithm runs "inference" on the prompt);
    logits are scaled by 1/sqrt(D) as in Eq. 1; a cosine whose norm product is
    below COS_EPS divides by COS_EPS instead (so a zero row gives 0), the
    convention of the usual library routine, since the paper does not say.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    T, D = Q.shape
    if K.shape != (T, D) or V.shape != (T, D) or T < 1:
        raise ValueError("Q, K, V must all be [T, D] with T >= 1")
    cos = np.empty(T, dtype=np.float64)
    scale = 1.0 / math.sqrt(D)
    for t in range(T):
        s = (K[: t + 1] @ Q[t]) * scale
        w = np.exp(s - s.max())
        out = (w / w.sum()) @ V[: t + 1]
        denom = max(float(np.linalg.norm(V[t]) * np.linalg.norm(out)), COS_EPS)
        cos[t] = float(V[t] @ out) / denom
    return float(cos.mean()), cos


def kv_importance(similarity: np.ndarray, G: int) -> np.ndarray:
    """Algorithm 1, step 2, plus the normalisation of the text ("Head Importance Heuristic").

    similarity: [L, Hq] mean cosines in [-1, 1] (one prompt, or already averaged
    over prompts).  The G consecutive heads that share a KV cache are averaged,
    the mean is mapped from [-1, 1] to [0, 1], and importance is its complement:
    I[l, h] = 1 - (mean_g s[l, h*G + g] + 1) / 2.

    Reading: the map to [0, 1] is the affine one, (s + 1) / 2; the paper says
    "normalize these values from range 0 to 1" and prints no formula.  The map
    is applied after the group mean; being affine it commutes with the mean.
    """
    s = np.asarray(similarity, dtype=np.float64)
    L, Hq = s.shape
    if G < 1 or Hq % G:
        raise ValueError("Hq must be a multiple of G")
    grouped = s.reshape(L, Hq // G, G).mean(axis=2)
    return 1.0 - (grouped + 1.0) / 2.0


# ---------------------------------------------------------------------------
# Scores of a whole prompt at once (the eviction that precedes the decode loop)
# ---------------------------------------------------------------------------

def prefill_scores(Q: np.ndarray, K: np.ndarray) -> np.ndarray:
    """Accumulated attention of every prompt token after a prefill of T tokens.

    Q: [G, T, D] query rows of the G heads that share the cache, K: [T, D].
    score_j = sum_g sum_{t >= j} p_g[t, j] with p_g[t, :] = softmax over j <= t of
    q_g[t] . k_j / sqrt(D): the column sums of the causal attention matrices, i.e.
    exactly what score_accumulate would have built up had the T tokens been
    decoded one by one without eviction (the heavy-hitter statistic the paper
    cites as a compatible eviction policy, applied to f_evict of Eqs. 5-6 before
    the first decode step).  Returns [T] fp64.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    G, T, D = Q.shape
    if K.shape != (T, D) or T < 1:
        raise ValueError("Q must be [G, T, D] and K [T, D] with T >= 1")
    score = np.zeros(T, dtype=np.float64)
    scale = 1.0 / math.sqrt(D)
    for g in range(G):
        for t in range(T):
            s = (K[: t + 1] @ Q[g, t]) * scale
            w = np.exp(s - s.max())
            score[: t + 1] += w / w.sum()
    return score


# ---------------------------------------------------------------------------
# Layer importance ("Layer Importance Heuristic") and the two-level allocation
# ---------------------------------------------------------------------------

def layer_similarity(X_in: np.ndarray, X_out: np.ndarray) -> Tuple[float, np.ndarray]:
    """Cosine between the input and the output hidden state of a layer, token by token, and its mean
    over the prompt: the heuristic the paper adopts for layer importance ("Layer Importance
    Heuristic").  X_in, X_out: [T, H].  Zero rows are handled as in head_similarity (norm product
    clamped from below by COS_EPS).  Importance follows as for heads: 1 - (mean + 1) / 2
    (kv_importance with G = 1)."""
    A = np.asarray(X_in, dtype=np.float64)
    Bm = np.asarray(X_out, dtype=np.float64)
    if A.ndim != 2 or A.shape != Bm.shape or A.shape[0] < 1:
        raise ValueError("X_in and X_out must both be [T, H] with T >= 1")
    cos = np.empty(A.shape[0], dtype=np.float64)
    for t in range(A.shape[0]):
        denom = max(float(np.linalg.norm(A[t]) * np.linalg.norm(Bm[t])), COS_EPS)
        cos[t] = float(A[t] @ Bm[t]) / denom
    return float(cos.mean()), cos


def alloc_two_level(layer_importance: Sequence[float], head_importance: np.ndarray, global_budget: int,
                    lo: int, hi: int, t: float, r: float) -> List[int]:
    """Layer pool first, head pool second ("Layer Importance Heuristic" + "Memory Allocation").

    The paper obtains importances for layers and for the KV caches inside a layer, and prints
    Algorithm 2 for the caches of one layer; how the layer importances become layer pools is not
    stated.  Reading taken, built only from the two rules already defined here:
      1. layer pools: alloc_proportional over the L layer importances with the global budget and
         the bounds [Hkv*lo, Hkv*hi] (so every layer can give each of its caches between lo and hi);
      2. inside a layer: the pool is split equally over its Hkv caches, the remainder going one
         token each to the most important caches first (ties: lower index); then Algorithm 2
         (alloc_threshold) with threshold t and reduction fraction r moves memory from the caches
         below the threshold to the most important ones of that layer.
    head_importance: [L, Hkv].  Returns L*Hkv budgets, layer-major.  Each layer's budgets sum to
    its pool and all budgets sum to global_budget; the bounds lo/hi constrain the pools, not the
    budgets Algorithm 2 produces (it does not clip, see alloc_threshold).
    """
    himp = np.asarray(head_importance, dtype=np.float64)
    L, Hkv = himp.shape
    if len(layer_importance) != L:
        raise ValueError("one importance per layer expected")
    pools = alloc_proportional(layer_importance, global_budget, Hkv * lo, Hkv * hi)
    out: List[int] = []
    for l in range(L):
        base, rem = divmod(pools[l], Hkv)
        order = sorted(range(Hkv), key=lambda i: (-himp[l, i], i))
        size = [base] * Hkv
        for i in order[:rem]:
            size[i] += 1
        out.extend(alloc_threshold(himp[l].tolist(), size, t, r))
    return out

