"""Pins for the oracle's eviction: brute force on small inputs and the structural
invariants that f_evict (Eqs. 5-6) and the sink/recent/top-score policy imply."""
import itertools

import numpy as np
import pytest

from oracle import baklava_oracle as O


def brute_select(score32, n, b, sink, recent):
    """Enumerate every subset of the middle of size k and keep the best one under the
    (score desc, index asc) order -- exponential, tiny inputs only."""
    if n <= b:
        return list(range(n))
    k = b - sink - recent
    mid = list(range(sink, n - recent))
    best, best_key = None, None
    for comb in itertools.combinations(mid, k):
        # rank vector: sorted by preference; compare lexicographically
        key = sorted(((-float(score32[j]), j) for j in comb))
        if best is None or key < best_key:
            best, best_key = comb, key
    return sorted(list(range(sink)) + list(best) + list(range(n - recent, n)))


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_subset_enumeration(seed):
    rng = np.random.default_rng(seed)
    n, sink, recent = 12, 2, 3
    for b in (5, 6, 8, 11, 12, 20):
        # coarse scores force ties
        score = rng.integers(0, 4, n).astype(np.float32) / 4
        assert O.compact_select(score, n, b, sink, recent) == brute_select(score, n, b, sink, recent)


def test_hand_worked_example():
    # n=10, sink=1, recent=2, budget=6 -> k=3 of middle {1..7}
    score = np.array([0.0, 0.5, 0.9, 0.5, 0.1, 0.9, 0.5, 0.2, 9.0, 9.0], dtype=np.float32)
    # top-3 of the middle: 0.9@2, 0.9@5, then 0.5 tie among {1,3,6} -> oldest (1)
    assert O.compact_select(score, 10, 6, 1, 2) == [0, 1, 2, 5, 8, 9]


def test_ties_prefer_older_rows():
    score = np.zeros(20, dtype=np.float32)
    assert O.compact_select(score, 20, 10, 2, 3) == [0, 1, 2, 3, 4, 5, 6, 17, 18, 19]


def test_fp32_comparison_precision():
    """Scores that differ only beyond fp32 precision are ties, broken by index."""
    score = np.array([0, 1.0, 1.0 + 1e-12, 0], dtype=np.float64)
    assert O.compact_select(score, 4, 3, 1, 1) == [0, 1, 3]


@pytest.mark.parametrize("seed", range(5))
def test_structural_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(50, 400))
    sink, recent = int(rng.integers(0, 6)), int(rng.integers(0, 20))
    b = int(rng.integers(sink + recent, n))
    score = rng.random(n).astype(np.float32)
    kept = O.compact_select(score, n, b, sink, recent)
    assert len(kept) == min(n, b)
    assert all(kept[i] < kept[i + 1] for i in range(len(kept) - 1))
    assert set(range(sink)) <= set(kept)
    assert set(range(n - recent, n)) <= set(kept)
    ks = set(kept)
    mid = range(sink, n - recent)
    kept_mid = [j for j in mid if j in ks]
    gone_mid = [j for j in mid if j not in ks]
    if kept_mid and gone_mid:
        worst_kept = max((-float(score[j]), j) for j in kept_mid)
        best_gone = min((-float(score[j]), j) for j in gone_mid)
        assert worst_kept < best_gone


def test_identity_when_within_budget_and_idempotent():
    rng = np.random.default_rng(3)
    D = 4
    c = O.Cache(D)
    for t in range(30):
        c.append(rng.standard_normal(D), rng.standard_normal(D), t)
    c.score = rng.random(30)
    assert c.compact(30, 2, 4) == list(range(30))
    assert c.compact(64, 2, 4) == list(range(30))
    first = c.compact(12, 2, 4)
    assert c.n == 12
    assert c.compact(12, 2, 4) == list(range(12))       # second compaction is the identity
    assert len(first) == 12


def test_rows_move_with_their_indices_and_keep_order():
    rng = np.random.default_rng(4)
    D = 8
    c = O.Cache(D)
    for t in range(40):
        c.append(rng.standard_normal(D), rng.standard_normal(D), 1000 + t)
    c.score = rng.random(40)
    K0, V0, s0, p0 = c.K.copy(), c.V.copy(), c.score.copy(), c.pos.copy()
    kept = c.compact(17, 3, 5)
    assert np.array_equal(c.K, K0[kept]) and np.array_equal(c.V, V0[kept])
    assert np.array_equal(c.score, s0[kept]) and np.array_equal(c.pos, p0[kept])
    assert np.all(np.diff(c.pos) > 0)                    # survivors keep arrival order (Eqs. 5-6)


def test_streaming_policy_and_its_score_policy_special_case():
    score = np.random.default_rng(5).random(50).astype(np.float32)
    st = O.compact_select(score, 50, 20, 4, 0, O.POLICY_STREAMING)
    assert st == [0, 1, 2, 3] + list(range(34, 50))
    # budget = sink + recent under the score policy is the same set
    assert O.compact_select(score, 50, 20, 4, 16, O.POLICY_SCORE) == st


def test_budget_below_sink_plus_recent_is_an_error():
    with pytest.raises(ValueError):
        O.compact_select(np.zeros(30, dtype=np.float32), 30, 10, 4, 16)


def test_eviction_removes_exactly_the_unselected_tokens():
    """Removing tokens one at a time as Eqs. 5-6 write it gives the same cache."""
    rng = np.random.default_rng(6)
    n, D = 25, 4
    K = rng.standard_normal((n, D))
    score = rng.random(n)
    kept = O.compact_select(score, n, 10, 2, 3)
    rows = [K[j] for j in range(n)]
    for m in sorted(set(range(n)) - set(kept), reverse=True):
        rows = rows[:m] + rows[m + 1:]                   # [k_1..k_{m-1}, k_{m+1}..]
    assert np.array_equal(np.array(rows), K[kept])
