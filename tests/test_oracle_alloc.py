"""Pins for the oracle's budget allocators."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import baklava_oracle as O
from paper_2502_13176_amd import synth


def exact_waterfill(imp, B, lo, hi):
    """Real-valued solution of b_i = clip(mu*I_i, lo, hi), sum b_i = B, in exact rationals."""
    I = [Fraction(v) for v in imp]
    m = len(I)
    # breakpoints of the piecewise-linear f(mu)
    pts = sorted({Fraction(lo) / v for v in I} | {Fraction(hi) / v for v in I})

    def f(mu):
        return sum(min(max(mu * v, lo), hi) for v in I)

    if f(pts[-1]) == B:
        mu = pts[-1]
    else:
        mu = None
        for a, z in zip(pts, pts[1:]):
            fa, fz = f(a), f(z)
            if fa <= B <= fz:
                mu = a if fz == fa else a + (z - a) * (B - fa) / (fz - fa)
                break
        assert mu is not None
    return [min(max(mu * v, lo), hi) for v in I]


@pytest.mark.parametrize("seed", range(12))
def test_close_to_exact_rational_waterfilling(seed):
    """The integer rule floors lam*w_i with the largest feasible integer lam (a divisor
    method), so a head's budget may exceed its exact real-valued share by up to one token
    per head times its share of the unclipped weight, plus one for the leftover pass."""
    rng = np.random.default_rng(seed)
    m = int(rng.integers(2, 9))
    imp = rng.lognormal(0, 1.2, m)
    lo, hi = 3, int(rng.integers(20, 200))
    B = int(rng.integers(m * lo, m * hi + 1))
    b = O.alloc_proportional(imp, B, lo, hi)
    ideal = exact_waterfill(imp, B, lo, hi)
    assert sum(b) == B
    free = [i for i in range(m) if lo < ideal[i] < hi]
    wsum = sum(Fraction(imp[i]) for i in free)
    for i, (bi, xi) in enumerate(zip(b, ideal)):
        slack = 1 + (m * Fraction(imp[i]) / wsum if free else 0) + Fraction(1, 1000)
        assert abs(Fraction(bi) - xi) <= slack


def linear_scan_alloc(imp, B, lo, hi):
    """Same rule as the oracle but the multiplier is found by counting up from zero in
    exact rationals, and the leftover pass uses exact fractional parts."""
    m = len(imp)
    top = max(imp)
    w = [max(Fraction(1, 2 ** 40), Fraction(int((v / top) * 2.0 ** 40), 2 ** 40)) for v in imp]

    def alloc(lam):
        return [min(max((lam * wi).__floor__(), lo), hi) for wi in w]

    lam = 0
    while sum(alloc(lam + 1)) <= B and lam < 10 ** 6:
        lam += 1
    b = alloc(lam)
    x = [(lam * wi).__floor__() for wi in w]
    elig = [i for i in range(m) if lo <= x[i] < hi]
    elig.sort(key=lambda i: (lam * w[i] - x[i], w[i], -i), reverse=True)
    for i in elig[:B - sum(b)]:
        b[i] += 1
    return b


@pytest.mark.parametrize("seed", range(10))
def test_matches_linear_scan_in_exact_rationals(seed):
    rng = np.random.default_rng(50 + seed)
    m = int(rng.integers(2, 7))
    # importances on a coarse grid keep the multiplier small enough to count up to
    imp = [float(x) for x in rng.integers(1, 9, m)]
    lo, hi = int(rng.integers(0, 3)), int(rng.integers(8, 40))
    B = int(rng.integers(m * lo, m * hi))
    assert O.alloc_proportional(imp, B, lo, hi) == linear_scan_alloc(imp, B, lo, hi)


@pytest.mark.parametrize("name", ["llama1", "llama32", "qwen", "long"])
def test_invariants_on_the_benchmark_workloads(name):
    w = synth.WORKLOADS[name]
    imp = synth.importance_scores(w)
    b = synth.budgets_for(w, O.alloc_proportional)
    assert len(b) == w.m
    assert sum(b) == w.global_budget
    assert min(b) >= w.lo and max(b) <= w.hi
    order = np.argsort(imp, kind="stable")
    sb = [b[i] for i in order]
    assert all(sb[i] <= sb[i + 1] for i in range(len(sb) - 1))      # monotone in importance
    if w.floor_frac:
        assert sum(1 for x in b if x == w.lo) >= round(w.floor_frac * w.m)


@pytest.mark.parametrize("name", ["llama1", "llama32", "qwen", "long"])
def test_benchmark_budgets_stay_close_to_exact_waterfilling(name):
    """The budgets the benchmark workloads run on (and tests/golden stores), against the real-valued
    shares clip(mu * I_i, lo, hi) that sum to the global budget, in exact rationals: clipped heads sit
    exactly at their bound, every other head within the divisor rule's deviation of its share."""
    w = synth.WORKLOADS[name]
    imp = synth.importance_scores(w)
    b = synth.budgets_for(w, O.alloc_proportional)
    n_floor = int(round(w.floor_frac * w.m))
    order = sorted(range(w.m), key=lambda i: (imp[i], i))
    rest = sorted(order[n_floor:])                         # the heads that share what the pinned ones leave
    assert all(b[i] == w.lo for i in order[:n_floor])
    B = w.global_budget - n_floor * w.lo
    sub = [b[i] for i in rest]
    ideal = exact_waterfill([imp[i] for i in rest], B, w.lo, w.hi)
    assert sum(sub) == B and sum(ideal) == B
    free = [k for k in range(len(rest)) if w.lo < ideal[k] < w.hi]
    wsum = sum(Fraction(imp[rest[k]]) for k in free)
    for k, (bi, xi) in enumerate(zip(sub, ideal)):
        if xi == w.hi:
            assert bi in (w.hi, w.hi - 1)                  # the largest multiplier may stop one floor short of the bound
        elif xi == w.lo:
            assert bi == w.lo
        else:
            slack = 1 + len(rest) * Fraction(imp[rest[k]]) / wsum
            assert abs(Fraction(bi) - xi) <= slack, (k, bi, float(xi))


def test_expected_global_budgets():
    assert synth.WORKLOADS["llama1"].global_budget == 32768
    assert synth.WORKLOADS["llama32"].global_budget == 2516582
    assert synth.WORKLOADS["qwen"].global_budget == 1835008
    assert synth.WORKLOADS["long"].global_budget == 5033164


def test_equal_importance_differs_by_at_most_one_and_older_first():
    b = O.alloc_proportional([2.5] * 7, 100, 0, 100)
    assert sum(b) == 100 and max(b) - min(b) <= 1
    assert b == sorted(b, reverse=True)                 # leftover goes to lower indices first


def test_power_of_two_scaling_leaves_budgets_unchanged():
    rng = np.random.default_rng(1)
    imp = rng.lognormal(0, 1, 16)
    a = O.alloc_proportional(imp, 5000, 10, 2000)
    for k in (-7, 3, 20):
        assert O.alloc_proportional(imp * 2.0 ** k, 5000, 10, 2000) == a


def test_extreme_budgets():
    imp = [0.1, 5.0, 1.0]
    assert O.alloc_proportional(imp, 30, 10, 50) == [10, 10, 10]
    assert O.alloc_proportional(imp, 150, 10, 50) == [50, 50, 50]


def test_hand_worked_proportional_example():
    # importance 1:2:5, B=80, wide clips -> exactly proportional 10, 20, 50
    assert O.alloc_proportional([1.0, 2.0, 5.0], 80, 0, 1000) == [10, 20, 50]
    # same with hi=40: head 2 saturates at 40, the other two share 40 as 1:2 -> 13.33, 26.67
    b = O.alloc_proportional([1.0, 2.0, 5.0], 80, 0, 40)
    assert b[2] == 40 and sum(b) == 80 and b[:2] in ([13, 27], [14, 26])
    assert b[:2] == [13, 27]                             # larger fractional part (0.67) wins the leftover


def test_infeasible_and_bad_inputs():
    with pytest.raises(ValueError):
        O.alloc_proportional([1.0, 1.0], 5, 3, 10)       # m*lo > B
    with pytest.raises(ValueError):
        O.alloc_proportional([1.0, 1.0], 25, 3, 10)      # m*hi < B
    with pytest.raises(ValueError):
        O.alloc_proportional([1.0, 0.0], 10, 3, 10)
    with pytest.raises(ValueError):
        O.alloc_proportional([1.0, float("nan")], 10, 3, 10)


# ---- Algorithm 2 (threshold reallocation).  No worked example is printed in the paper:
# ---- beyond the invariants below this function's parity is unpinned.

def test_threshold_conserves_total_memory():
    rng = np.random.default_rng(2)
    for _ in range(50):
        m = int(rng.integers(2, 40))
        imp = rng.random(m)
        size = [int(x) for x in rng.integers(10, 5000, m)]
        out = O.alloc_threshold(imp, size, float(rng.random()), float(rng.random()))
        assert sum(out) == sum(size)


def test_threshold_all_low_or_none_low_is_unchanged():
    size = [100, 200, 300]
    assert O.alloc_threshold([0.1, 0.2, 0.3], size, 0.5, 0.5) == size
    assert O.alloc_threshold([0.6, 0.7, 0.8], size, 0.5, 0.5) == size


def test_threshold_three_level_structure_from_uniform_start():
    imp = [0.9, 0.1, 0.5, 0.2, 0.8, 0.6, 0.7]
    out = O.alloc_threshold(imp, [1000] * 7, 0.3, 0.25)
    # low = {1, 3} lose 250 each; k = min(2, 5) = 2 -> the two most important (0, 4) gain 250 each
    assert out == [1250, 750, 1000, 750, 1250, 1000, 1000]


def test_threshold_k_is_capped_by_number_of_high_caches():
    imp = [0.1, 0.2, 0.15, 0.9]
    out = O.alloc_threshold(imp, [100] * 4, 0.5, 0.1)
    # n = 3 low caches free 30; k = min(3, 1) = 1 -> all of it to cache 3
    assert out == [90, 90, 90, 130]


def test_threshold_remainder_goes_to_most_important_first():
    imp = [0.9, 0.8, 0.1, 0.2, 0.05, 0.7]
    out = O.alloc_threshold(imp, [10, 10, 11, 11, 11, 10], 0.5, 0.5)
    # floor(5.5) = 5 freed thrice = 15; k = 3 -> 5 each
    assert out == [15, 15, 6, 6, 6, 15]
    out = O.alloc_threshold(imp, [10, 10, 11, 11, 9, 10], 0.5, 0.5)
    # freed 5 + 5 + 4 = 14; k = 3 -> 4 each, remainder 2 to importance 0.9 then 0.8
    assert out == [15, 15, 6, 6, 5, 14]


def test_layout_prefix_sums():
    off, cap, total = O.layout([5, 9], L=1, Hkv=2, batch=2, slack=3)
    assert cap == [8, 12, 8, 12]
    assert off == [0, 8, 20, 28]
    assert total == 40
    off, cap, total = O.layout([5, 9, 1, 2], L=2, Hkv=2, batch=1, slack=0)
    assert cap == [5, 9, 1, 2] and off == [0, 5, 14, 15] and total == 17


def test_leftover_tokens_never_lift_a_head_above_hi():
    """Shares 24 * [7, 4, 8, 5] / 24 = [7, 4, 8, 5]; hi = 7 clips head 2 and one token is left over.
    Head 0 sits at hi exactly and may not take it; of heads 1 and 3 the heavier one is next in line."""
    assert O.alloc_proportional([7, 4, 8, 5], 24, 1, 7) == [7, 4, 7, 6]


def test_invariants_on_many_small_cases():
    """Exact sum, bounds and monotonicity where clipping and leftovers dominate (few heads, tight bounds)."""
    rng = np.random.Generator(np.random.PCG64(7))
    for _ in range(3000):
        m = int(rng.integers(2, 6))
        imp = [float(v) for v in rng.integers(1, 9, size=m)]
        lo = int(rng.integers(0, 4))
        hi = int(rng.integers(lo + 1, 13))
        B = int(rng.integers(m * lo, m * hi + 1))
        b = O.alloc_proportional(imp, B, lo, hi)
        assert sum(b) == B and min(b) >= lo and max(b) <= hi, (imp, B, lo, hi, b)
        for i in range(m):
            for j in range(m):
                if imp[i] < imp[j]:
                    assert b[i] <= b[j], (imp, B, lo, hi, b)
                if imp[i] == imp[j]:
                    assert abs(b[i] - b[j]) <= 1, (imp, B, lo, hi, b)


def test_threshold_comparison_is_strict():
    """Algorithm 2 selects I_i < t: caches whose importance equals the threshold keep their size.
    I = [0.2, 0.5, 0.5, 0.9], t = 0.5, r = 1/2, 100 rows each: only cache 0 shrinks (by 50), n = 1,
    k = min(1, 3) = 1, and the most important cache receives the 50 rows."""
    assert O.alloc_threshold([0.2, 0.5, 0.5, 0.9], [100] * 4, 0.5, 0.5) == [50, 100, 100, 150]


def test_threshold_ties_among_receivers_go_to_the_lower_index():
    """Two equally important caches compete for one receiving place (k = min(1, 2) = 1): the paper
    does not say who wins; the reading taken is the lower index."""
    assert O.alloc_threshold([0.1, 0.9, 0.9], [100, 100, 100], 0.5, 0.5) == [50, 150, 100]
