"""Pins for the oracle's decode attention and score accumulation.

Everything the oracle is compared with here is independent of its own code:
closed forms worked by hand, a pure-Python triple loop, torch's CPU fp64
scaled-dot-product attention, and invariances that Eq. 1 implies.
"""
import math

import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import synth


def brute_attention(q, K, V):
    """Eq. 1 written as scalar loops with math.fsum (no numpy arithmetic)."""
    G, D = len(q), len(q[0])
    n = len(K)
    out = [[0.0] * D for _ in range(G)]
    probs = [[0.0] * n for _ in range(G)]
    for g in range(G):
        s = [math.fsum(q[g][d] * K[j][d] for d in range(D)) / math.sqrt(D) for j in range(n)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = math.fsum(e)
        for j in range(n):
            probs[g][j] = e[j] / z
        for d in range(D):
            out[g][d] = math.fsum(probs[g][j] * V[j][d] for j in range(n))
    return out, probs


@pytest.mark.parametrize("G,D,n,seed", [(1, 4, 1, 0), (2, 8, 5, 1), (4, 16, 33, 2), (7, 8, 64, 3)])
def test_matches_scalar_brute_force(G, D, n, seed):
    rng = np.random.default_rng(seed)
    q, K, V = rng.standard_normal((G, D)), rng.standard_normal((n, D)), rng.standard_normal((n, D))
    out, p = O.decode_attn(q, K, V)
    bo, bp = brute_attention(q.tolist(), K.tolist(), V.tolist())
    assert np.max(np.abs(out - np.array(bo))) < 1e-13
    assert np.max(np.abs(p - np.array(bp))) < 1e-14


def test_tiny_workload_brute_force():
    """The tiny workload's first head (fp32 inputs, D=64, 256 rows) against the scalar loops."""
    w = synth.WORKLOADS["tiny"]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    K = synth.payload(rng, (w.ctx, w.D), "f32").astype(np.float64)
    V = synth.payload(rng, (w.ctx, w.D), "f32").astype(np.float64)
    q = synth.payload(rng, (w.G, w.D), "f32").astype(np.float64)
    out, p = O.decode_attn(q, K, V)
    bo, bp = brute_attention(q.tolist(), K.tolist(), V.tolist())
    assert np.max(np.abs(out - np.array(bo))) < 1e-13
    assert np.max(np.abs(p - np.array(bp))) < 1e-15


def test_two_token_closed_form_pins_scale_and_operands():
    """q = k0 = ones(D), k1 = 0  =>  logits (sqrt(D), 0): p0 = 1/(1+exp(-sqrt(D))).

    A missing or wrong 1/sqrt(D) factor, a swapped K/V, or a transposed V all
    change the printed numbers below (worked by hand for D = 16: sqrt(D) = 4).
    """
    D = 16
    q = np.ones((1, D))
    K = np.vstack([np.ones(D), np.zeros(D)])
    V = np.vstack([np.arange(D, dtype=np.float64), -np.arange(D, dtype=np.float64) - 1.0])
    out, p = O.decode_attn(q, K, V)
    p0 = 1.0 / (1.0 + math.exp(-4.0))
    assert abs(p0 - 0.9820137900379085) < 1e-15
    assert abs(p[0, 0] - p0) < 1e-15 and abs(p[0, 1] - (1 - p0)) < 1e-15
    expect = p0 * V[0] + (1 - p0) * V[1]
    assert np.max(np.abs(out[0] - expect)) < 1e-14
    # out[0][3] = p0*3 - (1-p0)*4
    assert abs(out[0, 3] - (0.9820137900379085 * 3 - 0.0179862099620915 * 4)) < 1e-12


@pytest.mark.parametrize("G,D,n", [(4, 128, 300), (7, 128, 77), (2, 64, 256)])
def test_matches_torch_fp64_sdpa(G, D, n):
    rng = np.random.default_rng(11)
    q, K, V = rng.standard_normal((G, D)), rng.standard_normal((n, D)), rng.standard_normal((n, D))
    out, _ = O.decode_attn(q, K, V)
    tq = torch.from_numpy(q)[:, None, :]                 # [G, 1, D]: G heads, one query row
    tk = torch.from_numpy(K)[None].expand(G, n, D)
    tv = torch.from_numpy(V)[None].expand(G, n, D)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
    assert np.max(np.abs(out - ref)) < 1e-12


def test_weights_sum_to_one_and_are_positive():
    rng = np.random.default_rng(5)
    for n in (1, 2, 17, 1000):
        q, K, V = rng.standard_normal((4, 32)), 3 * rng.standard_normal((n, 32)), rng.standard_normal((n, 32))
        _, p = O.decode_attn(q, K, V)
        assert np.all(p >= 0)
        assert np.max(np.abs(p.sum(axis=1) - 1.0)) < 1e-12


def test_single_row_returns_that_value_row():
    rng = np.random.default_rng(6)
    q, K, V = rng.standard_normal((3, 8)), rng.standard_normal((1, 8)), rng.standard_normal((1, 8))
    out, p = O.decode_attn(q, K, V)
    assert np.array_equal(p, np.ones((3, 1)))
    assert np.array_equal(out, np.repeat(V, 3, axis=0))


def test_equal_keys_give_mean_of_values():
    rng = np.random.default_rng(7)
    k = rng.standard_normal(16)
    K = np.tile(k, (50, 1))
    V = rng.standard_normal((50, 16))
    out, p = O.decode_attn(rng.standard_normal((2, 16)), K, V)
    assert np.max(np.abs(p - 1 / 50)) < 1e-15
    assert np.max(np.abs(out - V.mean(axis=0))) < 1e-14


def test_key_shift_invariance():
    """Adding one vector to every key shifts every logit by the same amount: output unchanged."""
    rng = np.random.default_rng(8)
    q, K, V = rng.standard_normal((4, 32)), rng.standard_normal((40, 32)), rng.standard_normal((40, 32))
    out0, _ = O.decode_attn(q, K, V)
    out1, _ = O.decode_attn(q, K + rng.standard_normal(32), V)
    assert np.max(np.abs(out0 - out1)) < 1e-12


def test_row_permutation_invariance():
    """The output does not depend on the order of the cached rows, so compaction order cannot matter."""
    rng = np.random.default_rng(9)
    q, K, V = rng.standard_normal((4, 32)), rng.standard_normal((40, 32)), rng.standard_normal((40, 32))
    perm = rng.permutation(40)
    out0, p0 = O.decode_attn(q, K, V)
    out1, p1 = O.decode_attn(q, K[perm], V[perm])
    assert np.max(np.abs(out0 - out1)) < 1e-13
    assert np.max(np.abs(p0[:, perm] - p1)) < 1e-15


def test_identical_queries_in_group_identical_outputs():
    rng = np.random.default_rng(10)
    q1 = rng.standard_normal(16)
    q = np.tile(q1, (4, 1))
    out, _ = O.decode_attn(q, rng.standard_normal((9, 16)), rng.standard_normal((9, 16)))
    for g in range(1, 4):
        assert np.array_equal(out[0], out[g])


def test_large_logits_are_finite():
    rng = np.random.default_rng(12)
    q = 30 * rng.standard_normal((2, 64))
    K = 30 * rng.standard_normal((100, 64))
    out, p = O.decode_attn(q, K, rng.standard_normal((100, 64)))
    assert np.all(np.isfinite(out)) and abs(p.sum() - 2.0) < 1e-12


def test_empty_cache_is_an_error():
    with pytest.raises(ValueError):
        O.decode_attn(np.zeros((1, 4)), np.zeros((0, 4)), np.zeros((0, 4)))


def test_budget_at_least_context_reproduces_full_attention():
    """A head whose budget covers its whole context loses nothing: every step's output
    equals attention over the full history kept outside the cache object."""
    rng = np.random.default_rng(13)
    D, G, ctx = 16, 2, 40
    cache = O.Cache(D)
    Kh, Vh = [], []
    for t in range(ctx):
        k, v = rng.standard_normal(D), rng.standard_normal(D)
        q = rng.standard_normal((G, D))
        Kh.append(k), Vh.append(v)
        out, _, kept = O.decode_step(cache, q, k, v, t, t + 1, budget=ctx, sink=2, recent=4,
                                     interval=8, track_scores=True)
        full, _ = O.decode_attn(q, np.array(Kh), np.array(Vh))
        assert np.array_equal(out, full)
        if kept is not None:
            assert kept == list(range(t + 1))
    assert cache.n == ctx


def test_score_accumulation_closed_form():
    """Every query head's weights sum to 1, so without eviction the scores of a cache sum to
    G per decode step; a freshly appended row starts at 0 and receives its own weight."""
    rng = np.random.default_rng(14)
    D, G = 8, 3
    cache = O.Cache(D)
    for t in range(1, 21):
        O.decode_step(cache, rng.standard_normal((G, D)), rng.standard_normal(D), rng.standard_normal(D),
                      t, t, budget=100, sink=1, recent=1, interval=0, track_scores=True)
        assert abs(cache.score.sum() - G * t) < 1e-11
    assert cache.score[-1] > 0 and cache.score[-1] <= G
    # by hand: one row, one step -> its score is exactly G
    c2 = O.Cache(D)
    O.decode_step(c2, rng.standard_normal((G, D)), rng.standard_normal(D), rng.standard_normal(D),
                  0, 1, 10, 0, 0, 0, True)
    assert c2.score.tolist() == [float(G)]


def test_score_accumulate_sums_over_group():
    p = np.array([[0.25, 0.75], [0.5, 0.5]])
    s = O.score_accumulate(np.array([1.0, 2.0]), p)
    assert s.tolist() == [1.75, 3.25]


def test_eviction_happens_exactly_at_multiples_of_the_interval():
    """Step t evicts iff t is a multiple of the interval: a cache that starts at its budget b holds
    b + (t mod interval) rows after step t, and b again after every interval-th step."""
    rng = np.random.default_rng(5)
    D, b, interval = 8, 12, 4
    cache = O.Cache(D)
    cache.load(rng.standard_normal((b, D)), rng.standard_normal((b, D)), rng.random(b), np.arange(b))
    for t in range(1, 2 * interval + 2):
        _, _, kept = O.decode_step(cache, rng.standard_normal((2, D)), rng.standard_normal(D), rng.standard_normal(D),
                                   100 + t, t, budget=b, sink=2, recent=3, interval=interval, track_scores=True)
        if t % interval == 0:
            assert kept is not None and len(kept) == b and cache.n == b
        else:
            assert kept is None and cache.n == b + t % interval
