"""Pins of the oracle's layer-importance functions."""
import math

import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O


def test_closed_forms():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((9, 32))
    assert np.allclose(O.layer_similarity(X, X)[1], 1.0, atol=1e-15)
    assert np.allclose(O.layer_similarity(X, -3.0 * X)[1], -1.0, atol=1e-15)
    E = np.eye(8)
    mean, cos = O.layer_similarity(E[:4], E[4:])
    assert mean == 0.0 and np.array_equal(cos, np.zeros(4))
    # a known angle: 45 degrees between (1, 0) and (1, 1)
    mean, cos = O.layer_similarity(np.array([[1.0, 0.0]]), np.array([[1.0, 1.0]]))
    assert abs(cos[0] - 1 / math.sqrt(2)) <= 1e-15 and abs(mean - 1 / math.sqrt(2)) <= 1e-15
    # residual connection with a small update: cos = (1 + eps a.b/|a|^2) / |a + eps b| * |a| ...
    a, b = rng.standard_normal(16), rng.standard_normal(16)
    want = (a @ (a + 0.1 * b)) / (np.linalg.norm(a) * np.linalg.norm(a + 0.1 * b))
    assert abs(O.layer_similarity(a[None], (a + 0.1 * b)[None])[1][0] - want) <= 1e-15


def test_brute_force_and_library():
    rng = np.random.default_rng(1)
    A, Bm = rng.standard_normal((20, 48)), rng.standard_normal((20, 48))
    mean, cos = O.layer_similarity(A, Bm)
    for t in range(20):
        dot = sum(A[t, i] * Bm[t, i] for i in range(48))
        na = math.sqrt(sum(x * x for x in A[t]))
        nb = math.sqrt(sum(x * x for x in Bm[t]))
        assert abs(cos[t] - dot / (na * nb)) <= 1e-13
    want = torch.nn.functional.cosine_similarity(torch.from_numpy(A), torch.from_numpy(Bm), dim=1).numpy()
    assert np.allclose(cos, want, rtol=0, atol=1e-13) and abs(mean - want.mean()) <= 1e-13


def test_invariances_zero_rows_and_errors():
    rng = np.random.default_rng(2)
    A, Bm = rng.standard_normal((7, 16)), rng.standard_normal((7, 16))
    _, cos = O.layer_similarity(A, Bm)
    assert np.allclose(O.layer_similarity(5 * A, 0.2 * Bm)[1], cos, atol=1e-14)
    assert np.allclose(O.layer_similarity(Bm, A)[1], cos, atol=1e-15)          # symmetric
    A[3] = 0.0
    assert O.layer_similarity(A, Bm)[1][3] == 0.0
    with pytest.raises(ValueError):
        O.layer_similarity(A, Bm[:5])


def test_two_level_allocation_invariants():
    rng = np.random.default_rng(3)
    for L, Hkv in ((4, 8), (32, 8), (28, 4), (1, 2)):
        limp = rng.uniform(0.05, 1.0, L)
        himp = rng.uniform(0.0, 1.0, (L, Hkv))
        lo, hi = 128, 32768
        Bt = int(L * Hkv * 8192 * 0.3)
        b = O.alloc_two_level(limp, himp, Bt, lo, hi, 0.4, 0.25)
        assert len(b) == L * Hkv and sum(b) == Bt and min(b) >= 0
        pools = O.alloc_proportional(limp, Bt, Hkv * lo, Hkv * hi)
        for l in range(L):
            assert sum(b[l * Hkv:(l + 1) * Hkv]) == pools[l]                   # Algorithm 2 conserves the pool
        # more important layers get larger pools
        order = np.argsort(limp)
        assert all(pools[order[i]] <= pools[order[i + 1]] for i in range(L - 1))
    # no cache below the threshold: every layer is an equal split of its pool
    himp = np.full((3, 4), 0.9)
    b = O.alloc_two_level([1.0, 2.0, 3.0], himp, 3 * 4 * 1000, 100, 5000, 0.5, 0.5)
    for l in range(3):
        chunk = b[l * 4:(l + 1) * 4]
        assert max(chunk) - min(chunk) <= 1
    # equal layer importances and r = 0: the plain equal split
    b = O.alloc_two_level([1.0, 1.0], np.array([[0.1, 0.9], [0.9, 0.1]]), 4000, 10, 5000, 0.5, 0.0)
    assert b == [1000, 1000, 1000, 1000]
    # hand example: pools 1000 / 3000 (importances 1 : 3); layer 1 has one cache below t = 0.5, r = 0.5:
    # equal split 1500 / 1500, the low cache gives floor(0.5 * 1500) = 750 to the other
    b = O.alloc_two_level([1.0, 3.0], np.array([[0.8, 0.9], [0.2, 0.7]]), 4000, 10, 5000, 0.5, 0.5)
    assert b == [500, 500, 750, 2250]


def test_two_level_hand_worked_floor_pool_and_remainder():
    """Layer importances [1, 1000], 3 caches per layer, lo = 10, global budget 332: layer 0's share
    (0.33 rows) is lifted to the floor of 3 * lo = 30 rows, layer 1 takes the other 302.  Inside a
    layer the pool is split equally, the remainder going to the most important caches first:
    302 = 3 * 100 + 2 with importances [0.3, 0.9, 0.5] gives [100, 101, 101].  No importance lies
    below t = 0, so Algorithm 2 changes nothing."""
    got = O.alloc_two_level([1.0, 1000.0], np.array([[0.4, 0.4, 0.4], [0.3, 0.9, 0.5]]), 332, 10, 1000, 0.0, 0.5)
    assert got == [10, 10, 10, 100, 101, 101]
