"""Pins of the oracle's profiling functions (Algorithm 1) against things other than itself:
brute force, closed forms, a library routine used differently, and invariances."""
import math

import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O


def brute_head_similarity(Q, K, V):
    """Pure-Python loops, written from the definition: no numpy arithmetic."""
    T, D = len(Q), len(Q[0])
    cos = []
    for t in range(T):
        logits = [sum(Q[t][d] * K[j][d] for d in range(D)) / math.sqrt(D) for j in range(t + 1)]
        m = max(logits)
        e = [math.exp(x - m) for x in logits]
        z = sum(e)
        out = [sum(e[j] / z * V[j][d] for j in range(t + 1)) for d in range(D)]
        dot = sum(V[t][d] * out[d] for d in range(D))
        nv = math.sqrt(sum(x * x for x in V[t]))
        no = math.sqrt(sum(x * x for x in out))
        cos.append(dot / max(nv * no, 1e-8))
    return sum(cos) / T, cos


@pytest.mark.parametrize("T,D,seed", [(1, 4, 0), (2, 8, 1), (7, 16, 2), (33, 8, 3), (20, 64, 4)])
def test_brute_force_on_small_inputs(T, D, seed):
    rng = np.random.default_rng(seed)
    Q, K, V = (rng.standard_normal((T, D)) for _ in range(3))
    mean, cos = O.head_similarity(Q, K, V)
    bmean, bcos = brute_head_similarity(Q.tolist(), K.tolist(), V.tolist())
    assert np.allclose(cos, bcos, rtol=0, atol=1e-12)
    assert abs(mean - bmean) <= 1e-12


def test_first_token_attends_to_itself_only():
    rng = np.random.default_rng(5)
    Q, K, V = (rng.standard_normal((9, 16)) for _ in range(3))
    _, cos = O.head_similarity(Q, K, V)
    assert abs(cos[0] - 1.0) <= 1e-15             # out_0 = v_0
    mean1, cos1 = O.head_similarity(Q[:1], K[:1], V[:1])
    assert mean1 == pytest.approx(1.0, abs=1e-15) and cos1.shape == (1,)


def test_two_token_closed_form():
    """out_1 = sigma v_0 + (1 - sigma) v_1 with sigma = logistic((q_1.k_0 - q_1.k_1)/sqrt(D))."""
    rng = np.random.default_rng(6)
    D = 8
    Q, K, V = (rng.standard_normal((2, D)) for _ in range(3))
    _, cos = O.head_similarity(Q, K, V)
    sig = 1.0 / (1.0 + math.exp(-(Q[1] @ K[0] - Q[1] @ K[1]) / math.sqrt(D)))
    out = sig * V[0] + (1 - sig) * V[1]
    want = (V[1] @ out) / (np.linalg.norm(V[1]) * np.linalg.norm(out))
    assert abs(cos[1] - want) <= 1e-14


def test_uniform_attention_gives_prefix_means():
    """Q = 0: every weight is 1/(t+1), so out_t is the mean of v_0..v_t."""
    rng = np.random.default_rng(7)
    T, D = 40, 12
    K, V = rng.standard_normal((T, D)), rng.standard_normal((T, D))
    mean, cos = O.head_similarity(np.zeros((T, D)), K, V)
    prefix = np.cumsum(V, axis=0) / np.arange(1, T + 1)[:, None]
    want = np.sum(V * prefix, axis=1) / (np.linalg.norm(V, axis=1) * np.linalg.norm(prefix, axis=1))
    assert np.allclose(cos, want, rtol=0, atol=1e-13)
    assert abs(mean - want.mean()) <= 1e-13


def test_identity_attention_gives_similarity_one():
    """Orthogonal keys and queries aligned with their own key, scaled up: the attention matrix tends to
    the identity, the case the paper names as the maximum (cosine 1 for every token)."""
    T = D = 16
    K = np.eye(T) * 200.0
    Q = np.eye(T) * 200.0
    V = np.random.default_rng(8).standard_normal((T, D))
    mean, cos = O.head_similarity(Q, K, V)
    assert np.all(cos > 1 - 1e-12) and mean == pytest.approx(1.0, abs=1e-12)


def test_causality_future_rows_do_not_matter():
    rng = np.random.default_rng(9)
    Q, K, V = (rng.standard_normal((25, 8)) for _ in range(3))
    _, cos = O.head_similarity(Q, K, V)
    _, cos_short = O.head_similarity(Q[:10], K[:10], V[:10])
    assert np.array_equal(cos[:10], cos_short)
    K2, V2 = K.copy(), V.copy()
    K2[20:], V2[20:] = 5.0, -3.0                  # changing later rows leaves earlier tokens alone
    _, cos2 = O.head_similarity(Q, K2, V2)
    assert np.array_equal(cos[:20], cos2[:20])


def test_scale_invariances():
    rng = np.random.default_rng(10)
    Q, K, V = (rng.standard_normal((30, 16)) for _ in range(3))
    _, cos = O.head_similarity(Q, K, V)
    _, cos_v = O.head_similarity(Q, K, 7.5 * V)                 # cosine ignores the length of V rows
    assert np.allclose(cos, cos_v, rtol=0, atol=1e-13)
    _, cos_neg = O.head_similarity(Q, K, -V)                    # ... and a common sign flip
    assert np.allclose(cos, cos_neg, rtol=0, atol=1e-13)
    _, cos_qk = O.head_similarity(2.0 * Q, 0.5 * K, V)          # logits depend on q.k only
    assert np.allclose(cos, cos_qk, rtol=0, atol=1e-12)
    # adding a constant vector c to every key adds q_t.c to every logit of row t: softmax unchanged
    _, cos_shift = O.head_similarity(Q, K + 3.0 * np.ones(16), V)
    assert np.allclose(cos, cos_shift, rtol=0, atol=1e-12)


@pytest.mark.parametrize("T,D,seed", [(64, 32, 11), (200, 128, 12)])
def test_against_library_causal_attention(T, D, seed):
    """torch's fp64 scaled_dot_product_attention with is_causal=True and its cosine_similarity: a
    library routine reaching the same definition by another route."""
    rng = np.random.default_rng(seed)
    Q, K, V = (rng.standard_normal((T, D)) for _ in range(3))
    mean, cos = O.head_similarity(Q, K, V)
    tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0, 0]
    want = torch.nn.functional.cosine_similarity(torch.from_numpy(V), out, dim=1).numpy()
    assert np.allclose(cos, want, rtol=0, atol=1e-12)
    assert abs(mean - want.mean()) <= 1e-12


def test_zero_rows_give_zero_cosine():
    rng = np.random.default_rng(13)
    Q, K, V = (rng.standard_normal((6, 8)) for _ in range(3))
    V[3] = 0.0
    _, cos = O.head_similarity(Q, K, V)
    assert cos[3] == 0.0 and np.all(np.isfinite(cos))
    _, cos0 = O.head_similarity(Q, K, np.zeros((6, 8)))
    assert np.array_equal(cos0, np.zeros(6))


def test_shape_errors():
    with pytest.raises(ValueError):
        O.head_similarity(np.zeros((3, 4)), np.zeros((2, 4)), np.zeros((3, 4)))
    with pytest.raises(ValueError):
        O.head_similarity(np.zeros((0, 4)), np.zeros((0, 4)), np.zeros((0, 4)))


def test_kv_importance_hand_values():
    # 1 layer, 4 heads, groups of 2: similarities (1, 0) and (-1, 0.5)
    s = np.array([[1.0, 0.0, -1.0, 0.5]])
    imp = O.kv_importance(s, 2)
    # group means 0.5 and -0.25 -> normalised 0.75 and 0.375 -> importance 0.25 and 0.625
    assert imp.shape == (1, 2) and imp.tolist() == [[0.25, 0.625]]
    assert O.kv_importance(np.array([[1.0, 1.0]]), 2).tolist() == [[0.0]]      # identical input and output
    assert O.kv_importance(np.array([[-1.0, -1.0]]), 1).tolist() == [[1.0, 1.0]]
    with pytest.raises(ValueError):
        O.kv_importance(np.zeros((1, 3)), 2)


def test_kv_importance_range_and_monotonicity():
    rng = np.random.default_rng(14)
    s = rng.uniform(-1, 1, (5, 28))
    imp = O.kv_importance(s, 7)
    assert imp.shape == (5, 4) and np.all(imp >= 0) and np.all(imp <= 1)
    s2 = s.copy()
    s2[2, 7:14] -= 0.1                             # a less similar group is more important
    imp2 = O.kv_importance(s2, 7)
    assert imp2[2, 1] > imp[2, 1] and np.array_equal(np.delete(imp2, 9), np.delete(imp, 9))
    # the affine map commutes with the group mean
    per_head = 1.0 - (s + 1.0) / 2.0
    assert np.allclose(imp, per_head.reshape(5, 4, 7).mean(axis=2), rtol=0, atol=1e-15)
