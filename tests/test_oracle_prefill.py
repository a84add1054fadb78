"""Pins of the oracle's prefill_scores (column sums of the causal attention matrices)."""
import math

import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O


def brute(Q, K):
    G, T, D = len(Q), len(Q[0]), len(Q[0][0])
    score = [0.0] * T
    for g in range(G):
        for t in range(T):
            logits = [sum(Q[g][t][d] * K[j][d] for d in range(D)) / math.sqrt(D) for j in range(t + 1)]
            m = max(logits)
            e = [math.exp(x - m) for x in logits]
            z = sum(e)
            for j in range(t + 1):
                score[j] += e[j] / z
    return score


@pytest.mark.parametrize("G,T,D,seed", [(1, 1, 4, 0), (2, 5, 8, 1), (4, 17, 16, 2), (7, 9, 8, 3)])
def test_brute_force(G, T, D, seed):
    rng = np.random.default_rng(seed)
    Q, K = rng.standard_normal((G, T, D)), rng.standard_normal((T, D))
    assert np.allclose(O.prefill_scores(Q, K), brute(Q.tolist(), K.tolist()), rtol=0, atol=1e-12)


def test_total_mass_and_last_column():
    """Every row of every head's attention matrix sums to 1, so the scores sum to G*T; the last
    token is seen only by itself: its score is sum_g p_g[T-1, T-1] <= G; a single token scores G."""
    rng = np.random.default_rng(4)
    G, T, D = 3, 50, 16
    Q, K = rng.standard_normal((G, T, D)), rng.standard_normal((T, D))
    s = O.prefill_scores(Q, K)
    assert abs(s.sum() - G * T) <= 1e-10
    assert 0 < s[-1] <= G and s[0] >= G * 1.0                    # token 0 gets all of row 0 of each head
    assert O.prefill_scores(Q[:, :1], K[:1]).tolist() == [float(G)]


def test_uniform_attention_gives_harmonic_tails():
    """Q = 0: p[t, j] = 1/(t+1), so score_j = G * (H_T - H_j) with H_n the n-th harmonic number."""
    G, T, D = 2, 64, 8
    K = np.random.default_rng(5).standard_normal((T, D))
    s = O.prefill_scores(np.zeros((G, T, D)), K)
    Hn = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, T + 1))])
    want = G * (Hn[T] - Hn[:T])
    assert np.allclose(s, want, rtol=0, atol=1e-12)


def test_against_library_softmax_of_masked_logits():
    rng = np.random.default_rng(6)
    G, T, D = 4, 96, 32
    Q, K = rng.standard_normal((G, T, D)), rng.standard_normal((T, D))
    logits = torch.from_numpy(Q) @ torch.from_numpy(K).T / math.sqrt(D)            # [G, T, T]
    mask = torch.triu(torch.ones(T, T, dtype=torch.bool), diagonal=1)
    p = torch.softmax(logits.masked_fill(mask, float("-inf")), dim=-1)
    want = p.sum(dim=(0, 1)).numpy()
    assert np.allclose(O.prefill_scores(Q, K), want, rtol=0, atol=1e-11)


def test_equals_token_by_token_decode_accumulation():
    """Decoding the prompt one token at a time and accumulating decode_attn's weights with
    score_accumulate builds the same scores (new rows start at 0)."""
    rng = np.random.default_rng(7)
    G, T, D = 2, 30, 16
    Q, K, V = rng.standard_normal((G, T, D)), rng.standard_normal((T, D)), rng.standard_normal((T, D))
    score = np.zeros(0)
    for t in range(T):
        score = np.concatenate([score, [0.0]])
        _, p = O.decode_attn(Q[:, t], K[: t + 1], V[: t + 1])
        score = O.score_accumulate(score, p)
    assert np.allclose(O.prefill_scores(Q, K), score, rtol=0, atol=1e-12)


def test_causality_and_errors():
    rng = np.random.default_rng(8)
    Q, K = rng.standard_normal((2, 20, 8)), rng.standard_normal((20, 8))
    s = O.prefill_scores(Q, K)
    s_short = O.prefill_scores(Q[:, :12], K[:12])
    assert np.all(s[:12] >= s_short - 1e-15)                       # later tokens only add attention
    with pytest.raises(ValueError):
        O.prefill_scores(Q, K[:5])
