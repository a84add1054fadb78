"""GPU parity: baklava_prefill_scores (column sums of the causal attention matrices) against the
oracle, and the prefill -> scores -> eviction path end to end on a ragged arena."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu

# A score is a sum of up to G*T softmax weights, each 2^(fp32 logit - fp32 log-sum-exp): relative
# error per weight ~ (|logit| + |lse|) * 2^-24 * ln 2 plus the hardware exp2/log2 approximations
# (~1e-6), accumulated in fp32.  Bound taken: 2e-5 relative to max(1, score) (measured ~2e-6).
SCORE_RTOL = 2e-5
LSE_TOL = 1e-4  # log2 units, against the oracle's fp64 log-sum-exp


def _h():
    import gpu_harness
    return gpu_harness


def oracle_lse2(q64, k64):
    """fp64 log2-sum-exp of the scaled causal logits, written out from its definition."""
    T, D = q64.shape
    out = np.empty(T)
    for t in range(T):
        s = (k64[: t + 1] @ q64[t]) / np.sqrt(D) * np.log2(np.e)
        m = s.max()
        out[t] = m + np.log2(np.sum(np.exp2(s - m)))
    return out


def run_dense(batch, Hq, Hkv, T, seed, peaked=False, qscale=1.0):
    H = _h()
    dev = torch.device("cuda:0")
    rng = np.random.Generator(np.random.PCG64(seed))
    qb = synth.f32_to_bf16_bits(qscale * rng.standard_normal((batch, Hq, T, 128), dtype=np.float32))
    kb = synth.payload(rng, (batch, Hkv, T, 128), "bf16", peaked=peaked)
    vb = synth.payload(rng, (batch, Hkv, T, 128), "bf16")
    q, k, v = (H.to_device_storage(x, "bf16", dev) for x in (qb, kb, vb))
    _, _, lse = B.profile_similarity(q, k, v, want_cos=False, want_lse=True)
    score = torch.full((batch * Hkv * T,), float("nan"), dtype=torch.float32, device=dev)
    B.prefill_scores(q, k, lse, score, batch, Hq, Hkv, T)
    torch.cuda.synchronize()
    got = score.cpu().numpy().astype(np.float64).reshape(batch, Hkv, T)
    lse_h = lse.cpu().numpy().astype(np.float64)
    q64, k64 = synth.storage_to_f64(qb, "bf16"), synth.storage_to_f64(kb, "bf16")
    G = Hq // Hkv
    worst = 0.0
    for b in range(batch):
        for h in range(Hkv):
            want = O.prefill_scores(q64[b, h * G:(h + 1) * G], k64[b, h])
            err = np.abs(got[b, h] - want) / np.maximum(1.0, want)
            assert np.all(np.isfinite(got[b, h]))
            assert err.max() <= SCORE_RTOL, f"batch {b} kv head {h}: relative score error {err.max():.3e}"
            assert abs(got[b, h].sum() - G * T) <= 1e-4 * G * T          # every attention row sums to 1
            worst = max(worst, float(err.max()))
        for hq in range(0, Hq, max(1, Hq // 3)):
            want_lse = oracle_lse2(q64[b, hq], k64[b, hq // G])
            assert np.max(np.abs(lse_h[b, hq] - want_lse)) <= LSE_TOL
    return worst


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 127, 128, 129, 200, 257, 400])
def test_prompt_lengths_around_every_tile_boundary(T):
    worst = run_dense(1, 4, 2, T, 9600 + T)
    print(f"T={T}: worst relative score error {worst:.2e}", flush=True)


@pytest.mark.parametrize("batch,Hq,Hkv", [(2, 8, 2), (1, 7, 1), (3, 2, 2), (1, 16, 1)])
def test_head_grouping_and_batches(batch, Hq, Hkv):
    run_dense(batch, Hq, Hkv, 300, 9700 + Hq)


def test_peaked_and_large_logits():
    run_dense(1, 4, 2, 350, 9800, peaked=True, qscale=4.0)


def test_prefill_then_eviction_on_a_ragged_arena():
    """A prompt of T tokens is written into every cache of a layer (capacity >= T), the scores come
    from the kernel, and one eviction brings every cache down to its own budget: kept lists bit-exact
    against the oracle's selection on the kernel's scores, scores within tolerance of the oracle's."""
    H = _h()
    T = 1500
    w = synth.shrink(synth.WORKLOADS["llama32"], name="prefill", L=2, Hq=8, Hkv=4, batch=2, seed=31, sink=4,
                     recent=32, slack=T)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [100, 450, 37, 1499, 800, 64, 300, 1200]             # per (layer, KV head)
    arena = H.make_arena(w, budgets)
    lens = [T] * arena.n_caches
    st = H.fill_from_host(arena, w, lens, rng, scores="zero")
    dev = arena.device
    cpl = w.batch * w.Hkv
    G = w.G
    for layer in range(w.L):
        qb = synth.payload(rng, (w.batch, w.Hq, T, w.D), "bf16")
        q = H.to_device_storage(qb, "bf16", dev)
        q64 = synth.storage_to_f64(qb, "bf16")
        # dense copies of the layer's K / V rows for the attention pass that yields the normalisers
        kd = torch.stack([arena.k[int(arena.off_host[layer * cpl + s]):int(arena.off_host[layer * cpl + s]) + T]
                          for s in range(cpl)]).view(w.batch, w.Hkv, T, w.D).contiguous()
        vd = torch.stack([arena.v[int(arena.off_host[layer * cpl + s]):int(arena.off_host[layer * cpl + s]) + T]
                          for s in range(cpl)]).view(w.batch, w.Hkv, T, w.D).contiguous()
        _, _, lse = B.profile_similarity(q, kd, vd, want_cos=False, want_lse=True)
        # scores straight into the arena's score plane, K read from the arena through its offset table
        B.prefill_scores(q, arena.k, lse, arena.score, w.batch, w.Hq, w.Hkv, T, row_off=arena.off[layer * cpl:(layer + 1) * cpl])
        torch.cuda.synchronize()
        for s in range(cpl):
            c = layer * cpl + s
            b, h = divmod(s, w.Hkv)
            o = int(arena.off_host[c])
            got = arena.score[o:o + T].cpu().numpy()
            want = O.prefill_scores(q64[b, h * G:(h + 1) * G], synth.storage_to_f64(st.K[c], "bf16"))
            assert np.max(np.abs(got - want) / np.maximum(1.0, want)) <= SCORE_RTOL
            st.score[c] = got                                       # selection is judged on the kernel's own fp32 scores
    from test_gpu_compact import run_compact_and_check
    after = run_compact_and_check(arena, w, st)
    assert arena.lengths().tolist() == [budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)]
    # the sink rows and the recent window survive in every cache
    for c in range(arena.n_caches):
        pos = after.pos[c].tolist()
        assert pos[:4] == [0, 1, 2, 3] and pos[-32:] == list(range(T - 32, T))
    arena.close()


def test_full_size_prompt_scores_and_large_ratio_eviction():
    """One LLaMA-3-8B-shaped layer with a prompt of 32768 tokens per cache: the scores' total mass
    and the last 128 columns of two caches against the oracle (those need only the last rows'
    normalisers), then one eviction from 32768 rows to ragged budgets of 128..16384 rows with the
    kept lists judged on the kernel's scores."""
    H = _h()
    T = 32768
    w = synth.shrink(synth.WORKLOADS["llama32"], name="prefill32k", L=1, Hq=32, Hkv=8, batch=1, seed=32, sink=4,
                     recent=64, slack=T)
    budgets = [128, 16384, 4096, 700, 9999, 2048, 333, 12000]
    arena = H.make_arena(w, budgets)
    dev = arena.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    q = torch.randn((1, w.Hq, T, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    kd = torch.randn((1, w.Hkv, T, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vd = torch.randn((1, w.Hkv, T, w.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    for c in range(arena.n_caches):
        o = int(arena.off_host[c])
        arena.k[o:o + T].copy_(kd[0, c])
        arena.v[o:o + T].copy_(vd[0, c])
        arena.pos[o:o + T].copy_(torch.arange(T, dtype=torch.int32, device=dev))
    arena.set_lengths(np.full(arena.n_caches, T, dtype=np.int32))
    _, _, lse = B.profile_similarity(q, kd, vd, want_cos=False, want_lse=True)
    B.prefill_scores(q, arena.k, lse, arena.score, 1, w.Hq, w.Hkv, T, row_off=arena.off)
    torch.cuda.synchronize()
    G = w.G
    tail = 128
    for c in range(arena.n_caches):
        o = int(arena.off_host[c])
        got = arena.score[o:o + T].cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got)) and np.all(got >= 0)
        assert abs(got.sum() - G * T) <= 1e-4 * G * T
        assert 0 < got[-1] <= G + 1e-4
        if c in (0, 5):
            # columns j >= T - tail: only rows t >= j contribute, each needs its full softmax
            q64 = synth.storage_to_f64(H.from_device_storage(q[0, c * G:(c + 1) * G, T - tail:], "bf16"), "bf16")
            k64 = synth.storage_to_f64(H.from_device_storage(kd[0, c], "bf16"), "bf16")
            want = np.zeros(tail)
            for g in range(G):
                for i in range(tail):
                    t = T - tail + i
                    s = (k64[: t + 1] @ q64[g, i]) / np.sqrt(w.D)
                    p = np.exp(s - s.max())
                    p /= p.sum()
                    want[: i + 1] += p[T - tail: t + 1]
            err = np.abs(got[-tail:] - want) / np.maximum(1.0, want)
            assert err.max() <= SCORE_RTOL, f"cache {c}: {err.max():.3e}"
    st = H.download(arena, w)
    from test_gpu_compact import run_compact_and_check
    run_compact_and_check(arena, w, st)
    assert arena.lengths().tolist() == budgets
    arena.close()


def test_longest_context_prompt_through_both_prompt_kernels():
    """A prompt of 131072 tokens (the longest context any workload names), 4 query heads on 2 KV
    heads: the profiling kernel's per-token cosines on the first 1024 tokens (oracle, token by token)
    and on sampled late tokens (Eq. 1 row by row through the oracle's attention), its log-sum-exp
    on the same tokens, then the prompt-wide scores: total mass G*T per cache and the last 64
    columns against their definition."""
    H = _h()
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(515)
    Hq, Hkv, T, D = 4, 2, 131072, 128
    G = Hq // Hkv
    q = torch.randn((1, Hq, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((1, Hkv, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((1, Hkv, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    sim, cos, lse = B.profile_similarity(q, k, v, want_cos=True, want_lse=True)
    score = torch.full((Hkv * T,), float("nan"), dtype=torch.float32, device=dev)
    B.prefill_scores(q, k, lse, score, 1, Hq, Hkv, T)
    torch.cuda.synchronize()
    cos_h = cos.cpu().numpy().astype(np.float64)
    lse_h = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(cos_h)) and np.all(np.abs(cos_h) <= 1.0 + 1e-5)
    assert np.allclose(sim.cpu().numpy()[0], cos_h[0].mean(axis=1), rtol=0, atol=1e-5)
    head = 3
    q64 = synth.storage_to_f64(H.from_device_storage(q[0, head], "bf16"), "bf16")
    k64 = synth.storage_to_f64(H.from_device_storage(k[0, head // G], "bf16"), "bf16")
    v64 = synth.storage_to_f64(H.from_device_storage(v[0, head // G], "bf16"), "bf16")
    # the first tokens depend on nothing later: the oracle on the prefix is the oracle on the prompt
    _, want = O.head_similarity(q64[:1024], k64[:1024], v64[:1024])
    assert np.max(np.abs(cos_h[0, head, :1024] - want)) <= 1e-4
    assert np.max(np.abs(lse_h[0, head, :1024] - oracle_lse2(q64[:1024], k64[:1024]))) <= LSE_TOL
    for t in (1024, 65535, 65536, 100000, T - 129, T - 128, T - 2, T - 1):
        out, _ = O.decode_attn(q64[t][None, :], k64[: t + 1], v64[: t + 1])     # Eq. 1 for token t alone
        c = float(v64[t] @ out[0]) / max(float(np.linalg.norm(v64[t]) * np.linalg.norm(out[0])), O.COS_EPS)
        assert abs(cos_h[0, head, t] - c) <= 1e-4, f"token {t}"
        s = (k64[: t + 1] @ q64[t]) / np.sqrt(D) * np.log2(np.e)
        assert abs(lse_h[0, head, t] - (s.max() + np.log2(np.sum(np.exp2(s - s.max()))))) <= LSE_TOL, f"token {t}"
    got = score.cpu().numpy().astype(np.float64).reshape(Hkv, T)
    assert np.all(np.isfinite(got)) and np.all(got >= 0)
    tail = 64
    for c in range(Hkv):
        assert abs(got[c].sum() - G * T) <= 1e-4 * G * T
    qt = synth.storage_to_f64(H.from_device_storage(q[0, G:2 * G, T - tail:], "bf16"), "bf16")   # heads of KV head 1
    want = np.zeros(tail)
    for g in range(G):
        for i in range(tail):
            t = T - tail + i
            s = (k64[: t + 1] @ qt[g, i]) / np.sqrt(D)
            p = np.exp(s - s.max())
            p /= p.sum()
            want[: i + 1] += p[T - tail: t + 1]
    err = np.abs(got[1, -tail:] - want) / np.maximum(1.0, want)
    assert err.max() <= SCORE_RTOL, f"{err.max():.3e}"
