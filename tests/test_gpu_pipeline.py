"""GPU parity over the whole chain, stage by stage: profile a prompt (Algorithm 1) -> KV-cache and
layer importances -> two-level budgets (layer pools, Algorithm 2 inside each layer) -> ragged arena
-> prompt-wide scores and the first eviction (Eqs. 5-6) -> decode steps with score tracking and
periodic eviction (Eq. 7).

Every stage is judged against the oracle on the inputs that the previous stage actually produced on
the device: where floating point decides integers (similarities -> budgets, scores -> kept rows)
both sides take the decision on the same fp32 values, so the integer results must agree bit for
bit, and the floating-point values themselves are compared within their own tolerances."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu

MEAN_TOL = 2e-5     # mean cosine of a head / a layer
SCORE_RTOL = 2e-5   # prompt-wide scores, relative to max(1, score)
SCORE_TOL = 2e-3    # scores accumulated during decode steps


def _h():
    import gpu_harness
    return gpu_harness


def test_profile_to_budgets_to_prefill_eviction_to_decode():
    H = _h()
    L, Hq, Hkv, batch, T, D, hidden = 3, 8, 2, 2, 400, 128, 512
    G = Hq // Hkv
    keep = 0.45
    interval = 6
    w = synth.shrink(synth.WORKLOADS["long"], name="pipeline", L=L, Hq=Hq, Hkv=Hkv, batch=batch, seed=77, sink=4,
                     recent=16, slack=T, interval=interval)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    dev = torch.device("cuda:0")

    # ---- stage 1: the prompt.  Heads differ in how peaked their attention is (query scale) so that
    # their similarities, and with them the budgets, spread out.
    q_st, k_st, v_st = [], [], []
    for l in range(L):
        q = synth.storage_to_f64(synth.payload(rng, (batch, Hq, T, D), "bf16"), "bf16")
        q *= np.linspace(0.25, 6.0, Hq)[None, ::(-1 if l % 2 else 1), None, None]
        q_st.append(synth.f32_to_bf16_bits(q.astype(np.float32)))
        k_st.append(synth.payload(rng, (batch, Hkv, T, D), "bf16"))
        v_st.append(synth.payload(rng, (batch, Hkv, T, D), "bf16"))
    qd = [H.to_device_storage(a, "bf16", dev) for a in q_st]
    kd = [H.to_device_storage(a, "bf16", dev) for a in k_st]
    vd = [H.to_device_storage(a, "bf16", dev) for a in v_st]
    q64 = [synth.storage_to_f64(a, "bf16") for a in q_st]
    k64 = [synth.storage_to_f64(a, "bf16") for a in k_st]
    v64 = [synth.storage_to_f64(a, "bf16") for a in v_st]

    # ---- stage 2: Algorithm 1, step 1 on the device; the mean over the sequences of the batch is host work
    sim_gpu = np.zeros((L, Hq))
    lse = []
    for l in range(L):
        sim, _, lse_l = B.profile_similarity(qd[l], kd[l], vd[l], want_cos=False, want_lse=True)
        torch.cuda.synchronize()
        s = sim.cpu().numpy().astype(np.float64)                    # [batch, Hq]
        for b in range(batch):
            for h in range(Hq):
                want, _ = O.head_similarity(q64[l][b, h], k64[l][b, h // G], v64[l][b, h // G])
                assert abs(s[b, h] - want) <= MEAN_TOL, f"layer {l} sequence {b} head {h}"
        sim_gpu[l] = s.mean(axis=0)
        lse.append(lse_l)
    head_imp = B.kv_importance(sim_gpu, L, Hq, Hkv)                # step 2 + normalisation, host
    assert np.array_equal(head_imp, O.kv_importance(sim_gpu, G))
    assert np.ptp(head_imp) > 0.01                                  # the heads really differ

    # ---- stage 3: layer importance from the hidden states on both sides of each layer
    layer_sim = np.zeros(L)
    for l in range(L):
        x_in = synth.storage_to_f64(synth.payload(rng, (batch, T, hidden), "bf16"), "bf16")
        mix = [0.2, 1.0, 3.0][l]                                    # how much the layer changes its input
        x_out = x_in + mix * synth.storage_to_f64(synth.payload(rng, (batch, T, hidden), "bf16"), "bf16")
        xi = torch.from_numpy(x_in).to(torch.bfloat16).to(dev)
        xo = torch.from_numpy(x_out).to(torch.bfloat16).to(dev)
        sim, _ = B.layer_similarity(xi, xo, want_cos=False)
        torch.cuda.synchronize()
        s = sim.cpu().numpy().astype(np.float64)
        for b in range(batch):
            want, _ = O.layer_similarity(xi[b].float().cpu().numpy().astype(np.float64),
                                         xo[b].float().cpu().numpy().astype(np.float64))
            assert abs(s[b] - want) <= MEAN_TOL
        layer_sim[l] = s.mean()
    layer_imp = 1.0 - (layer_sim + 1.0) / 2.0                       # same map as for heads
    assert layer_imp[0] < layer_imp[1] < layer_imp[2]

    # ---- stage 4: budgets (integers): library and oracle on the same importances
    global_budget = int(L * Hkv * T * keep)
    lo, hi = w.sink + w.recent + 8, T
    budgets = B.alloc_two_level(layer_imp, head_imp, global_budget, lo, hi, t=float(np.median(head_imp)), r=0.3)
    assert budgets == O.alloc_two_level(layer_imp, head_imp, global_budget, lo, hi, float(np.median(head_imp)), 0.3)
    assert sum(budgets) == global_budget and min(budgets) >= w.sink + w.recent   # Algorithm 2 does not clip
    assert len(set(budgets)) > 2
    pools = np.asarray(budgets).reshape(L, Hkv).sum(axis=1)
    assert pools[0] <= pools[1] <= pools[2]                         # more important layers get larger pools

    # ---- stage 5: arena with those budgets; the prompt's K/V rows go in; scores come from the device
    arena = H.make_arena(w, budgets, track=True)
    cpl = batch * Hkv
    st = H.HostState(arena.n_caches)
    for c in range(arena.n_caches):
        l, s = divmod(c, cpl)
        b, h = divmod(s, Hkv)
        o = int(arena.off_host[c])
        arena.k[o:o + T].copy_(kd[l][b, h])
        arena.v[o:o + T].copy_(vd[l][b, h])
        arena.pos[o:o + T].copy_(torch.arange(T, dtype=torch.int32, device=dev))
    arena.set_lengths(np.full(arena.n_caches, T, dtype=np.int32))
    for l in range(L):
        B.prefill_scores(qd[l], arena.k, lse[l], arena.score, batch, Hq, Hkv, T,
                         row_off=arena.off[l * cpl:(l + 1) * cpl])
    torch.cuda.synchronize()
    st = H.download(arena, w)
    for c in range(arena.n_caches):
        l, s = divmod(c, cpl)
        b, h = divmod(s, Hkv)
        assert np.array_equal(st.K[c], k_st[l][b, h]) and np.array_equal(st.V[c], v_st[l][b, h])
        want = O.prefill_scores(q64[l][b, h * G:(h + 1) * G], k64[l][b, h])
        got = st.score[c].astype(np.float64)
        assert np.max(np.abs(got - want) / np.maximum(1.0, want)) <= SCORE_RTOL, f"cache {c}"

    # ---- stage 6: the eviction that precedes the decode loop, judged on the device's own scores
    from test_gpu_compact import run_compact_and_check
    st = run_compact_and_check(arena, w, st)
    budget_of = [budgets[(c // cpl) * Hkv + c % Hkv] for c in range(arena.n_caches)]
    n_live = [min(T, b) for b in budget_of]
    assert arena.lengths().tolist() == n_live

    # ---- stage 7: decode steps (fused append, score tracking), eviction every `interval` steps
    worst_out = worst_score = 0.0
    for t in range(1, 2 * interval + 2):
        pre = H.download(arena, w)
        q, qq64 = H.make_q(w, rng, L)
        knew = synth.payload(rng, (L, batch, Hkv, D), "bf16")
        vnew = synth.payload(rng, (L, batch, Hkv, D), "bf16")
        kn, vn = H.to_device_storage(knew, "bf16", dev), H.to_device_storage(vnew, "bf16", dev)
        qdev = H.to_device_storage(q, "bf16", dev)
        outd = torch.full((L, batch, Hq, D), float("nan"), dtype=torch.float32, device=dev)
        token_pos = T - 1 + t
        for l in range(L):
            arena.append_decode_attn(l, 1, kn[l], vn[l], token_pos, qdev[l], outd[l])
        torch.cuda.synchronize()
        out = outd.cpu().numpy().astype(np.float64)
        post = H.download(arena, w)
        kk, vv = synth.storage_to_f64(knew, "bf16"), synth.storage_to_f64(vnew, "bf16")
        for c in range(arena.n_caches):
            l, b, hs = H.q_rows_of_cache(w, c)
            h = c % Hkv
            oc = H.oracle_cache(w, pre, c)
            ref, _, _ = O.decode_step(oc, qq64[l, b, hs], kk[l, b, h], vv[l, b, h], token_pos, t,
                                      budget=0, sink=0, recent=0, interval=0, track_scores=True)
            err = float(np.max(np.abs(out[l, b, hs] - ref)))
            assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
            worst_out = max(worst_out, err)
            serr = np.abs(post.score[c].astype(np.float64) - oc.score)
            assert np.all((serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(oc.score))), f"step {t} cache {c}"
            worst_score = max(worst_score, float(serr.max()))
            assert post.pos[c][-1] == token_pos
        n_live = [n + 1 for n in n_live]
        if t % interval == 0:
            run_compact_and_check(arena, w, post)
            n_live = [min(n, b) for n, b in zip(n_live, budget_of)]
        assert arena.lengths().tolist() == n_live
    print(f"pipeline: budgets {budgets}, worst attention error {worst_out:.3e}, worst score error {worst_score:.3e}",
          flush=True)
    arena.close()
