"""The attention entry points only enqueue kernels, so a decode step can be captured into a HIP graph
and replayed: every replay is checked against the eager result and the oracle."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu


def _h():
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("track,warm", [(False, True), (True, True), (True, False)])
def test_decode_step_replays_from_a_graph(track, warm):
    """warm = False: the capture holds the context's very first launches (everything a launch needs
    beyond the launch itself was set up when the context was created)."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="graph", L=3, Hq=8, Hkv=2, batch=2, seed=51, slack=64)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [900, 300, 2500, 80, 700, 1300]
    arena = H.make_arena(w, budgets, track=track)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] + (c * 11) % 60 for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng, scores="zero")
    dev = arena.device
    q_static = torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.bfloat16, device=dev)
    out_static = torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.float32, device=dev)

    def step():
        for l in range(w.L):                       # one launch per layer, as a model issues them
            arena.decode_attn(l, 1, q_static[l], out_static[l])

    if warm:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                 # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
    arena.flush_scores(0, w.L)                     # the warm-up's weights, before the plane is cleared
    torch.cuda.synchronize()
    arena.score.zero_()                            # the warm-up accumulated scores when tracking is on
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        q, q64 = H.make_q(w, rng, w.L)
        q_static.copy_(H.to_device_storage(q, w.dtype, dev))
        torch.cuda.synchronize()                   # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        got = out_static.cpu().numpy().astype(np.float64)
        H.check_decode_against_oracle(arena, w, st, q64, got)
        eager = torch.full_like(out_static, float("nan"))
        for l in range(w.L):                       # the same launches, issued eagerly
            arena.decode_attn(l, 1, q_static[l], eager[l])
        torch.cuda.synchronize()
        assert torch.equal(eager, out_static)
        if track:
            # both the replay and the eager step added this step's attention: 2 * G per cache and step
            G = w.G
            arena.flush_scores(0, w.L)             # the latest call's weights may still be owed
            sc = arena.score.cpu().numpy().astype(np.float64)
            for c in range(arena.n_caches):
                o = int(arena.off_host[c])
                assert abs(sc[o:o + lens[c]].sum() - 2 * G * (rep + 1)) <= 1e-3
    arena.close()


def _replay_setup(track, slack, seed):
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="graphstep", L=3, Hq=8, Hkv=2, batch=2, seed=seed, slack=slack,
                     interval=slack, sink=4, recent=16)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [900, 300, 2500, 80, 700, 1300]
    arena = H.make_arena(w, budgets, track=track)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    dev = arena.device
    bufs = {
        "q": torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.bfloat16, device=dev),
        "k": torch.zeros((w.L, w.batch, w.Hkv, w.D), dtype=torch.bfloat16, device=dev),
        "v": torch.zeros((w.L, w.batch, w.Hkv, w.D), dtype=torch.bfloat16, device=dev),
        "out": torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.float32, device=dev),
        "pos": torch.zeros((1,), dtype=torch.int32, device=dev),
    }

    def step():
        for l in range(w.L):                       # Eq. 7 for one layer as one launch: append, then attend
            arena.append_decode_attn_replay(l, 1, bufs["k"][l], bufs["v"][l], bufs["pos"], bufs["q"][l], bufs["out"][l])

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                  # the capture holds the context's very first launches
        step()
    return H, w, rng, budgets, arena, st, bufs, graph


@pytest.mark.parametrize("track", [False, True])
def test_fused_step_replays_from_a_graph_across_evictions(track):
    """One captured decode step (fused append + attention for every layer; the token position and the
    room left in each cache are read on the device) is replayed for 8 steps with an eviction after
    every third one.  Every replay is checked against the oracle and against a second arena that
    takes the same steps through the eager entry point."""
    H, w, rng, budgets, arena, st, bufs, graph = _replay_setup(track, slack=3, seed=53)
    eager = H.make_arena(w, budgets, track=track)
    rng_e = np.random.Generator(np.random.PCG64(w.seed))
    H.fill_from_host(eager, w, st.lens(), rng_e, scores="uniform")       # the same seeded contents
    dev = arena.device
    caches = [H.oracle_cache(w, st, c) for c in range(arena.n_caches)]
    every = range(arena.n_caches)
    for t in range(1, 9):
        q, q64 = H.make_q(w, rng, w.L)
        knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        for name, a in (("q", q), ("k", knew), ("v", vnew)):
            bufs[name].copy_(H.to_device_storage(a, w.dtype, dev))
        bufs["pos"].fill_(7000 + t)
        torch.cuda.synchronize()                   # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        out = bufs["out"].cpu().numpy().astype(np.float64)
        out_e = torch.full_like(bufs["out"], float("nan"))
        for l in range(w.L):
            eager.append_decode_attn(l, 1, bufs["k"][l], bufs["v"][l], 7000 + t, bufs["q"][l], out_e[l])
        torch.cuda.synchronize()
        assert torch.equal(out_e, bufs["out"]), f"step {t}: replay and eager launches differ"
        k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
        for c in every:
            l, b, hs = H.q_rows_of_cache(w, c)
            ref, _, _ = O.decode_step(caches[c], q64[l, b, hs], k64[l, b, c % w.Hkv], v64[l, b, c % w.Hkv], 7000 + t, t,
                                      budget=0, sink=0, recent=0, interval=0, track_scores=track)
            err = float(np.max(np.abs(out[l, b, hs] - ref)))
            assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
        if t % w.interval == 0:
            arena.sync_lengths()                   # the replays moved the lengths on the device only
            assert arena.lengths().tolist() == arena.len.cpu().tolist() == eager.lengths().tolist()
            post = H.download(arena, w)
            for c in every:
                oc = caches[c]
                assert post.K[c].shape[0] == oc.n and np.array_equal(post.pos[c], oc.pos)
                serr = np.abs(post.score[c].astype(np.float64) - oc.score)
                assert np.all((serr <= 2e-3) | (serr <= 2e-3 * np.abs(oc.score))), f"step {t} cache {c}: scores"
            kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
            arena.compact(0, w.L, kept_dev)
            eager.compact(0, w.L)
            torch.cuda.synchronize()
            after = H.download(arena, w)
            H.check_eviction_against_oracle(arena, w, budgets, post, after, kept_dev, every)
            caches = [H.oracle_cache(w, after, c) for c in every]     # step-local: go on from the device's state
    a, e = H.download(arena, w), H.download(eager, w)
    for c in every:
        assert np.array_equal(a.K[c], e.K[c]) and np.array_equal(a.V[c], e.V[c]) and np.array_equal(a.pos[c], e.pos[c])
        assert np.array_equal(a.score[c].view(np.uint32), e.score[c].view(np.uint32))
    arena.close()
    eager.close()


def test_replayed_step_finds_a_cache_full():
    """Replays beyond the capacity: the full caches receive no row, are attended as they stand, and the
    next baklava_sync_lengths reports it once."""
    H, w, rng, budgets, arena, st, bufs, graph = _replay_setup(False, slack=2, seed=57)
    dev = arena.device
    caches = [H.oracle_cache(w, st, c) for c in range(arena.n_caches)]
    for t in range(1, 4):
        q, q64 = H.make_q(w, rng, w.L)
        knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        for name, a in (("q", q), ("k", knew), ("v", vnew)):
            bufs[name].copy_(H.to_device_storage(a, w.dtype, dev))
        bufs["pos"].fill_(t)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        out = bufs["out"].cpu().numpy().astype(np.float64)
        k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
        for c in range(arena.n_caches):
            l, b, hs = H.q_rows_of_cache(w, c)
            room = t <= w.slack                    # the third step finds every cache full
            ref, _, _ = O.decode_step(caches[c], q64[l, b, hs], k64[l, b, c % w.Hkv] if room else None,
                                      v64[l, b, c % w.Hkv] if room else None, t, t, 0, 0, 0, 0, False)
            assert float(np.max(np.abs(out[l, b, hs] - ref))) <= H.ATTN_TOL, f"step {t} cache {c}"
        if t == 2:
            arena.sync_lengths()                   # nothing to report yet
    with pytest.raises(B.BaklavaError) as e:
        arena.sync_lengths()
    assert e.value.status == B.ECAPACITY
    assert arena.lengths().tolist() == arena.cap_host.tolist() == arena.len.cpu().tolist()
    arena.sync_lengths()                           # reported once
    arena.close()
