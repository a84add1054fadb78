"""GPU parity over the whole life of a cache set: start empty, grow by fused appends, evict
periodically, reset and start again -- for the shapes and policies the other step tests do not
cover (fp32, D = 64, 16 query heads per KV head, streaming policy, changing split size)."""
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


def run_from_empty(w, budgets, policy, steps, chunks, kernel=B.KERNEL_AUTO, track=True):
    H = _h()
    rng = np.random.Generator(np.random.PCG64(w.seed))
    arena = H.make_arena(w, budgets, track=track, policy=policy)
    arena.set_option(B.OPT_KERNEL, kernel)
    cpl = w.batch * w.Hkv
    caches = [O.Cache(w.D) for _ in range(arena.n_caches)]
    for round_ in range(2):                          # second round after baklava_reset
        for t in range(1, steps + 1):
            H.set_chunk(arena, chunks[t % len(chunks)])
            q, q64 = H.make_q(w, rng, w.L)
            knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
            vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
            outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
            arena.append_decode_attn(0, w.L, H.to_device_storage(knew, w.dtype, arena.device),
                                     H.to_device_storage(vnew, w.dtype, arena.device), t,
                                     H.to_device_storage(q, w.dtype, arena.device), outd)
            torch.cuda.synchronize()
            out = outd.cpu().numpy().astype(np.float64)
            k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
            post = H.download(arena, w)
            for c in range(arena.n_caches):
                l, b, hs = H.q_rows_of_cache(w, c)
                h = c % w.Hkv
                oc = caches[c]
                ref, _, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, h], v64[l, b, h], t, t, 0, 0, 0, 0, track)
                assert post.K[c].shape[0] == oc.n
                assert np.max(np.abs(out[l, b, hs] - ref)) <= H.ATTN_TOL, f"round {round_} step {t} cache {c}"
                if track:
                    serr = np.abs(post.score[c].astype(np.float64) - oc.score)
                    assert np.all((serr <= 2e-3) | (serr <= 2e-3 * np.abs(oc.score)))
                    oc.score = post.score[c].astype(np.float64)      # step-local: continue from the GPU's fp32 scores
            if t % w.interval == 0:
                kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device)
                arena.compact(0, w.L, kept_dev)
                torch.cuda.synchronize()
                after = H.download(arena, w)
                for c in range(arena.n_caches):
                    bud = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
                    kept = caches[c].compact(bud, w.sink, w.recent, policy)
                    o = int(arena.off_host[c])
                    assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32))
                    assert np.array_equal(synth.storage_to_f64(after.K[c], w.dtype), caches[c].K)
                    assert np.array_equal(after.pos[c], caches[c].pos)
            assert arena.lengths().tolist() == arena.len.cpu().tolist() == [oc.n for oc in caches]
        arena.reset()
        torch.cuda.synchronize()
        assert arena.len.cpu().tolist() == [0] * arena.n_caches
        caches = [O.Cache(w.D) for _ in range(arena.n_caches)]
    arena.close()


@pytest.mark.parametrize("dtype,D,Hq,Hkv,policy", [
    ("bf16", 128, 16, 1, B.POLICY_SCORE),       # 16 query heads per KV head: MFMA only
    ("bf16", 128, 6, 2, B.POLICY_STREAMING),
    ("bf16", 64, 8, 2, B.POLICY_SCORE),         # vector-ALU kernel, 128-byte rows
    ("f32", 128, 4, 2, B.POLICY_SCORE),         # vector-ALU kernel, 512-byte rows
    ("f32", 64, 7, 1, B.POLICY_STREAMING),
])
def test_grow_from_empty_evict_reset(dtype, D, Hq, Hkv, policy):
    w = synth.shrink(synth.WORKLOADS["long"], name="life", L=2, Hq=Hq, Hkv=Hkv, D=D, batch=2, dtype=dtype,
                     seed=61, sink=3, recent=0 if policy == B.POLICY_STREAMING else 5, interval=9, slack=9)
    budgets = [40, 300, 270, 17][: w.L * w.Hkv]
    run_from_empty(w, budgets, policy, steps=30, chunks=[256, 512, 1024])


@pytest.mark.parametrize("policy", [B.POLICY_STREAMING, B.POLICY_SCORE])
def test_evict_every_step(policy):
    """Eviction after every decode step (capacity = budget + 1): under the streaming policy each cache
    is a sliding window behind its sink rows; under the score policy one middle row leaves per step.
    Caches that have not reached their budget yet pass through the eviction unchanged."""
    w = synth.shrink(synth.WORKLOADS["long"], name="every", L=2, Hq=8, Hkv=2, D=128, batch=2, dtype="bf16",
                     seed=62, sink=3, recent=0 if policy == B.POLICY_STREAMING else 5, interval=1, slack=1)
    budgets = [12, 45, 30, 8]
    run_from_empty(w, budgets, policy, steps=60, chunks=[256])


def test_two_contexts_used_alternately():
    """Two arenas of different shapes on one device, their calls interleaved on the same stream: a
    context keeps all of its state in its own workspace, so neither disturbs the other."""
    H = _h()
    wa = synth.shrink(synth.WORKLOADS["long"], name="ctxA", L=2, Hq=8, Hkv=2, D=128, batch=2, dtype="bf16", seed=71,
                      sink=2, recent=4, slack=16, interval=4)
    wb = synth.shrink(synth.WORKLOADS["long"], name="ctxB", L=1, Hq=7, Hkv=1, D=128, batch=3, dtype="bf16", seed=72,
                      sink=1, recent=2, slack=16, interval=4)
    ba, bb = [700, 90, 300, 1500], [400]
    ra, rb = np.random.Generator(np.random.PCG64(71)), np.random.Generator(np.random.PCG64(72))
    A, Bn = H.make_arena(wa, ba, track=True), H.make_arena(wb, bb, track=True)
    cpl_a = wa.batch * wa.Hkv
    sta = H.fill_from_host(A, wa, [ba[(c // cpl_a) * wa.Hkv + c % wa.Hkv] for c in range(A.n_caches)], ra, scores="zero")
    stb = H.fill_from_host(Bn, wb, [bb[0]] * Bn.n_caches, rb, scores="zero")
    for t in range(1, 6):
        calls = []
        for arena, w, r in ((A, wa, ra), (Bn, wb, rb)):
            q, q64 = H.make_q(w, r, w.L)
            knew, vnew = synth.payload(r, (w.L, w.batch, w.Hkv, w.D), "bf16"), synth.payload(r, (w.L, w.batch, w.Hkv, w.D), "bf16")
            outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
            calls.append((arena, w, H.download(arena, w), q64, knew, vnew, outd,
                          H.to_device_storage(q, "bf16", arena.device), H.to_device_storage(knew, "bf16", arena.device),
                          H.to_device_storage(vnew, "bf16", arena.device)))
        # layer by layer, the two contexts taking turns, no synchronisation in between
        for l in range(2):
            for arena, w, _, _, _, _, outd, qd, kd, vd in calls:
                if l < w.L:
                    arena.append_decode_attn(l, 1, kd[l], vd[l], 900 + t, qd[l], outd[l])
        if t % 4 == 0:
            A.compact(0, wa.L)
            Bn.compact(0, wb.L)
        torch.cuda.synchronize()
        for arena, w, pre, q64, knew, vnew, outd, _, _, _ in calls:
            out = outd.cpu().numpy().astype(np.float64)
            k64, v64 = synth.storage_to_f64(knew, "bf16"), synth.storage_to_f64(vnew, "bf16")
            budgets = ba if arena is A else bb
            cpl = w.batch * w.Hkv
            post = H.download(arena, w)
            for c in range(arena.n_caches):
                l, b, hs = H.q_rows_of_cache(w, c)
                h = c % w.Hkv
                oc = H.oracle_cache(w, pre, c)
                ref, _, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, h], v64[l, b, h], 900 + t, t, 0, 0, 0, 0, True)
                assert np.max(np.abs(out[l, b, hs] - ref)) <= H.ATTN_TOL, f"step {t} cache {c}"
                if t % 4 == 0:
                    # selection judged on fp32 scores within tolerance of the oracle's: lengths only here
                    assert post.K[c].shape[0] == min(oc.n, budgets[(c // cpl) * w.Hkv + c % w.Hkv])
                else:
                    serr = np.abs(post.score[c].astype(np.float64) - oc.score)
                    assert np.all((serr <= 2e-3) | (serr <= 2e-3 * np.abs(oc.score)))
    A.close()
    Bn.close()
