"""GPU parity on seeded random configurations: shapes, ragged lengths, schedules, launch ranges,
policies and kernels drawn together, so that combinations the systematic tests do not enumerate
are still visited.  Each configuration runs three decode steps (fused append, attention, score
update) and one eviction, judged step-locally against the oracle as in test_gpu_steps.py."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu

SCORE_TOL = 2e-3

# (dtype, D, Hq, Hkv, kernels that serve the shape)
SHAPES = [
    ("bf16", 128, 8, 2, (B.KERNEL_VALU, B.KERNEL_MFMA)), ("bf16", 128, 7, 1, (B.KERNEL_VALU, B.KERNEL_MFMA)),
    ("bf16", 128, 4, 4, (B.KERNEL_VALU, B.KERNEL_MFMA)), ("bf16", 128, 12, 1, (B.KERNEL_MFMA,)),
    ("bf16", 128, 32, 2, (B.KERNEL_MFMA,)), ("bf16", 128, 5, 5, (B.KERNEL_VALU, B.KERNEL_MFMA)),
    ("bf16", 64, 6, 2, (B.KERNEL_VALU,)), ("f32", 64, 8, 1, (B.KERNEL_VALU,)), ("f32", 128, 3, 1, (B.KERNEL_VALU,)),
]


def _h():
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("seed", list(range(300, 324)))
def test_seeded_random_configuration(seed):
    H = _h()
    r = np.random.Generator(np.random.PCG64(seed))
    dtype, D, Hq, Hkv, kernels = SHAPES[int(r.integers(len(SHAPES)))]
    kernel = kernels[int(r.integers(len(kernels)))]
    L, batch = int(r.integers(1, 4)), int(r.integers(1, 4))
    policy = B.POLICY_STREAMING if seed % 3 == 0 else B.POLICY_SCORE
    sink = int(r.integers(0, 5))
    recent = 0 if policy == B.POLICY_STREAMING else int(r.integers(0, 9))
    slack = int(r.choice([3, 8, 40, 300]))
    w = synth.shrink(synth.WORKLOADS["long"], name=f"random{seed}", L=L, Hq=Hq, Hkv=Hkv, D=D, batch=batch, dtype=dtype,
                     seed=seed, sink=sink, recent=recent, slack=slack, interval=3)
    # budgets from a few rows to a few thousand, log-uniform; lengths anywhere from 1 row to 2 below capacity
    budgets = [int(max(sink + recent + 1, round(float(np.exp(r.uniform(np.log(8), np.log(3000))))))) for _ in range(L * Hkv)]
    arena = H.make_arena(w, budgets, track=True, policy=policy)
    arena.set_option(B.OPT_KERNEL, kernel)
    H.set_chunk(arena, int(r.choice([256, 512, 1024])))
    target = int(r.choice([0, 1, 5, 64]))
    arena.set_option(B.OPT_TARGET_ITEMS, target)
    arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
    cpl = batch * Hkv
    cap = arena.cap_host
    lens = [int(r.integers(1, max(2, int(cap[c]) - 2))) for c in range(arena.n_caches)]
    H.fill_from_host(arena, w, lens, r, scores="uniform", peaked=bool(r.random() < 0.3))
    whole = bool(r.random() < 0.5)             # one launch over all layers, or one per layer
    print(f"seed {seed}: {dtype} D={D} Hq={Hq} Hkv={Hkv} L={L} batch={batch} kernel={kernel} policy={policy} "
          f"sink={sink} recent={recent} slack={slack} target={target} whole={whole} budgets={budgets}", flush=True)
    dev = arena.device
    for t in range(1, 4):
        pre = H.download(arena, w)
        if any(pre.K[c].shape[0] >= int(cap[c]) for c in range(arena.n_caches)):
            break                              # a cache is full: the next append would be refused
        q, q64 = H.make_q(w, r, L, scale=float(r.choice([1.0, 3.0])))
        knew, vnew = synth.payload(r, (L, batch, Hkv, D), dtype), synth.payload(r, (L, batch, Hkv, D), dtype)
        kd, vd, qd = (H.to_device_storage(a, dtype, dev) for a in (knew, vnew, q))
        outd = torch.full((L, batch, Hq, D), float("nan"), dtype=torch.float32, device=dev)
        token_pos = 5000 + t
        if whole:
            arena.append_decode_attn(0, L, kd, vd, token_pos, qd, outd)
        else:
            for l in range(L):
                arena.append_decode_attn(l, 1, kd[l], vd[l], token_pos, qd[l], outd[l])
        torch.cuda.synchronize()
        out = outd.cpu().numpy().astype(np.float64)
        post = H.download(arena, w)
        k64, v64 = synth.storage_to_f64(knew, dtype), synth.storage_to_f64(vnew, dtype)
        for c in range(arena.n_caches):
            l, b, hs = H.q_rows_of_cache(w, c)
            h = c % Hkv
            oc = H.oracle_cache(w, pre, c)
            ref, _, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, h], v64[l, b, h], token_pos, t,
                                      budget=0, sink=0, recent=0, interval=0, track_scores=True)
            assert post.K[c].shape[0] == pre.K[c].shape[0] + 1 and post.pos[c][-1] == token_pos
            assert np.array_equal(post.K[c][-1], knew[l, b, h]) and np.array_equal(post.V[c][-1], vnew[l, b, h])
            err = float(np.max(np.abs(out[l, b, hs] - ref)))
            assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
            serr = np.abs(post.score[c].astype(np.float64) - oc.score)
            assert np.all((serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(oc.score))), f"step {t} cache {c}: scores"
    # nothing was written beyond the rows the appends filled: the rest of every cache is still NaN
    torch.cuda.synchronize()
    live = arena.len.cpu().numpy()
    for c in range(arena.n_caches):
        o, n, cp = int(arena.off_host[c]), int(live[c]), int(cap[c])
        if n < cp:
            assert bool(torch.isnan(arena.k[o + n:o + cp].float()).all()) and bool(torch.isnan(arena.v[o + n:o + cp].float()).all())
            assert bool(torch.isnan(arena.score[o + n:o + cp]).all()) and bool((arena.pos[o + n:o + cp] == -1).all())
    # one eviction, judged on the device's own scores
    st = H.download(arena, w)
    kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
    arena.compact(0, L, kept_dev)
    torch.cuda.synchronize()
    after = H.download(arena, w)
    for c in range(arena.n_caches):
        bud = budgets[(c // cpl) * Hkv + c % Hkv]
        n = st.K[c].shape[0]
        kept = O.compact_select(st.score[c], n, bud, sink, recent, policy)
        o = int(arena.off_host[c])
        assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32)), f"cache {c}"
        assert after.K[c].shape[0] == len(kept) == min(n, bud)
        assert np.array_equal(after.K[c], st.K[c][kept]) and np.array_equal(after.V[c], st.V[c][kept])
        assert np.array_equal(after.score[c].view(np.uint32), st.score[c][kept].view(np.uint32))
        assert np.array_equal(after.pos[c], st.pos[c][kept])
    assert arena.lengths().tolist() == arena.len.cpu().tolist() == [k.shape[0] for k in after.K]
    arena.close()


# (Hq, Hkv) of the shapes the MFMA kernel serves; score tracking defers its updates on that kernel only
LAG_SHAPES = [(1, 1), (4, 2), (3, 1), (8, 2), (4, 1), (7, 1), (5, 5), (16, 2), (8, 1), (12, 1), (32, 2), (9, 3)]


@pytest.mark.parametrize("seed", list(range(400, 416)))
def test_seeded_random_windows_of_deferred_score_updates(seed):
    """Random shapes, schedules and call patterns for the deferred score update: windows of decode steps
    with no read-back in between (so that records fill, are applied by later calls and carry over), a
    flush of a random layer range now and then, an eviction after each window.  The oracle follows every
    window in fp64 from the device's state at its start; attention is compared step by step, the score
    plane at the end of the window, the eviction on the device's own scores."""
    H = _h()
    r = np.random.Generator(np.random.PCG64(seed))
    Hq, Hkv = LAG_SHAPES[int(r.integers(len(LAG_SHAPES)))]
    L, batch = int(r.integers(1, 4)), int(r.integers(1, 4))
    sink, recent = int(r.integers(0, 5)), int(r.integers(0, 9))
    slack = int(r.choice([6, 13, 24]))
    w = synth.shrink(synth.WORKLOADS["long"], name=f"window{seed}", L=L, Hq=Hq, Hkv=Hkv, batch=batch, seed=seed,
                     sink=sink, recent=recent, slack=slack, interval=slack)
    budgets = [int(max(sink + recent + 1, round(float(np.exp(r.uniform(np.log(8), np.log(5000))))))) for _ in range(L * Hkv)]
    arena = H.make_arena(w, budgets, track=True)
    arena.set_option(B.OPT_KERNEL, B.KERNEL_MFMA)
    target = int(r.choice([-1, 0, 1, 5, 64]))
    if target >= 0:
        H.set_chunk(arena, int(r.choice([256, 512, 1024])))
        arena.set_option(B.OPT_TARGET_ITEMS, target)
        arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
    fused = bool(r.random() < 0.6)
    cpl = batch * Hkv
    # lengths anywhere from one row up to the budget, or within a few rows of the budget
    lens = [int(r.integers(1, int(arena.cap_host[c]) - slack + 1)) if r.random() < 0.5
            else max(1, budgets[(c // cpl) * Hkv + c % Hkv] - int(r.integers(0, 4))) for c in range(arena.n_caches)]
    H.fill_from_host(arena, w, lens, r, scores="uniform", peaked=bool(r.random() < 0.3))
    print(f"seed {seed}: Hq={Hq} Hkv={Hkv} L={L} batch={batch} sink={sink} recent={recent} slack={slack} target={target} "
          f"fused={fused} budgets={budgets}", flush=True)
    dev = arena.device
    t = 0
    for window in range(3):
        start = H.download(arena, w)
        caches = [H.oracle_cache(w, start, c) for c in range(arena.n_caches)]
        room = min(int(arena.cap_host[c]) - start.K[c].shape[0] for c in range(arena.n_caches))
        steps = int(r.integers(1, room + 1)) if room > 0 else 0
        for _ in range(steps):
            t += 1
            q, q64 = H.make_q(w, r, L, scale=float(r.choice([1.0, 3.0])))
            knew, vnew = synth.payload(r, (L, batch, Hkv, w.D), w.dtype), synth.payload(r, (L, batch, Hkv, w.D), w.dtype)
            kd, vd, qd = (H.to_device_storage(a, w.dtype, dev) for a in (knew, vnew, q))
            outd = torch.full((L, batch, Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
            whole = bool(r.random() < 0.4)
            if not fused:
                arena.append(0, L, kd, vd, 7000 + t)
            if whole:
                arena.append_decode_attn(0, L, kd, vd, 7000 + t, qd, outd) if fused else arena.decode_attn(0, L, qd, outd)
            else:
                for l in range(L):
                    if fused:
                        arena.append_decode_attn(l, 1, kd[l], vd[l], 7000 + t, qd[l], outd[l])
                    else:
                        arena.decode_attn(l, 1, qd[l], outd[l])
            if r.random() < 0.15:                          # scores asked for in mid-window, for some of the layers
                lb = int(r.integers(0, L))
                arena.flush_scores(lb, int(r.integers(1, L - lb + 1)))
            torch.cuda.synchronize()
            out = outd.cpu().numpy().astype(np.float64)
            k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
            for c in range(arena.n_caches):
                l, b, hs = H.q_rows_of_cache(w, c)
                ref, _, _ = O.decode_step(caches[c], q64[l, b, hs], k64[l, b, c % Hkv], v64[l, b, c % Hkv], 7000 + t, t,
                                          budget=0, sink=0, recent=0, interval=0, track_scores=True)
                err = float(np.max(np.abs(out[l, b, hs] - ref)))
                assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
        post = H.download(arena, w)
        for c in range(arena.n_caches):
            oc = caches[c]
            assert post.K[c].shape[0] == oc.n and np.array_equal(post.pos[c], oc.pos[:oc.n])
            serr = np.abs(post.score[c].astype(np.float64) - oc.score[:oc.n])
            assert np.all((serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(oc.score[:oc.n]))), \
                f"window {window} ({steps} steps), cache {c}: score error {serr.max():.3e}"
        kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
        arena.compact(0, L, kept_dev)
        torch.cuda.synchronize()
        after = H.download(arena, w)
        for c in range(arena.n_caches):
            bud = budgets[(c // cpl) * Hkv + c % Hkv]
            n = post.K[c].shape[0]
            kept = O.compact_select(post.score[c], n, bud, sink, recent)
            o = int(arena.off_host[c])
            assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32)), f"cache {c}"
            assert after.K[c].shape[0] == len(kept) == min(n, bud)
            assert np.array_equal(after.K[c], post.K[c][kept]) and np.array_equal(after.V[c], post.V[c][kept])
            assert np.array_equal(after.score[c].view(np.uint32), post.score[c][kept].view(np.uint32))
        assert arena.lengths().tolist() == arena.len.cpu().tolist() == [k.shape[0] for k in after.K]
    arena.close()
