"""GPU parity over whole decode steps: append -> attention -> score update -> periodic eviction.

Protocol (eviction is a discontinuous function of the scores, so the comparison is made
step-local): before each step the oracle is loaded with the GPU's own pre-step cache state; it
recomputes the step in fp64; outputs and post-step scores must agree within tolerance; the
oracle's selection is then run on the GPU's fp32 post-step scores and must give the GPU's kept
list and lengths bit for bit."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu

SCORE_TOL = 2e-3


def _h():
    import gpu_harness
    return gpu_harness


# the vector-ALU kernel serves at most 8 query heads per KV head
STEP_CASES = [(kernel, fused, base, Hq, Hkv, target, 2)
              for base, Hq, Hkv, target in [("long", 8, 2, 0), ("qwen", 7, 1, 0), ("long", 8, 2, 3), ("long", 16, 1, 1)]
              for fused in (False, True)
              for kernel in (B.KERNEL_VALU, B.KERNEL_MFMA)
              if not (kernel == B.KERNEL_VALU and Hq // Hkv > 8)]
# 9 sequences x 8 KV heads = 72 caches per layer: more than a quarter of the compute units, so the
# library's own defaults (target -1: nothing is set here) give layer launches several waves of work items
STEP_CASES += [(B.KERNEL_MFMA, True, "long", 16, 8, -1, 9), (B.KERNEL_MFMA, False, "long", 16, 8, -1, 9)]


@pytest.mark.parametrize("kernel,fused,base,Hq,Hkv,target,batch", STEP_CASES)
def test_multi_step_with_kernel_updated_scores(kernel, fused, base, Hq, Hkv, target, batch):
    H = _h()
    w = synth.shrink(synth.WORKLOADS[base], name="steps", L=2, Hq=Hq, Hkv=Hkv, batch=batch, ctx=2048, lo=96,
                     hi=2048, interval=8, slack=8, sink=4, recent=16, steps=20 if batch == 2 else 9, floor_frac=0.0)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    assert budgets == synth.budgets_for(w, O.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    arena.set_option(B.OPT_KERNEL, kernel)
    if target >= 0:
        H.set_chunk(arena, 256)
        # target 3: at most 3 work items per layer launch, so work items of up to 2048 rows whose score
        # update spans several workgroups; 16 query heads per KV head with one item per cache: more logits
        # than the attention kernel can hold on chip, so it writes them out in several batches
        arena.set_option(B.OPT_TARGET_ITEMS, target)
        arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)]
    H.fill_from_host(arena, w, lens, rng, scores="zero")
    G = w.G
    worst_out = worst_score = 0.0
    for t in range(1, w.steps + 1):
        pre = H.download(arena, w)
        q, q64 = H.make_q(w, rng, w.L)
        knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        kd = H.to_device_storage(knew, w.dtype, arena.device)
        vd = H.to_device_storage(vnew, w.dtype, arena.device)
        token_pos = 100000 + t
        if fused:
            # one launch per layer: the new row joins each cache inside the attention kernel
            qd = H.to_device_storage(q, w.dtype, arena.device)
            outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
            for l in range(w.L):
                arena.append_decode_attn(l, 1, kd[l], vd[l], token_pos, qd[l], outd[l])
            torch.cuda.synchronize()
            out = outd.cpu().numpy().astype(np.float64)
        else:
            arena.append(0, w.L, kd, vd, token_pos)
            out = H.gpu_decode(arena, w, q)
        post = H.download(arena, w)
        k64 = synth.storage_to_f64(knew, w.dtype)
        v64 = synth.storage_to_f64(vnew, w.dtype)
        for c in range(arena.n_caches):
            l, b, hs = H.q_rows_of_cache(w, c)
            h = c % w.Hkv
            oc = H.oracle_cache(w, pre, c)
            ref, p, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, h], v64[l, b, h], token_pos, t,
                                      budget=0, sink=0, recent=0, interval=0, track_scores=True)
            # append: row bits, pos and length
            assert post.K[c].shape[0] == pre.K[c].shape[0] + 1
            assert np.array_equal(post.K[c][-1], knew[l, b, h]) and np.array_equal(post.V[c][-1], vnew[l, b, h])
            assert post.pos[c][-1] == token_pos
            err = float(np.max(np.abs(out[l, b, hs] - ref)))
            assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
            worst_out = max(worst_out, err)
            serr = np.abs(post.score[c].astype(np.float64) - oc.score)
            ok = (serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(oc.score))
            assert np.all(ok), f"step {t} cache {c}: score error {serr.max():.3e}"
            worst_score = max(worst_score, float(serr.max()))
        if t % w.interval == 0:
            kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device)
            arena.compact(0, w.L, kept_dev)
            torch.cuda.synchronize()
            after = H.download(arena, w)
            for c in range(arena.n_caches):
                bud = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
                kept = O.compact_select(post.score[c], post.K[c].shape[0], bud, w.sink, w.recent)
                o = int(arena.off_host[c])
                assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32)), \
                    f"step {t} cache {c}: kept list"
                assert after.K[c].shape[0] == len(kept) == bud
                assert np.array_equal(after.K[c], post.K[c][kept]) and np.array_equal(after.V[c], post.V[c][kept])
                assert np.array_equal(after.score[c], post.score[c][kept])
                assert np.array_equal(after.pos[c], post.pos[c][kept])
        assert arena.lengths().tolist() == arena.len.cpu().tolist()
    print(f"steps kernel={kernel} G={G}: worst attention error {worst_out:.3e}, worst score error {worst_score:.3e}",
          flush=True)
    arena.close()


# Score tracking adds a call's weights one call late (inside the next attention kernel) unless
# baklava_flush_scores is called; the step-local test above flushes after every step, so the deferred
# path gets a protocol of its own: the state is read back only at the start and the end of each window
# of `interval` steps; inside a window the calls follow each other as a model issues them.
LAG_CASES = [("long", 8, 2, 2, 0, True), ("long", 8, 2, 2, 3, False), ("qwen", 7, 1, 2, 0, True),
             ("long", 16, 1, 2, 1, True), ("long", 16, 8, 9, -1, True), ("long", 4, 4, 3, 2, False)]


@pytest.mark.parametrize("base,Hq,Hkv,batch,target,fused", LAG_CASES)
def test_deferred_score_updates_over_windows_of_steps(base, Hq, Hkv, batch, target, fused):
    H = _h()
    w = synth.shrink(synth.WORKLOADS[base], name="lag", L=2, Hq=Hq, Hkv=Hkv, batch=batch, ctx=2048, lo=96,
                     hi=2048, interval=10, slack=10, sink=4, recent=16, steps=30 if batch < 9 else 20, floor_frac=0.0,
                     seed=77 + Hq)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    arena.set_option(B.OPT_KERNEL, B.KERNEL_MFMA)
    if target >= 0:
        H.set_chunk(arena, 256)
        arena.set_option(B.OPT_TARGET_ITEMS, target)
        arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] - (c % 3) for c in range(arena.n_caches)]
    H.fill_from_host(arena, w, lens, rng, scores="uniform")
    dev = arena.device
    worst_out = worst_score = 0.0
    for t0 in range(0, w.steps, w.interval):
        start = H.download(arena, w)                       # brings the scores up to date first
        caches = [H.oracle_cache(w, start, c) for c in range(arena.n_caches)]
        for t in range(t0 + 1, t0 + w.interval + 1):
            q, q64 = H.make_q(w, rng, w.L)
            knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
            vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
            kd, vd, qd = (H.to_device_storage(a, w.dtype, dev) for a in (knew, vnew, q))
            outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
            whole = t % 3 == 0                             # both launch shapes inside one window
            if fused and whole:
                arena.append_decode_attn(0, w.L, kd, vd, 5000 + t, qd, outd)
            elif fused:
                for l in range(w.L):
                    arena.append_decode_attn(l, 1, kd[l], vd[l], 5000 + t, qd[l], outd[l])
            else:
                arena.append(0, w.L, kd, vd, 5000 + t)
                if whole:
                    arena.decode_attn(0, w.L, qd, outd)
                else:
                    for l in range(w.L):
                        arena.decode_attn(l, 1, qd[l], outd[l])
            torch.cuda.synchronize()
            out = outd.cpu().numpy().astype(np.float64)
            k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
            for c in range(arena.n_caches):
                l, b, hs = H.q_rows_of_cache(w, c)
                ref, _, _ = O.decode_step(caches[c], q64[l, b, hs], k64[l, b, c % w.Hkv], v64[l, b, c % w.Hkv], 5000 + t, t,
                                          budget=0, sink=0, recent=0, interval=0, track_scores=True)
                err = float(np.max(np.abs(out[l, b, hs] - ref)))
                assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
                worst_out = max(worst_out, err)
        # without a flush the plane lacks the weights of the calls still on record, and only those: a record
        # holds 32 / (G rounded up to 4, 8 or 16) calls, and the call that finds it full empties it
        room = 32 // (4 if w.G <= 4 else 8 if w.G <= 8 else 16)
        on_record = 0
        for _ in range(w.interval):
            on_record = 1 if on_record >= room else on_record + 1
        raw = H.download(arena, w, flush=False)
        post = H.download(arena, w)
        for c in range(arena.n_caches):
            oc = caches[c]
            assert post.K[c].shape[0] == oc.n and np.array_equal(post.pos[c], oc.pos[:oc.n])
            serr = np.abs(post.score[c].astype(np.float64) - oc.score[:oc.n])
            assert np.all((serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(oc.score[:oc.n]))), \
                f"window ending at step {t0 + w.interval}, cache {c}: score error {serr.max():.3e}"
            worst_score = max(worst_score, float(serr.max()))
            owed = post.score[c].astype(np.float64).sum() - raw.score[c].astype(np.float64).sum()
            assert abs(owed - on_record * w.G) <= 1e-3, \
                f"cache {c}: the unflushed plane lacks {owed:.6f}, not the weights of {on_record} calls"
        kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
        arena.compact(0, w.L, kept_dev)
        torch.cuda.synchronize()
        H.check_eviction_against_oracle(arena, w, budgets, post, H.download(arena, w), kept_dev, range(arena.n_caches))
        assert arena.lengths().tolist() == arena.len.cpu().tolist()
    print(f"deferred scores G={w.G}: worst attention error {worst_out:.3e}, worst score error {worst_score:.3e}", flush=True)
    arena.close()


def test_scores_sum_to_G_per_step_without_eviction():
    """Each query head's softmax weights sum to 1, so a cache's scores grow by exactly G per step."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["long"], name="sumG", L=1, Hq=8, Hkv=2, batch=1, seed=31, slack=64)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [1500, 300]
    for kernel in (B.KERNEL_VALU, B.KERNEL_MFMA):
        arena = H.make_arena(w, budgets, track=True)
        arena.set_option(B.OPT_KERNEL, kernel)
        H.set_chunk(arena, 512)
        H.fill_from_host(arena, w, budgets, rng, scores="zero")
        for t in range(1, 6):
            q, _ = H.make_q(w, rng, 1)
            kn = H.to_device_storage(synth.payload(rng, (1, 2, w.D), w.dtype), w.dtype, arena.device)
            arena.append(0, 1, kn, kn, t)
            H.gpu_decode(arena, w, q)
            st = H.download(arena, w)
            for c in range(2):
                assert abs(float(st.score[c].astype(np.float64).sum()) - w.G * t) < 1e-3
        arena.close()


def test_free_running_fp64_oracle_on_a_small_replica():
    """The oracle run on its own fp64 scores (not reloaded from the GPU each step): kept lists must
    agree wherever the gap between the last kept and the first evicted score exceeds twice the
    score tolerance; the number of caches inside that margin is reported."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["long"], name="free", L=1, Hq=8, Hkv=2, batch=2, ctx=1024, lo=64, hi=1024,
                     interval=4, slack=4, sink=4, recent=8, steps=12)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    cpl = w.batch * w.Hkv
    lens = [budgets[c % w.Hkv] for c in range(arena.n_caches)]
    st0 = H.fill_from_host(arena, w, lens, rng, scores="zero")
    caches = [H.oracle_cache(w, st0, c) for c in range(arena.n_caches)]
    diverged = [False] * arena.n_caches
    inside_margin = 0
    for t in range(1, w.steps + 1):
        q, q64 = H.make_q(w, rng, w.L)
        knew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        qd = H.to_device_storage(q, w.dtype, arena.device)
        outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
        arena.append_decode_attn(0, 1, H.to_device_storage(knew, w.dtype, arena.device),
                                 H.to_device_storage(vnew, w.dtype, arena.device), t, qd, outd)
        torch.cuda.synchronize()
        out = outd.cpu().numpy().astype(np.float64)
        k64, v64 = synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype)
        do_compact = t % w.interval == 0
        kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device)
        if do_compact:
            arena.compact(0, 1, kept_dev)
            torch.cuda.synchronize()
        for c in range(arena.n_caches):
            if diverged[c]:
                continue
            l, b, hs = H.q_rows_of_cache(w, c)
            oc = caches[c]
            ref, _, _ = O.decode_step(oc, q64[l, b, hs], k64[l, b, c % w.Hkv], v64[l, b, c % w.Hkv], t, t,
                                      0, 0, 0, 0, True)
            assert np.max(np.abs(out[l, b, hs] - ref)) <= H.ATTN_TOL
            if do_compact:
                bud = budgets[c % w.Hkv]
                n = oc.n
                mid = np.sort(oc.score[w.sink:n - w.recent])[::-1]
                k = bud - w.sink - w.recent
                gap = mid[k - 1] - mid[k] if 0 < k < len(mid) else np.inf
                kept = oc.compact(bud, w.sink, w.recent)
                o = int(arena.off_host[c])
                same = np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32))
                if gap > 2 * SCORE_TOL:
                    assert same, f"step {t} cache {c}: lists differ although the score gap is {gap:.3e}"
                elif not same:
                    inside_margin += 1
                    diverged[c] = True
    print(f"free-running oracle: {inside_margin} of {arena.n_caches} caches fell inside the score margin", flush=True)
    arena.close()


def test_256_step_trajectory_on_a_small_replica_of_the_long_workload():
    """The long workload's whole trajectory (256 steps, eviction every 32, scores from the kernel's
    softmax weights) on a replica with 2 layers, one sequence and an 8192-token context: every step
    is checked step-locally on every cache, every eviction bit for bit."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["long"], name="traj", L=2, batch=1, ctx=8192, lo=256, hi=8192)
    assert w.interval == 32 and w.steps == 256 and w.scores == "kernel"
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    assert budgets == synth.budgets_for(w, O.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    cpl = w.batch * w.Hkv
    H.fill_from_host(arena, w, [budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)], rng, scores="zero")
    dev = arena.device
    every = range(arena.n_caches)
    worst = (0.0, 0.0)
    for t in range(1, w.steps + 1):
        pre = H.download(arena, w)
        q, q64 = H.make_q(w, rng, w.L)
        knew, vnew = synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype), synth.payload(rng, (w.L, w.batch, w.Hkv, w.D), w.dtype)
        kd, vd, qd = (H.to_device_storage(a, w.dtype, dev) for a in (knew, vnew, q))
        outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
        for l in range(w.L):
            arena.append_decode_attn(l, 1, kd[l], vd[l], w.ctx + t, qd[l], outd[l])
        torch.cuda.synchronize()
        post = H.download(arena, w)
        e = H.check_step_against_oracle(arena, w, pre, post, outd.cpu().numpy().astype(np.float64), q64,
                                        synth.storage_to_f64(knew, w.dtype), synth.storage_to_f64(vnew, w.dtype),
                                        w.ctx + t, t, every)
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        if t % w.interval == 0:
            kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
            arena.compact(0, w.L, kept_dev)
            torch.cuda.synchronize()
            H.check_eviction_against_oracle(arena, w, budgets, post, H.download(arena, w), kept_dev, every)
        assert arena.lengths().tolist() == arena.len.cpu().tolist()
    print(f"256-step replica: worst attention error {worst[0]:.3e}, worst score error {worst[1]:.3e}", flush=True)
    arena.close()


def test_records_survive_option_changes_and_are_dropped_with_the_rows():
    """What the deferred score update has on record must come out right whatever happens between the
    calls: the other attention kernel takes over (it first adds what is on record), tracking is paused
    and resumed, a flush is repeated (the second one adds nothing), the work-item tables are rebuilt;
    and baklava_set_lengths / baklava_reset drop records together with the rows they belong to."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["long"], name="rec", L=2, Hq=8, Hkv=2, batch=2, ctx=2048, lo=96, hi=2048,
                     interval=64, slack=64, sink=4, recent=16, seed=88, floor_frac=0.0)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng, scores="zero")
    caches = [H.oracle_cache(w, st, c) for c in range(arena.n_caches)]
    dev = arena.device
    counted = 0                                            # calls whose weights the oracle has added

    def call(track=True):
        nonlocal counted
        q, q64 = H.make_q(w, rng, w.L)
        qd = H.to_device_storage(q, w.dtype, dev)
        outd = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
        for l in range(w.L):
            arena.decode_attn(l, 1, qd[l], outd[l])
        torch.cuda.synchronize()
        out = outd.cpu().numpy().astype(np.float64)
        for c in range(arena.n_caches):
            l, b, hs = H.q_rows_of_cache(w, c)
            ref, _, _ = O.decode_step(caches[c], q64[l, b, hs], None, None, 0, 0, 0, 0, 0, 0, track)
            assert float(np.max(np.abs(out[l, b, hs] - ref))) <= H.ATTN_TOL
        counted += 1 if track else 0

    def check_scores(what):
        post = H.download(arena, w)                        # flushes
        for c in range(arena.n_caches):
            serr = np.abs(post.score[c].astype(np.float64) - caches[c].score)
            assert np.all((serr <= SCORE_TOL) | (serr <= SCORE_TOL * np.abs(caches[c].score))), f"{what}: cache {c}, {serr.max():.3e}"
            assert abs(float(post.score[c].astype(np.float64).sum()) - w.G * counted) <= 1e-3, what

    arena.set_option(B.OPT_KERNEL, B.KERNEL_MFMA)
    call(); call(); call()                                 # three calls on record
    arena.set_option(B.OPT_KERNEL, B.KERNEL_VALU)          # the other kernel adds them before its own
    call()
    raw = H.download(arena, w, flush=False)
    for c in range(arena.n_caches):
        assert abs(float(raw.score[c].astype(np.float64).sum()) - w.G * 4) <= 1e-3   # nothing owed after a vector-ALU call
    arena.set_option(B.OPT_KERNEL, B.KERNEL_MFMA)
    call(); call()
    arena.set_option(B.OPT_TRACK_SCORES, 0)                # paused: these leave no record, the two before stay on it
    call(track=False); call(track=False)
    arena.set_option(B.OPT_TRACK_SCORES, 1)
    call()
    H.set_chunk(arena, 256)                                # new work-item tables: the records do not depend on them
    arena.set_option(B.OPT_TARGET_ITEMS, 2)
    for _ in range(9):                                     # the record (8 calls at G = 4) fills up and a call applies it
        call()
    check_scores("after option changes")
    arena.flush_scores(0, w.L)
    arena.flush_scores(0, w.L)                             # nothing on record: adds nothing
    check_scores("after repeated flushes")
    # records are dropped with the rows they belong to
    call(); call()
    arena.set_lengths(lens)                                # the caller declares the rows anew: two calls' weights are gone
    arena.score.zero_()
    for c in range(arena.n_caches):
        caches[c].score[:] = 0.0
    counted = 0
    call()
    check_scores("after set_lengths")
    call()
    arena.reset()
    torch.cuda.synchronize()
    assert arena.lengths().tolist() == [0] * arena.n_caches
    arena.set_lengths(lens)
    arena.score.zero_()
    for c in range(arena.n_caches):
        caches[c].score[:] = 0.0
    counted = 0
    call(); call()
    check_scores("after reset")
    arena.close()


def test_tiled_selection_threshold_does_not_change_the_result():
    """The same eviction with every cache ranked by one workgroup and with the long ones ranked tile by
    tile: identical lists and rows."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="thr", L=1, Hq=4, Hkv=4, batch=1, seed=89, sink=4, recent=64, slack=500)
    budgets = [12000, 40000, 9000, 300]
    results = []
    for rows in (1 << 30, 8192, 16384):
        rng = np.random.Generator(np.random.PCG64(w.seed))
        arena = H.make_arena(w, budgets)
        arena.set_option(B.OPT_TILED_SELECT_ROWS, rows)
        lens = [b + 500 - 37 * i for i, b in enumerate(budgets)]
        st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
        kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device)
        arena.compact(0, 1, kept_dev)
        torch.cuda.synchronize()
        after = H.download(arena, w)
        H.check_eviction_against_oracle(arena, w, budgets, st, after, kept_dev, range(arena.n_caches))
        results.append(kept_dev.cpu().numpy())
        arena.close()
    assert np.array_equal(results[0], results[1]) and np.array_equal(results[0], results[2])
