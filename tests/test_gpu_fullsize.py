"""GPU parity at the benchmark's full sizes, in the launch configurations bench.py times: sampled
caches against the oracle one by one, and properties that hold at any size on all caches."""
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


def sample_caches(arena, lens, rng, n_random=10):
    order = np.argsort(lens)
    picks = {int(order[0]), int(order[1]), int(order[-1]), int(order[-2]), 0, arena.n_caches - 1}
    picks |= {int(x) for x in rng.integers(0, arena.n_caches, n_random)}
    return sorted(picks)


def short_caches(lens, limit=4096, at_most=400):
    """Caches of at most `limit` rows, evenly thinned to `at_most` of them: cheap enough to check one by
    one, so evictions are compared on hundreds of caches rather than on a handful."""
    ids = [c for c in range(len(lens)) if lens[c] <= limit]
    stride = max(1, -(-len(ids) // at_most))
    return ids[::stride]


def check_evictions(H, arena, w, budgets, pre, post, kept_dev, caches, lens):
    cpl = w.batch * w.Hkv
    for c in caches:
        b = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
        kept = O.compact_select(pre.score[c], int(lens[c]), b, w.sink, w.recent)
        o = int(arena.off_host[c])
        got = kept_dev[o:o + len(kept)].cpu().numpy()
        assert np.array_equal(got, np.asarray(kept, dtype=np.int32)), f"cache {c}: kept list"
        assert np.array_equal(post.K[c], pre.K[c][kept]) and np.array_equal(post.V[c], pre.V[c][kept])
        assert np.array_equal(post.score[c].view(np.uint32), pre.score[c][kept].view(np.uint32))
        assert np.array_equal(post.pos[c], pre.pos[c][kept])


@pytest.mark.parametrize("name", ["llama32", "qwen", "long"])
def test_full_size_decode_and_compaction(name):
    H = _h()
    w = synth.WORKLOADS[name]
    rng = np.random.Generator(np.random.PCG64(w.seed + 7))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=(w.scores == "kernel"))
    gen = synth.fill_arena_on_device(arena, w)
    arena.score.copy_(torch.rand((arena.total_tokens,), generator=gen, device=arena.device, dtype=torch.float32))
    cpl = w.batch * w.Hkv
    # steady state between two compactions: every cache somewhere between budget and capacity
    lens = np.array([budgets[(c // cpl) * w.Hkv + c % w.Hkv] + (c * 7) % (w.slack + 1)
                     for c in range(arena.n_caches)], dtype=np.int32)
    lens = np.minimum(lens, arena.cap_host)
    arena.set_lengths(lens)
    tdt = torch.bfloat16
    q = torch.randn((w.L, w.batch, w.Hq, w.D), generator=gen, device=arena.device, dtype=torch.float32).to(tdt)
    out_layer = torch.full((w.L, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
    out_stack = torch.full_like(out_layer, float("nan"))
    for l in range(w.L):                               # the launch configuration bench.py times
        arena.decode_attn(l, 1, q[l], out_layer[l])
    arena.decode_attn(0, w.L, q, out_stack)            # and the single-launch one
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out_layer).all()) and bool(torch.isfinite(out_stack).all())
    # any size: both launch shapes compute the same softmax, only the split points differ
    assert float((out_layer - out_stack).abs().max()) <= 1e-5

    picks = sample_caches(arena, lens, rng)
    many = sorted(set(picks) | set(short_caches(lens)))      # evictions: these as well
    pre = H.download(arena, w, many)
    q64 = synth.storage_to_f64(H.from_device_storage(q, w.dtype), w.dtype)
    ol = out_layer.cpu().numpy().astype(np.float64)
    worst = H.check_decode_against_oracle(arena, w, pre, q64, ol, caches=picks)
    print(f"{name}: {len(picks)} sampled caches, lengths {min(lens[picks])}..{max(lens[picks])}, "
          f"attention max-abs error {worst:.3e}", flush=True)

    # eviction at full size
    kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device)
    arena.compact(0, w.L, kept_dev)
    torch.cuda.synchronize()
    new_len = arena.len.cpu().numpy()
    want = np.minimum(lens, np.array([budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)]))
    assert np.array_equal(new_len, want) and np.array_equal(arena.lengths(), want)
    post = H.download(arena, w, many)
    check_evictions(H, arena, w, budgets, pre, post, kept_dev, many, lens)
    print(f"{name}: eviction lists and moved rows bit-exact on {len(many)} caches", flush=True)
    # any size: every kept list is strictly ascending and starts with the sink rows
    for c in sample_caches(arena, lens, rng, 40):
        o, n = int(arena.off_host[c]), int(new_len[c])
        kl = kept_dev[o:o + n]
        assert bool((kl[1:] > kl[:-1]).all()) and kl[:w.sink].tolist() == list(range(w.sink))
        assert int(kl[-1]) == int(lens[c]) - 1
    # attention after eviction still matches the oracle on the moved rows
    arena.decode_attn(0, w.L, q, out_stack)
    torch.cuda.synchronize()
    H.check_decode_against_oracle(arena, w, post, q64, out_stack.cpu().numpy().astype(np.float64), caches=picks)
    arena.close()
    del arena
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["llama32", "qwen"])
def test_tracked_decode_loop_at_full_size(name):
    """The decode loop as bench.py times it (one fused launch per layer, attention weights accumulated
    per row, eviction every 64 steps) at full size for 65 steps.  Steps 1, 64 and 65 are checked
    step-locally on sampled caches; between steps 1 and 63 nothing is flushed, so the scores grow
    through the attention kernel's deferred updates alone, and at step 63 they must match an oracle that
    ran the same 62 steps on its own; the eviction after step 64 is compared bit for bit on the sampled
    caches and on hundreds of short ones."""
    H = _h()
    w = synth.WORKLOADS[name]
    rng = np.random.Generator(np.random.PCG64(w.seed + 23))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    gen = synth.fill_arena_on_device(arena, w)          # K, V ~ N(0,1), scores U(0,1), pos = row index
    cpl = w.batch * w.Hkv
    bud_of = np.array([budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)], dtype=np.int32)
    arena.set_lengths(bud_of)
    dev = arena.device
    picks = sample_caches(arena, bud_of, rng, n_random=6)
    order = np.argsort(bud_of)
    runners = sorted({int(order[0]), int(order[-1]), int(order[len(order) // 2])} | {int(x) for x in rng.integers(0, arena.n_caches, 4)})
    shape_q, shape_kv = (w.L, w.batch, w.Hq, w.D), (w.L, w.batch, w.Hkv, w.D)
    out = torch.zeros(shape_q, dtype=torch.float32, device=dev)
    free = {}                                           # cache -> oracle cache that runs steps 2..63 on its own
    for t in range(1, 66):
        q = torch.randn(shape_q, generator=gen, device=dev).to(torch.bfloat16)
        kn = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
        vn = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
        local = t in (1, 64, 65)
        pre = H.download(arena, w, sorted(set(picks) | set(runners))) if local else None
        if t == 64:
            for c in runners:                           # 62 steps of deferred updates against the oracle's own run
                oc = free[c]
                serr = np.abs(pre.score[c].astype(np.float64) - oc.score)
                assert pre.K[c].shape[0] == oc.n and np.array_equal(pre.pos[c], oc.pos)
                assert np.all((serr <= 2e-3) | (serr <= 2e-3 * np.abs(oc.score))), f"cache {c}: scores after 63 steps, {serr.max():.3e}"
            print(f"{name}, step 63: scores of {len(runners)} caches match the oracle's own 62-step run", flush=True)
        for l in range(w.L):
            arena.append_decode_attn(l, 1, kn[l], vn[l], w.ctx + t, q[l], out[l])
        torch.cuda.synchronize()
        q64 = synth.storage_to_f64(H.from_device_storage(q, "bf16"), "bf16")
        k64 = synth.storage_to_f64(H.from_device_storage(kn, "bf16"), "bf16")
        v64 = synth.storage_to_f64(H.from_device_storage(vn, "bf16"), "bf16")
        got = out.cpu().numpy().astype(np.float64)
        if local:
            post = H.download(arena, w, sorted(set(picks) | set(runners)))
            e = H.check_step_against_oracle(arena, w, pre, post, got, q64, k64, v64, w.ctx + t, t, picks)
            print(f"{name}, step {t}: {len(picks)} sampled caches, worst attention error {e[0]:.3e}, "
                  f"worst score error {e[1]:.3e}", flush=True)
            if t == 1:
                free = {c: H.oracle_cache(w, post, c) for c in runners}
        elif t <= 63:
            for c in runners:
                l, b, hs = H.q_rows_of_cache(w, c)
                ref, _, _ = O.decode_step(free[c], q64[l, b, hs], k64[l, b, c % w.Hkv], v64[l, b, c % w.Hkv], w.ctx + t, t,
                                          budget=0, sink=0, recent=0, interval=0, track_scores=True)
                err = float(np.max(np.abs(got[l, b, hs] - ref)))
                assert err <= H.ATTN_TOL, f"step {t} cache {c}: attention error {err:.3e}"
        if t == 64:
            lens = arena.lengths()
            many = sorted(set(picks) | set(short_caches(lens)))
            before = H.download(arena, w, many)
            kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
            arena.compact(0, w.L, kept_dev)
            torch.cuda.synchronize()
            check_evictions(H, arena, w, budgets, before, H.download(arena, w, many), kept_dev, many, lens)
            assert np.array_equal(arena.lengths(), bud_of) and np.array_equal(arena.len.cpu().numpy(), bud_of)
            print(f"{name}: eviction after step 64 bit-exact on {len(many)} caches", flush=True)
    arena.close()
    del arena
    torch.cuda.empty_cache()


def test_cache_longer_than_the_longest_work_item():
    """A cache of 2^22 + 299 live rows (2.1 GB of K and V): a work item never spans more than 2^22
    rows, so even a target of one item per launch cuts this cache in two.  Attention in three
    schedules (two items, one wave of items, the whole-model schedule), the score update over all
    rows and one eviction are checked against the oracle on the full cache; a second, small layer
    keeps the launch over layer 0 a layer-range launch."""
    H = _h()
    big = (1 << 22) + 100
    w = synth.shrink(synth.WORKLOADS["llama1"], name="maxrun", L=2, Hq=4, Hkv=1, batch=1, seed=91, sink=4, recent=64,
                     slack=200)
    budgets = [big, 100]
    arena = H.make_arena(w, budgets, track=True)
    dev = arena.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    n0 = [big + 199, 250]                                  # one append still fits
    for c in range(2):
        o, n = int(arena.off_host[c]), n0[c]
        for a in range(0, n, 1 << 20):                     # in pieces: the fp32 draw of a piece stays small
            e = min(n, a + (1 << 20))
            arena.k[o + a:o + e].copy_(torch.randn((e - a, w.D), generator=gen, device=dev).to(torch.bfloat16))
            arena.v[o + a:o + e].copy_(torch.randn((e - a, w.D), generator=gen, device=dev).to(torch.bfloat16))
        arena.score[o:o + n].copy_(torch.rand((n,), generator=gen, device=dev))
        arena.pos[o:o + n].copy_(torch.arange(n, dtype=torch.int32, device=dev))
    arena.set_lengths(np.asarray(n0, dtype=np.int32))
    q = torch.randn((2, 1, w.Hq, w.D), generator=gen, device=dev).to(torch.bfloat16)
    q64 = synth.storage_to_f64(H.from_device_storage(q, "bf16"), "bf16")
    pre = H.download(arena, w)
    K64 = [synth.storage_to_f64(pre.K[c], "bf16") for c in range(2)]
    V64 = [synth.storage_to_f64(pre.V[c], "bf16") for c in range(2)]
    ref = [O.decode_attn(q64[c, 0], K64[c], V64[c])[0] for c in range(2)]
    print("maxrun: oracle attention over the stored caches done", flush=True)

    def decode(layer_begin, layer_count):
        out = torch.full((layer_count, 1, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
        arena.decode_attn(layer_begin, layer_count, q[layer_begin:layer_begin + layer_count], out)
        torch.cuda.synchronize()
        return out.cpu().numpy().astype(np.float64)

    # layer-range launch, default target (one wave of work items) and a target of one item (run clamped to 2^22 rows)
    for target in (None, 1):
        if target is not None:
            arena.set_option(B.OPT_TARGET_ITEMS, target)
            arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
        o0 = decode(0, 1)
        err = float(np.max(np.abs(o0[0, 0] - ref[0])))
        assert err <= H.ATTN_TOL, f"layer-range launch, target {target}: {err:.3e}"
        ow = decode(0, 2)
        for c in range(2):
            err = float(np.max(np.abs(ow[c, 0] - ref[c])))
            assert err <= H.ATTN_TOL, f"whole-model launch, target {target}, cache {c}: {err:.3e}"
    n_items = B.plan_schedule(arena.off_host, arena.cap_host, 2, 1, 512, False, target_items=1)
    runs = [it[2] for it in n_items if it[0] == 0]
    assert len(runs) == 2 and max(runs) <= 1 << 22 and sum(runs) == big + 200   # the clamp: two runs, not one

    # one fused step (still two items): append, attention, score update over every row; the attention
    # calls above have added to the scores, so the step starts from the scores as they are now
    arena.flush_scores(0, 2)
    torch.cuda.synchronize()
    for c in range(2):
        o = int(arena.off_host[c])
        pre.score[c] = arena.score[o:o + n0[c]].cpu().numpy()
    knew = torch.randn((2, 1, 1, w.D), generator=gen, device=dev).to(torch.bfloat16)
    vnew = torch.randn((2, 1, 1, w.D), generator=gen, device=dev).to(torch.bfloat16)
    outd = torch.full((2, 1, w.Hq, w.D), float("nan"), dtype=torch.float32, device=dev)
    for l in range(2):
        arena.append_decode_attn(l, 1, knew[l], vnew[l], 777, q[l], outd[l])
    torch.cuda.synchronize()
    out = outd.cpu().numpy().astype(np.float64)
    post = H.download(arena, w)
    kn64 = synth.storage_to_f64(H.from_device_storage(knew, "bf16"), "bf16")
    vn64 = synth.storage_to_f64(H.from_device_storage(vnew, "bf16"), "bf16")
    for c in range(2):
        oc = O.Cache(w.D)
        oc.load(K64[c], V64[c], pre.score[c].astype(np.float64), pre.pos[c])
        r, _, _ = O.decode_step(oc, q64[c, 0], kn64[c, 0, 0], vn64[c, 0, 0], 777, 1, budget=0, sink=0, recent=0,
                                interval=0, track_scores=True)
        assert post.K[c].shape[0] == n0[c] + 1 and post.pos[c][-1] == 777
        assert float(np.max(np.abs(out[c, 0] - r))) <= H.ATTN_TOL
        serr = np.abs(post.score[c].astype(np.float64) - oc.score)
        assert np.all((serr <= 2e-3) | (serr <= 2e-3 * np.abs(oc.score))), f"cache {c}: scores"
    del K64, V64
    print("maxrun: fused step checked", flush=True)

    # eviction of the 200 + 151 rows above the budgets, lists and moved rows bit-exact
    kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev)
    arena.compact(0, 2, kept_dev)
    torch.cuda.synchronize()
    after = H.download(arena, w)
    for c in range(2):
        kept = O.compact_select(post.score[c], post.K[c].shape[0], budgets[c], w.sink, w.recent)
        o = int(arena.off_host[c])
        assert np.array_equal(kept_dev[o:o + len(kept)].cpu().numpy(), np.asarray(kept, dtype=np.int32)), f"cache {c}"
        assert after.K[c].shape[0] == budgets[c]
        idx = np.asarray(kept)
        assert np.array_equal(after.K[c], post.K[c][idx]) and np.array_equal(after.V[c], post.V[c][idx])
        assert np.array_equal(after.score[c].view(np.uint32), post.score[c][idx].view(np.uint32))
        assert np.array_equal(after.pos[c], post.pos[c][idx])
    assert arena.lengths().tolist() == budgets
    arena.close()


def test_long_workload_trajectory_at_full_size():
    """The long workload as bench.py runs it (1024 caches of up to 131072 rows, one fused launch per
    layer, scores from the kernel, eviction every 32 steps), all 256 steps at full size; steps 1, 32,
    33 and 256 are checked step-locally on sampled caches (the longest and the shortest among them),
    the evictions after steps 32 and 256 bit for bit on the same caches; lengths on all caches."""
    H = _h()
    w = synth.WORKLOADS["long"]
    rng = np.random.Generator(np.random.PCG64(w.seed + 11))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets, track=True)
    gen = synth.fill_arena_on_device(arena, w)
    cpl = w.batch * w.Hkv
    bud_of = np.array([budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)], dtype=np.int32)
    arena.set_lengths(bud_of)
    arena.score.zero_()
    dev = arena.device
    picks = sample_caches(arena, bud_of, rng, n_random=6)
    checked = (1, 32, 33, 256)
    shape_q, shape_kv = (w.L, w.batch, w.Hq, w.D), (w.L, w.batch, w.Hkv, w.D)
    out = torch.zeros(shape_q, dtype=torch.float32, device=dev)
    for t in range(1, w.steps + 1):
        q = torch.randn(shape_q, generator=gen, device=dev).to(torch.bfloat16)
        kn = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
        vn = torch.randn(shape_kv, generator=gen, device=dev).to(torch.bfloat16)
        pre = H.download(arena, w, picks) if t in checked else None
        for l in range(w.L):
            arena.append_decode_attn(l, 1, kn[l], vn[l], w.ctx + t, q[l], out[l])
        post = None
        if t in checked:
            post = H.download(arena, w, picks)
            q64 = synth.storage_to_f64(H.from_device_storage(q, "bf16"), "bf16")
            e = H.check_step_against_oracle(arena, w, pre, post, out.cpu().numpy().astype(np.float64), q64,
                                            synth.storage_to_f64(H.from_device_storage(kn, "bf16"), "bf16"),
                                            synth.storage_to_f64(H.from_device_storage(vn, "bf16"), "bf16"),
                                            w.ctx + t, t, picks)
            print(f"long, step {t}: {len(picks)} sampled caches, worst attention error {e[0]:.3e}, "
                  f"worst score error {e[1]:.3e}", flush=True)
        if t % w.interval == 0:
            kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=dev) if post is not None else None
            arena.compact(0, w.L, kept_dev)
            if post is not None:
                torch.cuda.synchronize()
                H.check_eviction_against_oracle(arena, w, budgets, post, H.download(arena, w, picks), kept_dev, picks)
            assert np.array_equal(arena.lengths(), bud_of)
        else:
            assert np.array_equal(arena.lengths(), bud_of + t % w.interval)
    torch.cuda.synchronize()
    assert np.array_equal(arena.len.cpu().numpy(), bud_of)
    assert bool(torch.isfinite(arena.score).all())
    arena.close()
    del arena
    torch.cuda.empty_cache()
