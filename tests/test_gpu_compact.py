"""GPU parity: baklava_compact against the oracle's eviction -- kept-index lists and lengths
bit-exact, moved K/V/score/pos rows bit-identical to the rows they came from."""
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


def run_compact_and_check(arena, w, st, policy=B.POLICY_SCORE, layer_begin=0, layer_count=None, want_lists=True):
    H = _h()
    layer_count = w.L if layer_count is None else layer_count
    kept_dev = torch.full((arena.total_tokens,), -1, dtype=torch.int32, device=arena.device) if want_lists else None
    arena.compact(layer_begin, layer_count, kept_dev)
    torch.cuda.synchronize()
    after = H.download(arena, w)
    dev_len = arena.len.cpu().numpy()
    host_len = arena.lengths()
    cpl = w.batch * w.Hkv
    for c in range(arena.n_caches):
        n = st.K[c].shape[0]
        in_range = layer_begin * cpl <= c < (layer_begin + layer_count) * cpl
        if not in_range:
            assert dev_len[c] == n and host_len[c] == n
            assert np.array_equal(after.K[c], st.K[c]) and np.array_equal(after.V[c], st.V[c])
            continue
        b = int(arena.budget_host[(c // cpl) * w.Hkv + c % w.Hkv])
        recent = w.recent
        kept = O.compact_select(st.score[c], n, b, w.sink, recent, policy)
        assert dev_len[c] == len(kept) == min(n, b), f"cache {c}"
        assert host_len[c] == len(kept)
        if want_lists:
            o = int(arena.off_host[c])
            got = kept_dev[o:o + len(kept)].cpu().numpy()
            assert np.array_equal(got, np.asarray(kept, dtype=np.int32)), f"cache {c}: kept list differs"
        # rows moved bit-exactly
        assert np.array_equal(after.K[c], st.K[c][kept]), f"cache {c}: K rows"
        assert np.array_equal(after.V[c], st.V[c][kept]), f"cache {c}: V rows"
        assert np.array_equal(after.score[c].view(np.uint32), st.score[c][kept].view(np.uint32))
        assert np.array_equal(after.pos[c], st.pos[c][kept])
    return after


def test_tiny_workload_decode_compact_decode():
    """One decode over the full 256-row caches, eviction to budgets {64, 192} from U(0,1) scores,
    one decode over the compacted caches: all three results against the oracle."""
    H = _h()
    w = synth.WORKLOADS["tiny"]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    arena = H.make_arena(w)
    st = H.fill_from_host(arena, w, [w.ctx] * arena.n_caches, rng, scores="uniform")
    q, q64 = H.make_q(w, rng, w.L)
    H.check_decode_against_oracle(arena, w, st, q64, H.gpu_decode(arena, w, q))
    after = run_compact_and_check(arena, w, st)
    assert arena.lengths().tolist() == [64, 192]
    q2, q264 = H.make_q(w, rng, w.L)
    H.check_decode_against_oracle(arena, w, after, q264, H.gpu_decode(arena, w, q2))
    # a second compaction changes nothing
    again = run_compact_and_check(arena, w, after)
    for c in range(arena.n_caches):
        assert np.array_equal(again.K[c], after.K[c])
    arena.close()


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
def test_ragged_compaction_all_row_sizes(dtype, D):
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="cmp", L=3, Hq=8, Hkv=4, D=D, batch=2, dtype=dtype,
                     seed=21, sink=4, recent=16, slack=700)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [20, 21, 100, 128, 129, 300, 511, 512, 513, 1000, 33, 64]
    arena = H.make_arena(w, budgets)
    cpl = w.batch * w.Hkv
    lens = []
    for c in range(arena.n_caches):
        b = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
        extra = [0, 1, 64, 700, 127, 129, 333, -5][c % 8]      # at, just over, far over and under budget
        lens.append(max(1, b + extra))
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    after = run_compact_and_check(arena, w, st, layer_begin=1, layer_count=1)      # one layer only
    after = run_compact_and_check(arena, w, after)                                 # then everything
    arena.close()


def test_ties_zero_scores_and_signed_zero():
    """All-equal scores (ties everywhere), coarse scores with many ties, and -0.0 vs +0.0."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="ties", L=1, Hq=6, Hkv=3, batch=1, seed=22, sink=2,
                     recent=3, slack=3000)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [40, 700, 1500]
    arena = H.make_arena(w, budgets)
    lens = [900, 2600, 4400]
    st = H.fill_from_host(arena, w, lens, rng, scores="zero")
    # cache 0: all zero; cache 1: coarse grid; cache 2: zeros of both signs plus a few values
    s1 = (rng.integers(0, 5, lens[1]) / 4).astype(np.float32)
    s2 = np.where(rng.random(lens[2]) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
    s2[rng.integers(0, lens[2], 50)] = rng.random(50).astype(np.float32)
    s2[rng.integers(0, lens[2], 20)] = -rng.random(20).astype(np.float32)
    for c, s in ((1, s1), (2, s2)):
        o = int(arena.off_host[c])
        arena.score[o:o + lens[c]].copy_(torch.from_numpy(s).to(arena.device))
        st.score[c] = s
    run_compact_and_check(arena, w, st)
    arena.close()


def test_streaming_policy():
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="stream", L=2, Hq=4, Hkv=2, batch=2, seed=23, sink=4,
                     recent=0, slack=500)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [100, 257, 64, 4]
    arena = H.make_arena(w, budgets, policy=B.POLICY_STREAMING)
    cpl = w.batch * w.Hkv
    lens = [budgets[(c // cpl) * w.Hkv + c % w.Hkv] + (c * 37) % 400 for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    after = run_compact_and_check(arena, w, st, policy=B.POLICY_STREAMING)
    for c in range(arena.n_caches):
        b = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
        if lens[c] > b:
            expect = list(range(min(4, b))) + list(range(lens[c] - (b - 4), lens[c]))
            assert after.pos[c].tolist() == expect
    arena.close()


def test_budget_equal_sink_plus_recent_keeps_no_middle_row():
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="edge", L=1, Hq=2, Hkv=1, batch=1, seed=24, sink=4,
                     recent=16, slack=100)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    arena = H.make_arena(w, [20])
    st = H.fill_from_host(arena, w, [120], rng, scores="uniform")
    after = run_compact_and_check(arena, w, st)
    assert after.pos[0].tolist() == [0, 1, 2, 3] + list(range(104, 120))
    arena.close()


def test_infeasible_budget_is_refused_at_creation():
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="bad", L=1, Hq=2, Hkv=1, batch=1, sink=4, recent=16)
    with pytest.raises(B.BaklavaError) as e:
        H.make_arena(w, [19])
    assert e.value.status == B.EINFEASIBLE


@pytest.mark.parametrize("slack", [1, 64, 700])
def test_long_caches_move_in_several_segments(slack):
    """Budgets around and above the move's segment size (4096 rows): rows whose source lies in the
    next segment travel through the halo copy."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="segs", L=1, Hq=8, Hkv=4, batch=2, seed=25, sink=4,
                     recent=16, slack=slack)
    rng = np.random.Generator(np.random.PCG64(w.seed + slack))
    budgets = [4095, 4096, 4097, 13000]
    arena = H.make_arena(w, budgets)
    lens = [b + slack for b in budgets] + [b + max(1, slack // 2) for b in budgets]
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    after = run_compact_and_check(arena, w, st)
    # evictions concentrated at the very front: every later row shifts by the full amount
    st2 = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    for c in range(arena.n_caches):
        s = np.ones(lens[c], dtype=np.float32)
        s[4:4 + 2 * slack] = 0.0
        o = int(arena.off_host[c])
        arena.score[o:o + lens[c]].copy_(torch.from_numpy(s).to(arena.device))
        st2.score[c] = s
    run_compact_and_check(arena, w, st2)
    arena.close()


@pytest.mark.parametrize("policy", [B.POLICY_SCORE, B.POLICY_STREAMING])
@pytest.mark.parametrize("scores", ["uniform", "equal", "coarse", "signed_zero"])
def test_caches_selected_tile_by_tile(scores, policy):
    """Caches beyond 8192 rows of capacity are ranked by several workgroups (tiles of 8192 rows, one
    kernel per radix pass): lengths at, just over and far over the budget, live lengths that end
    inside the first, a middle and the last tile, ties that span tiles (the older row must win across
    a tile boundary), short caches in the same launch, a launch over one layer only."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama32"], name="tiles", L=2, Hq=4, Hkv=4, batch=1, seed=26, sink=4,
                     recent=16, slack=300)
    rng = np.random.Generator(np.random.PCG64(w.seed + policy))
    budgets = [8100, 8192, 8193, 20, 16300, 16384, 24581, 500]
    extra = [300, 1, 150, 77, 0, 300, 299, 37]
    arena = H.make_arena(w, budgets, policy=policy)
    arena.set_option(B.OPT_TILED_SELECT_ROWS, 8192)       # the smallest threshold: six of the eight caches are tiled
    assert sum(1 for c in arena.cap_host if c > 8192) == 6
    lens = [b + e for b, e in zip(budgets, extra)]
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    if scores != "uniform":
        for c in range(arena.n_caches):
            n = lens[c]
            if scores == "equal":
                s = np.full(n, 0.25, dtype=np.float32)
            elif scores == "coarse":
                s = (rng.integers(0, 7, n) / 8).astype(np.float32)
            else:
                s = np.where(rng.random(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
                s[rng.integers(0, n, 40)] = rng.random(40).astype(np.float32)
                s[rng.integers(0, n, 40)] = -rng.random(40).astype(np.float32)
            o = int(arena.off_host[c])
            arena.score[o:o + n].copy_(torch.from_numpy(s).to(arena.device))
            st.score[c] = s
    after = run_compact_and_check(arena, w, st, policy=policy, layer_begin=1, layer_count=1)   # tiles of layer 1 only
    after = run_compact_and_check(arena, w, after, policy=policy)                              # then both layers
    run_compact_and_check(arena, w, after, policy=policy)                                      # nothing left to evict
    arena.close()


@pytest.mark.parametrize("seed", list(range(500, 512)))
def test_seeded_random_evictions(seed):
    """Random cache sizes on both sides of the threshold for tile-by-tile selection, random budgets, sink
    and recent windows, live lengths and score distributions (continuous, few distinct values, all equal,
    signed zeros, negative values), both policies, a random layer range first and all layers after it."""
    H = _h()
    r = np.random.Generator(np.random.PCG64(seed))
    policy = B.POLICY_STREAMING if seed % 4 == 0 else B.POLICY_SCORE
    L, Hkv, batch = int(r.integers(1, 4)), int(r.integers(1, 4)), int(r.integers(1, 3))
    sink = int(r.integers(0, 6))
    recent = 0 if policy == B.POLICY_STREAMING else int(r.integers(0, 40))
    slack = int(r.choice([1, 50, 700, 9000]))
    w = synth.shrink(synth.WORKLOADS["tiny"], name=f"evict{seed}", L=L, Hq=Hkv, Hkv=Hkv, batch=batch, seed=seed,
                     sink=sink, recent=recent, slack=slack)
    budgets = [int(max(sink + recent + 1, round(float(np.exp(r.uniform(np.log(16), np.log(30000))))))) for _ in range(L * Hkv)]
    arena = H.make_arena(w, budgets, policy=policy)
    threshold = int(r.choice([8192, 12000, 36864]))
    arena.set_option(B.OPT_TILED_SELECT_ROWS, threshold)
    cap = arena.cap_host
    lens = [int(cap[c]) if r.random() < 0.3 else int(r.integers(0, int(cap[c]) + 1)) for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, r, scores="uniform")
    kind = str(r.choice(["uniform", "coarse", "equal", "signed_zero", "negative"]))
    print(f"seed {seed}: policy={policy} L={L} Hkv={Hkv} batch={batch} sink={sink} recent={recent} slack={slack} "
          f"threshold={threshold} scores={kind} budgets={budgets}", flush=True)
    if kind != "uniform":
        for c in range(arena.n_caches):
            n = lens[c]
            if n == 0:
                continue
            if kind == "equal":
                s = np.full(n, 0.25, dtype=np.float32)
            elif kind == "coarse":
                s = (r.integers(0, 5, n) / 4).astype(np.float32)
            elif kind == "negative":
                s = (r.random(n) * 2 - 1).astype(np.float32)
            else:
                s = np.where(r.random(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
                s[r.integers(0, n, 8)] = r.random(8).astype(np.float32)
            o = int(arena.off_host[c])
            arena.score[o:o + n].copy_(torch.from_numpy(s).to(arena.device))
            st.score[c] = s
    lb = int(r.integers(0, L))
    lc = int(r.integers(1, L - lb + 1))
    after = run_compact_and_check(arena, w, st, policy=policy, layer_begin=lb, layer_count=lc)
    after = run_compact_and_check(arena, w, after, policy=policy)
    run_compact_and_check(arena, w, after, policy=policy, want_lists=False)
    arena.close()
