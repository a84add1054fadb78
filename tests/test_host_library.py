"""CPU-side checks of libbaklava: it loads, exports what the header declares, and its host
allocators agree bit-for-bit with the oracle and with the stored budgets."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "baklava.h")).read()
    declared = set(re.findall(r"\b(baklava_[a-z_]+)\s*\(", header))
    declared -= {"baklava_ctx", "baklava_desc"}
    assert declared == set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror():
    assert B.strerror(B.OK) == "ok"
    assert "capacity" in B.strerror(B.ECAPACITY)
    assert B.strerror(99) == "unknown status"


@pytest.mark.parametrize("name", ["llama1", "llama32", "qwen", "long"])
def test_proportional_budgets_match_oracle_and_golden(name):
    w = synth.WORKLOADS[name]
    mine = synth.budgets_for(w, B.alloc_proportional)
    assert mine == synth.budgets_for(w, O.alloc_proportional)
    golden = [int(x) for x in open(os.path.join(ROOT, "tests", "golden", f"budgets_{name}.txt"))
              if not x.startswith("#")]
    assert mine == golden


@pytest.mark.parametrize("seed", range(40))
def test_proportional_random_vs_oracle(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 300))
    imp = rng.lognormal(0, 2.0, m) if seed % 2 else 1 + rng.pareto(1.1, m)
    if seed % 5 == 0:
        imp = np.round(imp, 1) + 0.1          # many exact ties
    lo = int(rng.integers(0, 200))
    hi = lo + int(rng.integers(0, 100000))
    Bt = int(rng.integers(m * lo, m * hi + 1))
    assert B.alloc_proportional(imp, Bt, lo, hi) == O.alloc_proportional(imp, Bt, lo, hi)


def test_proportional_error_codes():
    def status(imp, Bt, lo, hi):
        with pytest.raises(B.BaklavaError) as e:
            B.alloc_proportional(imp, Bt, lo, hi)
        return e.value.status
    assert status([1.0, 1.0], 5, 3, 10) == B.EINFEASIBLE
    assert status([1.0, 1.0], 25, 3, 10) == B.EINFEASIBLE
    assert status([1.0, 0.0], 10, 3, 10) == B.EINVAL
    assert status([1.0, float("inf")], 10, 3, 10) == B.EINVAL
    assert status([1.0, 1.0], 10, 5, 3) == B.EINVAL


@pytest.mark.parametrize("seed", range(30))
def test_threshold_random_vs_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    m = int(rng.integers(1, 200))
    imp = np.round(rng.random(m), 2) if seed % 3 == 0 else rng.random(m)
    size = rng.integers(0, 40000, m)
    t, r = float(rng.random()), float(rng.random())
    assert B.alloc_threshold(imp, size, t, r) == O.alloc_threshold(imp, size, t, r)


def test_threshold_error_codes():
    with pytest.raises(B.BaklavaError) as e:
        B.alloc_threshold([0.1, 0.9], [10, 10], 0.5, 1.5)
    assert e.value.status == B.EINVAL
    # Algorithm 2 orders importances and compares them with t: a NaN or an infinity has no place there,
    # on either side
    for imp, t in (([0.1, float("nan"), 0.9], 0.5), ([0.1, float("inf"), 0.9], 0.5), ([0.1, 0.9], float("nan"))):
        with pytest.raises(B.BaklavaError) as e:
            B.alloc_threshold(imp, [10] * len(imp), t, 0.5)
        assert e.value.status == B.EINVAL
        with pytest.raises(ValueError):
            O.alloc_threshold(imp, [10] * len(imp), t, 0.5)
    with pytest.raises(B.BaklavaError) as e:
        B.alloc_two_level([1.0, 2.0], [[0.2, float("nan")], [0.5, 0.6]], 400, 10, 400, 0.5, 0.5)
    assert e.value.status == B.EINVAL


def test_create_refuses_an_arena_that_is_not_packed():
    """The offsets must be the packed prefix sums of the capacities (what baklava_layout writes): the
    check comes before anything touches a device, so it runs without one."""
    w = synth.WORKLOADS["tiny"]
    b = np.asarray([64, 192], dtype=np.int32)
    off, cap, total = B.layout(b, w.L, w.Hkv, w.batch, w.slack)
    d = B.Desc()
    d.L, d.Hq, d.Hkv, d.D, d.batch, d.dtype = w.L, w.Hq, w.Hkv, w.D, w.batch, B.F32
    d.sink, d.recent = w.sink, w.recent
    fake = 0x1000                                         # never dereferenced: the call fails on the offsets
    d.k = d.v = d.score = d.pos = d.off = d.cap = d.len = d.budget = d.workspace = fake
    d.workspace_bytes = 1 << 30
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    for bad in (off + np.array([0, 16]), off[::-1].copy(), off + 8):
        bad = np.ascontiguousarray(bad, dtype=np.int64)
        ctx = C.c_void_p()
        st = B.lib().baklava_create(C.byref(d), bad.ctypes.data_as(i64p), cap.ctypes.data_as(i32p), None,
                                    b.ctypes.data_as(i32p), C.byref(ctx))
        assert st == B.EINVAL and not ctx.value


@pytest.mark.parametrize("name", ["tiny", "llama1", "qwen"])
def test_layout_matches_oracle(name):
    w = synth.WORKLOADS[name]
    b = synth.budgets_for(w, O.alloc_proportional)
    off, cap, total = B.layout(b, w.L, w.Hkv, w.batch, w.slack)
    ooff, ocap, ototal = O.layout(b, w.L, w.Hkv, w.batch, w.slack)
    assert off.tolist() == ooff and cap.tolist() == ocap and total == ototal


def test_workspace_bytes_is_a_pure_host_query():
    w = synth.WORKLOADS["llama1"]
    b = synth.budgets_for(w, B.alloc_proportional)
    _, cap, total = B.layout(b, w.L, w.Hkv, w.batch, w.slack)
    d = B.Desc()
    d.L, d.Hq, d.Hkv, d.D, d.batch, d.dtype = w.L, w.Hq, w.Hkv, w.D, w.batch, B.BF16
    d.sink, d.recent = w.sink, w.recent
    i32p = C.POINTER(C.c_int32)
    bud = np.ascontiguousarray(b, dtype=np.int32)
    n0 = B.lib().baklava_workspace_bytes(C.byref(d), cap.ctypes.data_as(i32p), bud.ctypes.data_as(i32p))
    d.track_scores = 1
    n1 = B.lib().baklava_workspace_bytes(C.byref(d), cap.ctypes.data_as(i32p), bud.ctypes.data_as(i32p))
    # score tracking adds, per cache, 32 packed query rows and (max, 1/sum) pairs of its pending calls
    n_caches = w.L * w.batch * w.Hkv
    lag_q, lag_ml = n_caches * 32 * w.D * 2, n_caches * 32 * 2 * 4
    assert n0 > 0 and n1 == n0 + ((lag_q + 255) // 256) * 256 + ((lag_ml + 255) // 256) * 256
    d.D = 96
    assert B.lib().baklava_workspace_bytes(C.byref(d), cap.ctypes.data_as(i32p), bud.ctypes.data_as(i32p)) == 0


@pytest.mark.parametrize("name,chunk", [("llama32", 512), ("llama32", 2048), ("qwen", 768), ("long", 4096), ("tiny", 256)])
@pytest.mark.parametrize("whole", [False, True])
@pytest.mark.parametrize("target", [0, 768])
def test_split_k_schedule_covers_every_row_once(name, chunk, whole, target):
    w = synth.WORKLOADS[name]
    b = synth.budgets_for(w, B.alloc_proportional)
    off, cap, total = B.layout(b, w.L, w.Hkv, w.batch, w.slack)
    cpl = w.batch * w.Hkv
    items = B.plan_schedule(off, cap, w.L, cpl, chunk, whole, target_items=target)
    n_caches = w.L * cpl
    units = [range(n_caches)] if whole else [range(l * cpl, (l + 1) * cpl) for l in range(w.L)]
    first = {it[0]: it for it in items if it[1] == 0}
    run_of = {}                                                 # run length of each cache
    for u in units:
        at_chunk = sum(max(1, -(-int(cap[c]) // chunk)) for c in u)
        goal = max(target, len(u))                              # a unit has at least one item per cache
        n_u = sum(first[c][4] for c in u)
        if not target or at_chunk <= goal:
            assert n_u == at_chunk                              # few enough items already: unchanged
            for c in u:
                run_of[c] = chunk
            continue
        assert n_u <= goal
        best = chunk                                            # shortest common run that meets the goal
        while sum(max(1, -(-int(cap[c]) // best)) for c in u) > goal:
            best += 64
        for c in u:
            _, _, count, _, nsplit, _ = first[c]
            if nsplit > 1:
                run_of[c] = count
                assert count == chunk or cap[c] > nsplit * (count - 64)   # runs as equal as 64-row steps allow
            else:
                run_of[c] = max(chunk, -(-int(cap[c]) // 64) * 64)
            assert run_of[c] <= best
            assert nsplit <= max(1, -(-int(cap[c]) // best))    # balancing adds no item
    seen_rows = np.zeros(n_caches, dtype=np.int64)
    slots = set()
    first_slot = {}
    for (c, start, count, slot, nsplit, row0) in items:
        run = run_of[c]
        assert run % 64 == 0 and run >= chunk
        assert 0 <= count <= run and start % run == 0 and start + count <= cap[c]
        assert row0 == off[c] + start
        assert nsplit == max(1, -(-int(cap[c]) // run))
        assert slot not in slots
        slots.add(slot)
        seen_rows[c] += count
        first_slot.setdefault(c, slot - start // run)
        assert slot == first_slot[c] + start // run            # a cache's slots are consecutive
    assert slots == set(range(len(items)))                      # slots are a permutation of 0..n-1
    assert np.array_equal(seen_rows, cap.astype(np.int64))     # every row of every cache exactly once
    # slots are numbered cache by cache
    assert [first_slot[c] for c in range(n_caches)] == sorted(first_slot[c] for c in range(n_caches))
    caches_in_order = [it[0] for it in items if it[1] == 0]
    if whole:
        caps = [int(cap[c]) for c in caches_in_order]
        assert caps == sorted(caps, reverse=True)               # long caches first over the whole model
    else:
        for l in range(w.L):                                    # a layer is a contiguous slice, long first
            sl = caches_in_order[l * cpl:(l + 1) * cpl]
            assert sorted(sl) == list(range(l * cpl, (l + 1) * cpl))
            caps = [int(cap[c]) for c in sl]
            assert caps == sorted(caps, reverse=True)
            lo = min(it[3] for it in items if it[0] in sl)
            n_l = sum(1 for it in items if it[0] in set(sl))
            pos = [i for i, it in enumerate(items) if it[0] in set(sl)]
            assert pos == list(range(lo, lo + n_l))             # launch positions == slot range of the layer


def test_split_k_schedule_errors():
    off, cap, _ = B.layout([300, 5000], 1, 2, 1, 0)
    for bad_chunk in (0, 100, 255, 300, (1 << 22) + 64):
        with pytest.raises(B.BaklavaError) as e:
            B.plan_schedule(off, cap, 1, 2, bad_chunk, False)
        assert e.value.status == B.EINVAL
    assert len(B.plan_schedule(off, cap, 1, 2, 256, False)) == 2 + 20
    with pytest.raises(B.BaklavaError) as e:
        B.plan_schedule(off, cap, 1, 2, 256, False, max_items=5)
    assert e.value.status == B.ECAPACITY


def test_kv_importance_matches_oracle():
    rng = np.random.default_rng(77)
    for L, Hq, Hkv in ((1, 4, 2), (32, 32, 8), (28, 28, 4), (3, 5, 5)):
        s = rng.uniform(-1, 1, (L, Hq))
        got = B.kv_importance(s, L, Hq, Hkv)
        assert got.shape == (L, Hkv)
        assert np.allclose(got, O.kv_importance(s, Hq // Hkv), rtol=0, atol=1e-15)
    assert B.kv_importance([[1.0, 0.0, -1.0, 0.5]], 1, 4, 2).tolist() == [[0.25, 0.625]]
    for bad in ([[2.0, 0.0]], [[float("nan"), 0.0]]):
        with pytest.raises(B.BaklavaError) as e:
            B.kv_importance(bad, 1, 2, 1)
        assert e.value.status == B.EINVAL
    with pytest.raises(B.BaklavaError) as e:
        B.kv_importance([[0.0, 0.0, 0.0]], 1, 3, 2)
    assert e.value.status == B.EINVAL


def test_profile_workspace_bytes():
    assert B.profile_workspace_bytes(1, 4, 128) == 256
    assert B.profile_workspace_bytes(2, 32, 8192) == 2 * 32 * 64 * 4
    assert B.profile_workspace_bytes(0, 4, 128) == 0


@pytest.mark.parametrize("seed", range(12))
def test_two_level_allocation_matches_oracle(seed):
    rng = np.random.default_rng(500 + seed)
    L, Hkv = int(rng.integers(1, 40)), int(rng.integers(1, 9))
    limp = rng.uniform(0.01, 1.0, L)
    himp = np.round(rng.uniform(0.0, 1.0, (L, Hkv)), 2) if seed % 3 == 0 else rng.uniform(0.0, 1.0, (L, Hkv))
    lo, hi = 64, 40000
    Bt = int(rng.integers(L * Hkv * lo, L * Hkv * hi + 1))
    t, r = float(rng.random()), float(rng.random())
    got = B.alloc_two_level(limp, himp, Bt, lo, hi, t, r)
    assert got == O.alloc_two_level(limp, himp, Bt, lo, hi, t, r)
    assert sum(got) == Bt


def test_two_level_allocation_errors():
    with pytest.raises(B.BaklavaError) as e:
        B.alloc_two_level([1.0, 1.0], [[0.5, 0.5], [0.5, 0.5]], 10, 64, 100, 0.5, 0.5)      # below L*Hkv*lo
    assert e.value.status == B.EINFEASIBLE
    with pytest.raises(B.BaklavaError) as e:
        B.alloc_two_level([1.0, 1.0], [[0.5, 0.5], [0.5, 0.5]], 400, 64, 200, 0.5, 1.5)
    assert e.value.status == B.EINVAL


def test_schedule_runs_never_exceed_the_row_limit():
    """One enormous cache and a target of one item: the run stops at 2^22 rows."""
    cap = np.array([(1 << 24) + 100, 300], dtype=np.int32)
    off = np.array([0, (1 << 24) + 100], dtype=np.int64)
    items = B.plan_schedule(off, cap, 1, 2, 256, False, target_items=1)
    big = [it for it in items if it[0] == 0]
    assert len(big) == 5 and max(it[2] for it in big) <= 1 << 22          # ceil(cap / 2^22) runs, made equal
    assert sum(it[2] for it in big) == cap[0] and big[0][2] == (-(-int(cap[0]) // 5) + 63) // 64 * 64


def test_hand_worked_allocation_examples_through_the_library():
    """The hand-worked examples that pin the oracle, asked of the C library directly."""
    assert B.alloc_proportional([7, 4, 8, 5], 24, 1, 7) == [7, 4, 7, 6]
    assert B.alloc_threshold([0.2, 0.5, 0.5, 0.9], [100] * 4, 0.5, 0.5) == [50, 100, 100, 150]
    assert B.alloc_threshold([0.1, 0.9, 0.9], [100, 100, 100], 0.5, 0.5) == [50, 150, 100]
    got = B.alloc_two_level([1.0, 1000.0], np.array([[0.4, 0.4, 0.4], [0.3, 0.9, 0.5]]), 332, 10, 1000, 0.0, 0.5)
    assert got == [10, 10, 10, 100, 101, 101]
    rng = np.random.Generator(np.random.PCG64(7))
    for _ in range(500):                                        # small cases where clipping and leftovers dominate
        m = int(rng.integers(2, 6))
        imp = [float(v) for v in rng.integers(1, 9, size=m)]
        lo = int(rng.integers(0, 4))
        hi = int(rng.integers(lo + 1, 13))
        Bt = int(rng.integers(m * lo, m * hi + 1))
        assert B.alloc_proportional(imp, Bt, lo, hi) == O.alloc_proportional(imp, Bt, lo, hi)
