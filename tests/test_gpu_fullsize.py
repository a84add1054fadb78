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
    pre = H.download(arena, w, picks)
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
    post = H.download(arena, w, picks)
    for c in picks:
        b = budgets[(c // cpl) * w.Hkv + c % w.Hkv]
        kept = O.compact_select(pre.score[c], int(lens[c]), b, w.sink, w.recent)
        o = int(arena.off_host[c])
        got = kept_dev[o:o + len(kept)].cpu().numpy()
        assert np.array_equal(got, np.asarray(kept, dtype=np.int32)), f"cache {c}: kept list"
        assert np.array_equal(post.K[c], pre.K[c][kept]) and np.array_equal(post.V[c], pre.V[c][kept])
        assert np.array_equal(post.score[c], pre.score[c][kept]) and np.array_equal(post.pos[c], pre.pos[c][kept])
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
