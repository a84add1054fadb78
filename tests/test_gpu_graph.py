"""The attention entry points only enqueue kernels, so a decode step can be captured into a HIP graph
and replayed: every replay is checked against the eager result and the oracle."""
import numpy as np
import pytest
import torch

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
