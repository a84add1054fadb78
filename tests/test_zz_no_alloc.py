"""baklava_layer_similarity_static (partial sums in a fixed device array, nothing allocated) against
baklava_layer_similarity (caller's workspace): the same kernels, so the results must be identical,
bit for bit, on calls in a row that share the array, the later ones with smaller inputs."""
import numpy as np
import pytest
import torch

from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu


def _h():
    import gpu_harness
    return gpu_harness


def _pair(rng, shape, dev):
    H = _h()
    a = synth.payload(rng, shape, "bf16")
    b = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(a) + 0.5 * rng.standard_normal(shape, dtype=np.float32))
    return H.to_device_storage(a, "bf16", dev), H.to_device_storage(b, "bf16", dev)


def test_static_scratch_entry_point_matches_the_workspace_one():
    dev = torch.device("cuda:0")
    rng = np.random.Generator(np.random.PCG64(7100))
    # the second and third inputs are smaller than the first: what the first call left in the array
    # beyond their own partial sums must not reach their results
    shapes = [(3, 333, 1024), (2, 50, 520), (1, 1, 8), (3, 333, 1024)]
    inputs = [_pair(rng, s, dev) for s in shapes]
    outs = [(torch.full((s[0],), float("nan"), dtype=torch.float32, device=dev),
             torch.full((s[0], s[1]), float("nan"), dtype=torch.float32, device=dev)) for s in shapes]
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    for (a, b), (sim, cos) in zip(inputs, outs):          # back to back on one stream, no sync between
        B.layer_similarity_static(a, b, sim, cos)
    B.layer_similarity_static(inputs[1][0], inputs[1][1], outs[1][0], None)   # without the per-token output
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(dev)["allocation.all.allocated"] == before  # torch's allocator saw no request
    for (a, b), (sim, cos) in zip(inputs, outs):
        want_sim, want_cos = B.layer_similarity(a, b)
        torch.cuda.synchronize()
        assert torch.equal(sim, want_sim) and torch.equal(cos, want_cos)
        assert torch.isfinite(sim).all()


def test_static_scratch_limit_and_argument_errors():
    dev = torch.device("cuda:0")
    L = B.lib()
    a = torch.zeros((1, 16, 64), dtype=torch.bfloat16, device=dev)
    sim = torch.zeros((4,), dtype=torch.float32, device=dev)
    call = L.baklava_layer_similarity_static
    # one tile too many: rejected from the sizes alone, before any pointer is used
    n_seq = 4
    T = (B.LAYER_STATIC_MAX_TILES // n_seq) * 16 + 1
    assert call(a.data_ptr(), a.data_ptr(), n_seq, T, 64, B.BF16, None, sim.data_ptr(), None) == B.ECAPACITY
    assert call(a.data_ptr(), a.data_ptr(), 1, 16, 60, B.BF16, None, sim.data_ptr(), None) == B.EINVAL
    assert call(a.data_ptr(), a.data_ptr(), 1, 16, 64, B.F32, None, sim.data_ptr(), None) == B.EINVAL
    assert call(None, a.data_ptr(), 1, 16, 64, B.BF16, None, sim.data_ptr(), None) == B.EINVAL
    assert call(a.data_ptr(), a.data_ptr(), 1, 16, 64, B.BF16, None, sim.data_ptr(), None) == B.OK
    torch.cuda.synchronize()
    assert float(sim[0]) == 0.0          # zero rows: cosine 0 by the clamp of the norm product
