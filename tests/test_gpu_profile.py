"""GPU parity: baklava_profile_similarity (Algorithm 1, step 1) against the oracle, token by token
and for the per-head mean; baklava_kv_importance closes the loop to the budget allocator."""
import numpy as np
import pytest
import torch

from oracle import baklava_oracle as O
from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu

# Per-token cosines: the kernel keeps each softmax weight as two bf16 terms (~16 bits) for the
# second product, takes exp2 from the hardware approximation (relative error ~1e-6 after the
# fp32 logit's own rounding of up to |logit| * 2^-24 * ln 2) and accumulates in fp32.  The cosine
# ignores the common scale of the weights; what remains is a relative error of ~2^-16 per weight,
# independent across keys.  Bound taken: 1e-4 per token (2e-3 / 20, the attention tolerance is not
# needed here), 2e-5 for the mean over a prompt.
COS_TOL = 1e-4
MEAN_TOL = 2e-5


def _h():
    import gpu_harness
    return gpu_harness


def run_case(q_bits, k_bits, v_bits):
    """q_bits [batch, Hq, T, D], k_bits / v_bits [batch, Hkv, T, D]: bf16 bit patterns (uint16)."""
    H = _h()
    dev = torch.device("cuda:0")
    q, k, v = (H.to_device_storage(x, "bf16", dev) for x in (q_bits, k_bits, v_bits))
    sim, cos = B.profile_similarity(q, k, v)
    torch.cuda.synchronize()
    sim, cos = sim.cpu().numpy().astype(np.float64), cos.cpu().numpy().astype(np.float64)
    q64, k64, v64 = (synth.storage_to_f64(x, "bf16") for x in (q_bits, k_bits, v_bits))
    batch, Hq, T, D = q64.shape
    G = Hq // k64.shape[1]
    worst_cos = worst_mean = 0.0
    for b in range(batch):
        for h in range(Hq):
            want_mean, want_cos = O.head_similarity(q64[b, h], k64[b, h // G], v64[b, h // G])
            assert np.all(np.isfinite(cos[b, h]))
            e = float(np.max(np.abs(cos[b, h] - want_cos)))
            assert e <= COS_TOL, f"batch {b} head {h}: per-token cosine error {e:.3e}"
            em = abs(float(sim[b, h]) - want_mean)
            assert em <= MEAN_TOL, f"batch {b} head {h}: mean error {em:.3e}"
            # the mean the kernel reports is the mean of the cosines it reports
            assert abs(float(sim[b, h]) - float(cos[b, h].mean())) <= 1e-5
            worst_cos, worst_mean = max(worst_cos, e), max(worst_mean, em)
    return sim, cos, worst_cos, worst_mean


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 350, 700])
def test_prompt_lengths_around_every_tile_boundary(T):
    rng = np.random.Generator(np.random.PCG64(9000 + T))
    q = synth.payload(rng, (1, 4, T, 128), "bf16")
    k = synth.payload(rng, (1, 2, T, 128), "bf16")
    v = synth.payload(rng, (1, 2, T, 128), "bf16")
    _, cos, wc, wm = run_case(q, k, v)
    assert abs(cos[0, 0, 0] - 1.0) <= 1e-6            # the first token sees only itself
    print(f"T={T}: worst per-token error {wc:.2e}, worst mean error {wm:.2e}", flush=True)


@pytest.mark.parametrize("batch,Hq,Hkv", [(2, 8, 2), (1, 7, 1), (3, 2, 2), (1, 16, 1)])
def test_head_grouping_and_batches(batch, Hq, Hkv):
    rng = np.random.Generator(np.random.PCG64(9100 + Hq))
    T = 300
    q = synth.payload(rng, (batch, Hq, T, 128), "bf16")
    k = synth.payload(rng, (batch, Hkv, T, 128), "bf16")
    v = synth.payload(rng, (batch, Hkv, T, 128), "bf16")
    run_case(q, k, v)


def test_peaked_and_large_logits():
    """A few keys dominate (x8 rows) and all logits are large (queries x4): the running-max rescale."""
    rng = np.random.Generator(np.random.PCG64(9200))
    T = 400
    q = synth.f32_to_bf16_bits(4.0 * rng.standard_normal((1, 4, T, 128), dtype=np.float32))
    k = synth.payload(rng, (1, 2, T, 128), "bf16", peaked=True)
    v = synth.payload(rng, (1, 2, T, 128), "bf16")
    run_case(q, k, v)


def test_graded_heads_from_uniform_to_identity_attention():
    """Keys equal to the queries times a per-head temperature: from uniform attention (similarity of
    prefix means) to nearly the identity (similarity close to 1, importance close to 0), the range
    the paper's heat maps show; then Algorithm 1 step 2 and the allocator on the result."""
    rng = np.random.Generator(np.random.PCG64(9300))
    T, Hq = 512, 8
    base = rng.standard_normal((1, Hq, T, 128), dtype=np.float32)
    temps = np.array([0.0, 0.02, 0.05, 0.1, 0.15, 0.2, 0.3, 0.4], dtype=np.float32)
    q = synth.f32_to_bf16_bits(base)
    k = synth.f32_to_bf16_bits(base * temps[None, :, None, None])          # one KV head per query head
    v = synth.payload(rng, (1, Hq, T, 128), "bf16")
    sim, _, _, _ = run_case(q, k, v)
    s = sim[0]
    assert np.all(np.diff(s) > 0)                    # sharper attention -> output closer to the input row
    assert s[0] < 0.2 and s[-1] > 0.9
    imp = B.kv_importance(s[None, :], 1, Hq, Hq)
    assert np.allclose(imp, O.kv_importance(s[None, :], 1), rtol=0, atol=1e-15)
    budgets = B.alloc_proportional(imp[0] + 1e-6, 8 * 1024, 64, 4096)
    assert sum(budgets) == 8 * 1024 and all(b0 >= b1 for b0, b1 in zip(budgets, budgets[1:]))


def test_zero_value_rows_give_zero_cosine():
    rng = np.random.Generator(np.random.PCG64(9400))
    T = 150
    q = synth.payload(rng, (1, 2, T, 128), "bf16")
    k = synth.payload(rng, (1, 1, T, 128), "bf16")
    v = synth.payload(rng, (1, 1, T, 128), "bf16")
    v[0, 0, 40] = 0                                   # bf16 +0.0
    v[0, 0, 0] = 0                                    # the first token's output row is then zero as well
    _, cos, _, _ = run_case(q, k, v)
    assert cos[0, 0, 40] == 0.0 and cos[0, 1, 40] == 0.0 and cos[0, 0, 0] == 0.0


def test_results_are_deterministic_and_errors_are_reported():
    H = _h()
    rng = np.random.Generator(np.random.PCG64(9500))
    dev = torch.device("cuda:0")
    T = 260
    q = H.to_device_storage(synth.payload(rng, (1, 4, T, 128), "bf16"), "bf16", dev)
    k = H.to_device_storage(synth.payload(rng, (1, 2, T, 128), "bf16"), "bf16", dev)
    v = H.to_device_storage(synth.payload(rng, (1, 2, T, 128), "bf16"), "bf16", dev)
    s1, c1 = B.profile_similarity(q, k, v)
    s2, c2 = B.profile_similarity(q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(s1, s2) and torch.equal(c1, c2)
    s3, c3 = B.profile_similarity(q, k, v, want_cos=False)
    torch.cuda.synchronize()
    assert c3 is None and torch.equal(s1, s3)
    # error paths: too small a workspace, wrong head dimension
    sim = torch.empty((1, 4), dtype=torch.float32, device=dev)
    ws = torch.empty((256,), dtype=torch.uint8, device=dev)
    st = B.lib().baklava_profile_similarity(q.data_ptr(), k.data_ptr(), v.data_ptr(), 1, 4, 2, T, 128, B.BF16, None,
                                            sim.data_ptr(), None, ws.data_ptr(), 8, None)
    assert st == B.ECAPACITY
    st = B.lib().baklava_profile_similarity(q.data_ptr(), k.data_ptr(), v.data_ptr(), 1, 4, 2, T, 64, B.BF16, None,
                                            sim.data_ptr(), None, ws.data_ptr(), 256, None)
    assert st == B.EINVAL
    st = B.lib().baklava_profile_similarity(q.data_ptr(), k.data_ptr(), v.data_ptr(), 1, 4, 3, T, 128, B.BF16, None,
                                            sim.data_ptr(), None, ws.data_ptr(), 256, None)
    assert st == B.EINVAL


def test_full_size_layer_sampled_heads_and_any_size_properties():
    """The configuration bench.py times (one LLaMA-3-8B-shaped layer, prompt of 8192 tokens): three
    heads against the oracle token by token, every head against properties that hold at any size."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    Hq, Hkv, T, D = 32, 8, 8192, 128
    q = torch.randn((1, Hq, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((1, Hkv, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((1, Hkv, T, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    sim, cos = B.profile_similarity(q, k, v)
    torch.cuda.synchronize()
    sim_h, cos_h = sim.cpu().numpy().astype(np.float64), cos.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(cos_h)) and np.all(np.abs(cos_h) <= 1.0 + 1e-5)
    assert np.all(np.abs(cos_h[0, :, 0] - 1.0) <= 1e-6)                 # every head's first token
    assert np.allclose(sim_h[0], cos_h[0].mean(axis=1), rtol=0, atol=1e-5)
    H = _h()
    G = Hq // Hkv
    worst = 0.0
    for h in (0, 13, 31):
        q64 = synth.storage_to_f64(H.from_device_storage(q[0, h], "bf16"), "bf16")
        k64 = synth.storage_to_f64(H.from_device_storage(k[0, h // G], "bf16"), "bf16")
        v64 = synth.storage_to_f64(H.from_device_storage(v[0, h // G], "bf16"), "bf16")
        want_mean, want_cos = O.head_similarity(q64, k64, v64)
        e = float(np.max(np.abs(cos_h[0, h] - want_cos)))
        assert e <= COS_TOL and abs(sim_h[0, h] - want_mean) <= MEAN_TOL
        worst = max(worst, e)
    print(f"T=8192 layer: worst per-token cosine error on 3 sampled heads {worst:.2e}", flush=True)
