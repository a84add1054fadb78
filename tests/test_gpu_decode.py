"""GPU parity: baklava_decode_attn against the fp64 oracle (Eq. 1 / Eq. 7), element by element."""
import numpy as np
import pytest
import torch

from paper_2502_13176_amd import binding as B
from paper_2502_13176_amd import synth

pytestmark = pytest.mark.gpu


def _h():
    import gpu_harness
    return gpu_harness


def _kernels_for(w):
    ks = []
    if w.G <= 8:
        ks.append(B.KERNEL_VALU)
    if w.dtype == "bf16" and w.D == 128:
        ks.append(B.KERNEL_MFMA)
    return ks


def test_tiny_workload_full_cache():
    H = _h()
    w = synth.WORKLOADS["tiny"]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    arena = H.make_arena(w)
    st = H.fill_from_host(arena, w, [w.ctx] * arena.n_caches, rng, scores="uniform")
    q, q64 = H.make_q(w, rng, w.L)
    out = H.gpu_decode(arena, w, q)
    err = H.check_decode_against_oracle(arena, w, st, q64, out)
    print(f"tiny: max-abs error {err:.3e}", flush=True)
    arena.close()


@pytest.mark.parametrize("kernel", [B.KERNEL_VALU, B.KERNEL_MFMA])
@pytest.mark.parametrize("chunk", [256, 1024, 4096, 16384])
def test_llama_single_layer_at_full_size(kernel, chunk):
    """LLaMA-3-8B-shaped layer, context 8192, budgets summing to half of 8*8192, caches at budget."""
    H = _h()
    w = synth.WORKLOADS["llama1"]
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = synth.budgets_for(w, B.alloc_proportional)
    arena = H.make_arena(w, budgets)
    arena.set_option(B.OPT_KERNEL, kernel)
    H.set_chunk(arena, chunk)
    lens = [budgets[c % w.Hkv] for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng)
    q, q64 = H.make_q(w, rng, w.L)
    out = H.gpu_decode(arena, w, q)
    err = H.check_decode_against_oracle(arena, w, st, q64, out)
    print(f"llama1 kernel={kernel} chunk={chunk}: max-abs error {err:.3e}", flush=True)
    arena.close()


RAGGED_LENS = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 1000, 1023, 1025, 2500]


@pytest.mark.parametrize("dtype,D,Hq,Hkv", [
    ("bf16", 128, 8, 2), ("bf16", 128, 7, 1), ("bf16", 128, 2, 2), ("bf16", 128, 16, 2), ("bf16", 128, 16, 1),
    ("bf16", 64, 8, 2), ("f32", 64, 4, 2), ("f32", 128, 7, 1), ("f32", 128, 2, 1),
])
def test_ragged_lengths_all_shapes(dtype, D, Hq, Hkv):
    """Lengths around every tile boundary of both kernels, several layers and sequences, with a
    layer sub-range launch as well as the whole stack."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="ragged", L=2, Hq=Hq, Hkv=Hkv, D=D, batch=2, dtype=dtype,
                     seed=77, sink=1, recent=1, slack=0)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    n_caches = w.L * w.batch * w.Hkv
    budgets = [4096] * (w.L * w.Hkv)
    lens = [RAGGED_LENS[(3 * c + 1) % len(RAGGED_LENS)] for c in range(n_caches)]
    arena = H.make_arena(w, budgets)
    st = H.fill_from_host(arena, w, lens, rng)
    q, q64 = H.make_q(w, rng, w.L)
    for kernel in _kernels_for(w):
        arena.set_option(B.OPT_KERNEL, kernel)
        for chunk in (256, 512, 4096):
            H.set_chunk(arena, chunk)
            out = H.gpu_decode(arena, w, q)
            H.check_decode_against_oracle(arena, w, st, q64, out)
        # second layer alone
        out1 = H.gpu_decode(arena, w, q[1:2], layer_begin=1, layer_count=1)
        H.check_decode_against_oracle(arena, w, st, q64[1:2], out1, caches=range(n_caches // 2, n_caches),
                                          layer_begin=1)
        # item targets below the item count at 256-row runs: runs grow (per layer / over the model)
        # until few items are left, down to one item per cache
        H.set_chunk(arena, 256)
        for target in (1, 7, 23):
            arena.set_option(B.OPT_TARGET_ITEMS, target)
            arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, target)
            out = H.gpu_decode(arena, w, q)
            H.check_decode_against_oracle(arena, w, st, q64, out)
            out1 = H.gpu_decode(arena, w, q[1:2], layer_begin=1, layer_count=1)
            H.check_decode_against_oracle(arena, w, st, q64[1:2], out1, caches=range(n_caches // 2, n_caches),
                                          layer_begin=1)
        arena.set_option(B.OPT_TARGET_ITEMS, 0)
        arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, 0)
    arena.close()


@pytest.mark.parametrize("kernel", [B.KERNEL_VALU, B.KERNEL_MFMA])
def test_result_does_not_depend_on_split_factor(kernel):
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="split", Hq=8, Hkv=2, seed=5, slack=0)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [7000, 3333]
    arena = H.make_arena(w, budgets)
    arena.set_option(B.OPT_KERNEL, kernel)
    st = H.fill_from_host(arena, w, budgets, rng)
    q, q64 = H.make_q(w, rng, w.L)
    outs = []
    for chunk in (8192, 3584, 1024, 256):      # 1, 2, 7 and 28 splits of the long cache
        H.set_chunk(arena, chunk)
        outs.append(H.gpu_decode(arena, w, q))
        H.check_decode_against_oracle(arena, w, st, q64, outs[-1])
    for o in outs[1:]:
        assert np.max(np.abs(o - outs[0])) <= 1e-5
    arena.close()


@pytest.mark.parametrize("kernel", [B.KERNEL_VALU, B.KERNEL_MFMA])
def test_peaked_and_large_logits(kernel):
    """A few keys scaled up so single rows dominate the softmax, and logits of magnitude ~80:
    the running-max rescaling must stay finite and accurate."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="peaked", Hq=8, Hkv=2, seed=9, slack=0)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [3000, 1500]
    arena = H.make_arena(w, budgets)
    arena.set_option(B.OPT_KERNEL, kernel)
    st = H.fill_from_host(arena, w, budgets, rng, peaked=True)
    q, q64 = H.make_q(w, rng, w.L)
    H.check_decode_against_oracle(arena, w, st, q64, H.gpu_decode(arena, w, q))
    st = H.fill_from_host(arena, w, budgets, rng, scale=7.0)
    q, q64 = H.make_q(w, rng, w.L, scale=7.0)
    H.check_decode_against_oracle(arena, w, st, q64, H.gpu_decode(arena, w, q))
    # ascending logits: the running maximum changes in every slab
    n = 2048
    K = np.zeros((n, w.D), dtype=np.float32)
    K[:, 0] = np.linspace(-40, 40, n)
    Vv = rng.standard_normal((n, w.D)).astype(np.float32)
    arena2 = H.make_arena(synth.shrink(w, Hq=4, Hkv=1), [n])
    arena2.set_option(B.OPT_KERNEL, kernel)
    w2 = synth.shrink(w, Hq=4, Hkv=1)
    st2 = H.HostState(1)
    st2.K[0], st2.V[0] = synth.f32_to_bf16_bits(K), synth.f32_to_bf16_bits(Vv)
    arena2.k[:n].copy_(H.to_device_storage(st2.K[0], "bf16", arena2.device))
    arena2.v[:n].copy_(H.to_device_storage(st2.V[0], "bf16", arena2.device))
    arena2.set_lengths([n])
    qq = np.zeros((1, 1, 4, w.D), dtype=np.float32)
    qq[..., 0] = [11.0, -11.0, 3.0, 0.5]
    qs = synth.f32_to_bf16_bits(qq)
    H.check_decode_against_oracle(arena2, w2, st2, synth.storage_to_f64(qs, "bf16"), H.gpu_decode(arena2, w2, qs))
    arena.close()
    arena2.close()


def test_error_paths():
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="err", Hq=4, Hkv=2, seed=3, slack=2)
    arena = H.make_arena(w, [300, 200])
    q = torch.zeros((1, 1, 4, 128), dtype=torch.bfloat16, device=arena.device)
    out = torch.zeros((1, 1, 4, 128), dtype=torch.float32, device=arena.device)
    with pytest.raises(B.BaklavaError) as e:           # empty caches
        arena.decode_attn(0, 1, q, out)
    assert e.value.status == B.ESTATE
    with pytest.raises(B.BaklavaError) as e:
        arena.decode_attn(0, 2, q, out)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.BaklavaError) as e:
        arena.set_lengths([303, 1])
    assert e.value.status == B.ECAPACITY
    arena.set_lengths([302, 1])
    kn = torch.zeros((1, 2, 128), dtype=torch.bfloat16, device=arena.device)
    with pytest.raises(B.BaklavaError) as e:           # cache 0 is full
        arena.append(0, 1, kn, kn, 5)
    assert e.value.status == B.ECAPACITY
    assert arena.lengths().tolist() == [302, 1]
    with pytest.raises(B.BaklavaError) as e:
        H.set_chunk(arena, 100)
    assert e.value.status == B.EINVAL
    arena.reset()
    assert arena.lengths().tolist() == [0, 0]
    torch.cuda.synchronize()
    assert arena.len.cpu().tolist() == [0, 0]
    arena.close()


@pytest.mark.parametrize("kernel", [B.KERNEL_VALU, B.KERNEL_MFMA])
def test_fused_append_at_item_boundaries(kernel):
    """baklava_append_decode_attn with the new row landing first / last in a work item, in a new
    work item of its own, and in an empty cache; the result must equal append followed by
    attention, and the oracle."""
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="fusedb", L=1, Hq=8, Hkv=2, batch=4, seed=41, slack=600)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    budgets = [500, 300]
    arena = H.make_arena(w, budgets)
    arena.set_option(B.OPT_KERNEL, kernel)
    H.set_chunk(arena, 256)
    lens = [0, 255, 256, 257, 511, 512, 513, 767]
    st = H.fill_from_host(arena, w, lens, rng)
    for step in range(3):
        q, q64 = H.make_q(w, rng, 1)
        knew = synth.payload(rng, (1, w.batch, w.Hkv, w.D), w.dtype)
        vnew = synth.payload(rng, (1, w.batch, w.Hkv, w.D), w.dtype)
        outd = torch.full((1, w.batch, w.Hq, w.D), float("nan"), dtype=torch.float32, device=arena.device)
        arena.append_decode_attn(0, 1, H.to_device_storage(knew, w.dtype, arena.device),
                                 H.to_device_storage(vnew, w.dtype, arena.device), 900 + step,
                                 H.to_device_storage(q, w.dtype, arena.device), outd)
        torch.cuda.synchronize()
        out = outd.cpu().numpy().astype(np.float64)
        post = H.download(arena, w)
        assert arena.lengths().tolist() == [n + step + 1 for n in lens]
        assert arena.len.cpu().tolist() == arena.lengths().tolist()
        for c in range(arena.n_caches):
            b, h = divmod(c, w.Hkv)
            assert np.array_equal(post.K[c][:-1], st.K[c]) and np.array_equal(post.V[c][:-1], st.V[c])
            assert np.array_equal(post.K[c][-1], knew[0, b, h]) and np.array_equal(post.V[c][-1], vnew[0, b, h])
            assert post.pos[c][-1] == 900 + step and post.score[c][-1] == 0.0
        H.check_decode_against_oracle(arena, w, post, q64, out)
        st = post
    arena.close()


def test_stream_probe_modes():
    """The measurement aid: the copy really copies, the read-only sweeps leave both buffers alone,
    unknown modes and odd sizes are refused."""
    dev = torch.device("cuda:0")
    n = (1 << 22) + 4096 + 16                      # not a multiple of the probe's block size
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    dst = torch.zeros((n,), dtype=torch.uint8, device=dev)
    B.stream_probe(dst, src, n, 0)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    keep = dst.clone()
    for mode in (1, 2, 3):
        B.stream_probe(dst, src, n, mode)
    torch.cuda.synchronize()
    assert torch.equal(dst, keep)
    for bad in (lambda: B.stream_probe(dst, src, n, 4), lambda: B.stream_probe(dst, src, n - 8, 0),
                lambda: B.stream_probe(dst, src, 0, 1)):
        with pytest.raises(B.BaklavaError) as e:
            bad()
        assert e.value.status == B.EINVAL


@pytest.mark.parametrize("kernel", [B.KERNEL_VALU, B.KERNEL_MFMA])
@pytest.mark.parametrize("mode", [1, 2])
def test_kernel_timing_record(kernel, mode):
    """The measurement aid behind the roofline figure: both ways of timing the attention kernel count
    every launch, report a positive time that a host clock around the same calls bounds from above,
    leave the results alone, and the record is empty again after it has been read."""
    import time
    H = _h()
    w = synth.shrink(synth.WORKLOADS["llama1"], name="timed", L=3, Hq=8, Hkv=2, batch=2, seed=43, slack=64)
    rng = np.random.Generator(np.random.PCG64(w.seed))
    arena = H.make_arena(w, [700, 300] * w.L, track=True)       # the tracked instance of the kernel is timed too
    lens = [int(arena.cap_host[c]) - 1 - 37 * (c % 3) for c in range(arena.n_caches)]
    st = H.fill_from_host(arena, w, lens, rng, scores="uniform")
    arena.set_option(B.OPT_KERNEL, kernel)
    H.set_chunk(arena, 256)
    q, q64 = H.make_q(w, rng, w.L)
    ref = H.gpu_decode(arena, w, q)
    arena.set_option(B.OPT_TIME_KERNEL, mode)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    outs = [H.gpu_decode(arena, w, q) for _ in range(3)]           # one launch over all layers each
    qd = H.to_device_storage(q, w.dtype, arena.device)
    out_l = torch.empty((1, w.batch, w.Hq, w.D), dtype=torch.float32, device=arena.device)
    for l in range(w.L):
        arena.decode_attn(l, 1, qd[l:l + 1], out_l)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    with pytest.raises(B.BaklavaError) as e:                        # a record in one mode is read before the mode changes
        arena.set_option(B.OPT_TIME_KERNEL, 3 - mode)
    assert e.value.status == B.ESTATE
    ms, launches = arena.profile_read()
    assert launches == 3 + w.L and 0.0 < ms <= wall_ms
    assert arena.profile_read() == (0.0, 0)
    arena.set_option(B.OPT_TIME_KERNEL, 0)
    for o in outs:
        assert np.array_equal(o, ref)
    H.check_decode_against_oracle(arena, w, st, q64, ref)
    with pytest.raises(B.BaklavaError):
        arena.set_option(B.OPT_TIME_KERNEL, 3)
    arena.close()
