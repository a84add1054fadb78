#!/usr/bin/env python3
"""Benchmark of the ragged per-head KV-cache decode path on one MI355X.

One "step" is one decode step of the whole model: for every layer append the new K/V row to each
cache and run single-query attention over the ragged caches, with the attention weights accumulated
per cached row (the statistic the eviction policy ranks rows by); every `interval` steps every cache
is evicted back to its budget.  Inputs are synthetic and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is K/V bytes read by attention per second over the timed steps
(appends and whatever evictions fall into the region are in the time, not in the bytes; the region's
eviction count is stated, and `eviction` gives the cost of the loop's evictions per step).  Beside
the headline: the same steps with score tracking off, the other launch mode, the second model shape
(qwen) with the same regions, the streaming probes, the one-time kernels and the CPU oracle's rate.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=576,
                    help="untimed steps of the same decode loop before the timed region (default 576: nine evictions at "
                         "an interval of 64, eighteen at 32, after which an eviction costs what it costs in a long "
                         "generation; the first ones after the synthetic start move nearly every row)")
    ap.add_argument("--workload", default="llama32", choices=["tiny", "llama1", "llama32", "qwen", "long"])
    ap.add_argument("--mode", default="layer", choices=["layer", "stack"],
                    help="layer: one attention launch per layer (as a model would issue them); "
                         "stack: one launch over all layers")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 vector-ALU, 2 MFMA")
    ap.add_argument("--chunk", type=int, default=0, help="rows per split-K work item (0 = library default)")
    ap.add_argument("--no-profiling-row", action="store_true",
                    help="skip the measurements of the profiling, prompt-score and layer-importance kernels")
    ap.add_argument("--target-items-whole", type=int, default=-1,
                    help="work items per whole-model launch to aim for (-1 = library default, 0 = off)")
    ap.add_argument("--target-items", type=int, default=-1,
                    help="work items per layer launch to aim for (-1 = library default, 0 = off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-track", action="store_true", help="never accumulate attention scores")
    ap.add_argument("--no-second-workload", action="store_true",
                    help="skip the row of the second model shape (qwen beside llama32)")
    ap.add_argument("--event-mode", type=int, default=2, choices=(1, 2),
                    help="how the roofline region times the attention kernel: 1 = events recorded on the stream "
                         "before and after each launch, 2 = events carried by the kernel's own dispatch")
    ap.add_argument("--evictions", type=int, default=10, help="evictions of the decode loop to time (see `eviction`)")
    ap.add_argument("--emit-row", action="store_true",
                    help="print only this workload's row (how the second workload is measured: in a process of its own)")
    ap.add_argument("--no-compaction", action="store_true", help="attention and appends only")
    ap.add_argument("--keep-pct", type=int, default=0,
                    help="percent of the context kept globally instead of the workload's own (the other reading of "
                         "'compression X%%': X%% kept rather than X%% evicted)")
    ap.add_argument("--interval", type=int, default=0,
                    help="evict every N steps instead of the workload's own interval (capacity = budget + N)")
    ap.add_argument("--policy", default="score", choices=["score", "streaming"],
                    help="eviction policy: sink + recent + top scores, or sink + most recent rows")
    ap.add_argument("--no-other-mode", action="store_true",
                    help="skip the extra region in the other launch mode (keeps profiler traces to one mode)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle leg")
    return ap.parse_args()


def blas_threads():
    """Threads the BLAS under numpy will use for the oracle's matrix products (what `cores` reports)."""
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(arena, w, q_dev, torch, target_seconds):
    """The fp64 oracle's decode attention timed on this machine's host cores over a bounded sample of
    the same caches (layer 0 first, then further layers until the time target is met): once with the
    BLAS pool as it comes (all cores the box grants) and once limited to a single thread, on the same
    caches, each leg with half of the time target."""
    import numpy as np
    from oracle import baklava_oracle as O
    from paper_2502_13176_amd import binding as B
    from paper_2502_13176_amd import synth
    from threadpoolctl import threadpool_limits
    lens = arena.lengths()
    q_host = q_dev.view(torch.int16).cpu().numpy().view(np.uint16) if w.dtype == "bf16" else q_dev.cpu().numpy()
    q64 = synth.storage_to_f64(q_host, w.dtype)
    cpl = w.batch * w.Hkv
    # the library's answer on the same state, for the error of the sampled caches
    arena.set_option(B.OPT_TRACK_SCORES, 0)      # this call only serves the comparison
    out_dev = torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.float32, device=arena.device)
    arena.decode_attn(0, w.L, q_dev, out_dev)
    torch.cuda.synchronize()
    out_host = out_dev.cpu().numpy().astype(np.float64)

    def leg(seconds, max_caches):
        worst, t_used, bytes_done, n_done = 0.0, 0.0, 0, 0
        for c in range(min(arena.n_caches, max_caches)):
            o, n = int(arena.off_host[c]), int(lens[c])
            if w.dtype == "bf16":
                Ks = arena.k[o:o + n].view(torch.int16).cpu().numpy().view(np.uint16)
                Vs = arena.v[o:o + n].view(torch.int16).cpu().numpy().view(np.uint16)
            else:
                Ks, Vs = arena.k[o:o + n].cpu().numpy(), arena.v[o:o + n].cpu().numpy()
            l, rem = divmod(c, cpl)
            b, h = divmod(rem, w.Hkv)
            t0 = time.perf_counter()
            ref, _ = O.decode_attn(q64[l, b, h * w.G:(h + 1) * w.G], synth.storage_to_f64(Ks, w.dtype),
                                   synth.storage_to_f64(Vs, w.dtype))
            t_used += time.perf_counter() - t0
            worst = max(worst, float(np.max(np.abs(out_host[l, b, h * w.G:(h + 1) * w.G] - ref))))
            bytes_done += n * w.token_bytes
            n_done += 1
            if t_used >= seconds:
                break
        return worst, t_used, bytes_done, n_done

    threads_all = blas_threads()
    worst, t_all, bytes_all, n_all = leg(target_seconds / 2, arena.n_caches)
    with threadpool_limits(limits=1):
        threads_one = blas_threads()
        worst1, t_one, bytes_one, n_one = leg(target_seconds / 2, n_all)
    return {
        "value": round(bytes_all / t_all / 1e9, 4), "unit": "GB/s", "cores": int(threads_all), "kind": "oracle",
        "sample": f"fp64 oracle decode attention over the first {n_all} of {arena.n_caches} caches of {w.name} "
                  f"({bytes_all / 1e6:.1f} MB of K/V, {t_all:.1f} s), widening of the stored rows included",
        "single_thread": {"value": round(bytes_one / t_one / 1e9, 4), "unit": "GB/s", "cores": int(threads_one),
                          "sample": f"the same caches, the first {n_one} ({bytes_one / 1e6:.1f} MB, {t_one:.1f} s), "
                                    "BLAS pool limited to one thread"},
        "max_abs_error_vs_oracle_on_sample": max(worst, worst1),
    }


def stream_probe(torch, B, device, nbytes=1 << 32, reps=5):
    """Bandwidth of the library's trivial streaming kernels on this device (a copy and a
    read-only sweep of `nbytes`), timed with events on the launch stream."""
    src = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    dst = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    src.fill_(1)
    out = {"bytes": nbytes}
    for mode, name in ((0, "copy"), (1, "read"), (2, "read_nt"), (3, "read_nt_64_workgroups")):
        B.stream_probe(dst, src, nbytes, mode)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.stream_probe(dst, src, nbytes, mode)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        moved = nbytes * (2 if mode == 0 else 1)
        out[f"{name}_GBps"] = round(moved / ms / 1e6, 1)
    del src, dst
    return out


def profiling_row(torch, B, device, with_cpu_baseline, T=8192, Hq=32, Hkv=8, reps=10):
    """The profiling kernel (Algorithm 1 step 1) on one LLaMA-3-8B-shaped layer of a T-token prompt:
    algorithmic flops (2 D T (T+1) per head: both products, causal half only) per second, timed with
    events on the launch stream; the oracle's rate on the host cores beside it."""
    D = 128
    gen = torch.Generator(device=device)
    gen.manual_seed(4242)
    q = torch.randn((1, Hq, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((1, Hkv, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((1, Hkv, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    sim = torch.empty((1, Hq), dtype=torch.float32, device=device)
    nbytes = B.profile_workspace_bytes(1, Hq, T)
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    stream = torch.cuda.current_stream().cuda_stream

    def run():
        st = B.lib().baklava_profile_similarity(q.data_ptr(), k.data_ptr(), v.data_ptr(), 1, Hq, Hkv, T, D, B.BF16,
                                                None, sim.data_ptr(), None, ws.data_ptr(), nbytes, stream)
        if st != B.OK:
            raise RuntimeError(f"baklava_profile_similarity: status {st}")
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = Hq * 2 * D * T * (T + 1)
    row = {
        "what": "Algorithm 1 step 1: causal attention + token-wise cosine(v_t, out_t) + mean, one layer",
        "config": {"workload": f"LLaMA-3-8B-shaped layer: {Hq} heads, {Hkv} KV heads, D={D}, prompt of {T} tokens, bf16"},
        "us": round(ms * 1e3, 1),
        "roofline": {"bound": "mfma", "kernel": "profile_attn_kernel", "achieved": round(flops / ms / 1e9, 1),
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / ms / 1e9 / 2500.0, 4), "traffic": None,
                     "algorithmic_flops_per_launch": flops},
    }
    if with_cpu_baseline:
        import time
        import numpy as np
        from oracle import baklava_oracle as O
        from paper_2502_13176_amd import synth
        heads = 8
        threads = blas_threads()
        q64 = synth.storage_to_f64(q[0, :heads].view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        G = Hq // Hkv
        n_kv = (heads + G - 1) // G
        k64 = synth.storage_to_f64(k[0, :n_kv].view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        v64 = synth.storage_to_f64(v[0, :n_kv].view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        t0 = time.perf_counter()
        want = [O.head_similarity(q64[h], k64[h // G], v64[h // G])[0] for h in range(heads)]
        dt = time.perf_counter() - t0
        got = sim[0, :heads].cpu().numpy()
        row["cpu_baseline"] = {"value": round(heads * 2 * D * T * (T + 1) / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": int(threads), "kind": "oracle",
                               "sample": f"fp64 oracle head_similarity on {heads} of {Hq} heads ({dt:.1f} s)"}
        row["max_abs_error_vs_oracle_on_sample"] = float(np.max(np.abs(got - np.array(want))))
    return row


def prefill_row(torch, B, synth, device, with_cpu_baseline, T=32768, reps=5):
    """The step before the decode loop for one sequence of the llama32 workload: attention scores of
    a T-token prompt for every cache of one layer (column sums of the causal attention matrices, first
    product only: D T (T+1) algorithmic flops per head), then one eviction from T rows to the layer's
    ragged budgets."""
    import numpy as np
    w = synth.WORKLOADS["llama32"]
    Hq, Hkv, D = w.Hq, w.Hkv, w.D
    budgets = synth.budgets_for(w, B.alloc_proportional)[:Hkv]          # layer 0 of the workload
    arena = B.Arena(1, Hq, Hkv, D, 1, w.dtype, budgets, T, w.sink, w.recent)
    gen = torch.Generator(device=device)
    gen.manual_seed(777)
    q = torch.randn((1, Hq, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((1, Hkv, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((1, Hkv, T, D), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    for c in range(arena.n_caches):
        o = int(arena.off_host[c])
        arena.k[o:o + T].copy_(k[0, c])
        arena.v[o:o + T].copy_(v[0, c])
    arena.pos.zero_()
    arena.set_lengths(np.full(arena.n_caches, T, dtype=np.int32))
    _, _, lse = B.profile_similarity(q, k, v, want_cos=False, want_lse=True)

    def run():
        B.prefill_scores(q, arena.k, lse, arena.score, 1, Hq, Hkv, T, row_off=arena.off)
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = Hq * D * T * (T + 1)
    run()                      # the eviction follows the scores on the stream, as in a prefill: the device is
    e0.record()                # still busy while the host enqueues it, so the events time the device's work
    arena.compact(0, 1)
    e1.record()
    torch.cuda.synchronize()
    ms_evict = e0.elapsed_time(e1)
    kept = int(arena.lengths().astype(np.int64).sum())
    row = {
        "what": "attention scores of a whole prompt (column sums of the causal attention matrices) for one layer, "
                "then one eviction from the prompt length to the layer's budgets",
        "config": {"workload": f"one sequence of llama32, one layer: {Hq} heads, {Hkv} KV heads, D={D}, prompt of {T} "
                               f"tokens, budgets {min(budgets)}..{max(budgets)} rows"},
        "scores_us": round(ms * 1e3, 1),
        "roofline": {"bound": "mfma", "kernel": "prefill_score_kernel", "achieved": round(flops / ms / 1e9, 1),
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / ms / 1e9 / 2500.0, 4), "traffic": None,
                     "algorithmic_flops_per_launch": flops},
        "eviction_us": round(ms_evict * 1e3, 1), "rows_before": Hkv * T, "rows_kept": kept,
    }
    if with_cpu_baseline:
        import time
        from oracle import baklava_oracle as O
        threads = blas_threads()
        Ts, G = 4096, Hq // Hkv
        q64 = synth.storage_to_f64(q[0, :G, :Ts].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        k64 = synth.storage_to_f64(k[0, 0, :Ts].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        t0 = time.perf_counter()
        O.prefill_scores(q64, k64)
        dt = time.perf_counter() - t0
        row["cpu_baseline"] = {"value": round(G * D * Ts * (Ts + 1) / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(threads),
                               "kind": "oracle", "sample": f"fp64 oracle prefill_scores on the first {Ts} tokens of one "
                                                            f"KV head's {G} query heads ({dt:.1f} s)"}
    arena.close()
    return row


def layer_row(torch, B, synth, device, with_cpu_baseline, n_layers=32, T=8192, hidden=4096, reps=10):
    """The layer-importance kernel on the hidden states of a T-token prompt at the input and output of
    every layer of a LLaMA-3-8B-shaped model: 2 * hidden * 2 algorithmic bytes per (layer, token)."""
    import numpy as np
    gen = torch.Generator(device=device)
    gen.manual_seed(999)
    a = torch.randn((n_layers, T, hidden), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    b = (a.float() + 0.3 * torch.randn((n_layers, T, hidden), generator=gen, device=device,
                                       dtype=torch.float32)).to(torch.bfloat16)       # residual stream + update
    sim = torch.empty((n_layers,), dtype=torch.float32, device=device)
    nbytes = int(B.lib().baklava_layer_workspace_bytes(n_layers, T))
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=device)
    stream = torch.cuda.current_stream().cuda_stream

    def run():
        st = B.lib().baklava_layer_similarity(a.data_ptr(), b.data_ptr(), n_layers, T, hidden, B.BF16, None,
                                              sim.data_ptr(), ws.data_ptr(), nbytes, stream)
        if st != B.OK:
            raise RuntimeError(f"baklava_layer_similarity: status {st}")
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nbytes_alg = 2 * n_layers * T * hidden * 2
    row = {
        "what": "layer importance heuristic: token-wise cosine between each layer's input and output hidden state, mean per layer",
        "config": {"workload": f"LLaMA-3-8B-shaped: {n_layers} layers, hidden {hidden}, prompt of {T} tokens, bf16"},
        "us": round(ms * 1e3, 1),
        "roofline": {"bound": "hbm", "kernel": "layer_cosine_kernel", "achieved": round(nbytes_alg / ms / 1e6, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(nbytes_alg / ms / 1e6 / 8000.0, 4),
                     "traffic": read_traffic(None, None, name="layer_cosine_kernel_llama_32layers_T8192.txt")
                     if (n_layers, T, hidden) == (32, 8192, 4096) else None,
                     "algorithmic_bytes_per_launch": nbytes_alg},
    }
    if with_cpu_baseline:
        import time
        from oracle import baklava_oracle as O
        threads = blas_threads()
        a64 = synth.storage_to_f64(a[0].view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        b64 = synth.storage_to_f64(b[0].view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
        t0 = time.perf_counter()
        want, _ = O.layer_similarity(a64, b64)
        dt = time.perf_counter() - t0
        row["cpu_baseline"] = {"value": round(2 * T * hidden * 2 / dt / 1e9, 4), "unit": "GB/s", "cores": int(threads),
                               "kind": "oracle", "sample": f"fp64 oracle layer_similarity on 1 of {n_layers} layers ({dt:.2f} s), "
                                                            "bytes counted as stored (bf16)"}
        row["abs_error_vs_oracle_on_sample"] = abs(float(sim[0]) - want)
    return row


def read_traffic(workload, mode, tracked=False, name=None):
    """HBM bytes per launch of a kernel from the committed counter summary for this very workload, launch
    mode and tracking state, or None when no such summary is committed."""
    path = os.path.join(ROOT, "profiles", name or f"decode_partial_mfma_{workload}_{mode}{'_tracked' if tracked else ''}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def measure_workload(args, name, torch, B, synth, np, want_full_eviction=True):
    """All regions of one workload.  Returns (row, arena, w, q): the caller closes the arena."""
    w = synth.WORKLOADS[name]
    if args.interval > 0:
        w = synth.shrink(w, interval=args.interval, slack=args.interval)
    if args.keep_pct > 0:
        w = synth.shrink(w, keep_pct=args.keep_pct)
    budgets = synth.budgets_for(w, B.alloc_proportional)
    # Score tracking is what the eviction policy ranks rows by (accumulated attention), so it is on for
    # every workload that evicts by score; the same steps with it switched off are reported beside it.
    tracked = not args.no_track and w.dtype == "bf16"
    policy = B.POLICY_STREAMING if args.policy == "streaming" else B.POLICY_SCORE
    arena = B.Arena(w.L, w.Hq, w.Hkv, w.D, w.batch, w.dtype, budgets, w.slack, w.sink, w.recent, policy, tracked)
    gen = synth.fill_arena_on_device(arena, w)
    cpl = w.batch * w.Hkv
    lens0 = np.array([budgets[(c // cpl) * w.Hkv + c % w.Hkv] for c in range(arena.n_caches)], dtype=np.int32)
    lens0 = np.minimum(lens0, w.ctx)
    arena.set_lengths(lens0)
    if args.kernel:
        arena.set_option(B.OPT_KERNEL, args.kernel)
    if args.target_items >= 0:
        arena.set_option(B.OPT_TARGET_ITEMS, args.target_items)
    if args.target_items_whole >= 0:
        arena.set_option(B.OPT_TARGET_ITEMS_WHOLE, args.target_items_whole)
    if args.chunk:
        arena.set_option(B.OPT_CHUNK_TOKENS, args.chunk)
        arena.set_option(B.OPT_CHUNK_TOKENS_WHOLE, args.chunk)

    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dev = arena.device
    q = torch.randn((w.L, w.batch, w.Hq, w.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
    k_new = torch.randn((w.L, w.batch, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
    v_new = torch.randn((w.L, w.batch, w.Hkv, w.D), generator=gen, device=dev, dtype=torch.float32).to(tdt)
    out = torch.zeros((w.L, w.batch, w.Hq, w.D), device=dev, dtype=torch.float32)
    torch.cuda.synchronize()

    interval = 0 if args.no_compaction else w.interval
    st = {"t": 0, "kv_bytes": 0, "evictions": 0, "untracked_since_eviction": False, "track": tracked}
    eviction_events = []      # (step, tracked throughout since the eviction before, start event, end event)

    def set_track(on):
        if tracked:
            arena.set_option(B.OPT_TRACK_SCORES, 1 if on else 0)
            st["track"] = on

    def step(mode):
        st["t"] += 1
        t = st["t"]
        if mode == "layer":
            for l in range(w.L):
                arena.append_decode_attn(l, 1, k_new[l], v_new[l], w.ctx + t, q[l], out[l])
        else:
            arena.append_decode_attn(0, w.L, k_new, v_new, w.ctx + t, q, out)
        st["kv_bytes"] += int(arena.lengths().astype(np.int64).sum()) * w.token_bytes
        st["untracked_since_eviction"] |= not st["track"]
        if interval and t % interval == 0:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            arena.compact(0, w.L)
            e1.record()
            eviction_events.append((t, not st["untracked_since_eviction"], e0, e1))
            st["untracked_since_eviction"] = False
            st["evictions"] += 1
        elif not interval and (t % w.slack == 0):
            arena.set_lengths(lens0)      # appends only: start again from the budgets before a cache overflows

    def align(n_steps, mode):
        """Untimed steps up to the next eviction when one would otherwise fall among the next n_steps: a
        region shorter than the eviction interval then holds none, and says so."""
        if interval and n_steps < interval:
            while st["t"] % interval + n_steps >= interval:
                step(mode)

    def region(n_steps, mode, time_kernel=False):
        """n_steps decode steps bracketed by synchronisation; with time_kernel every attention launch is
        also timed with HIP events on the launch stream (--event-mode)."""
        align(n_steps, mode)
        arena.set_option(B.OPT_TIME_KERNEL, args.event_mode if time_kernel else 0)
        st["kv_bytes"] = 0
        st["evictions"] = 0
        t_first = st["t"] + 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            step(mode)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms, launches = arena.profile_read() if time_kernel else (0.0, 0)
        arena.set_option(B.OPT_TIME_KERNEL, 0)
        r = {"launch_mode": mode, "steps": n_steps, "track_scores": bool(st["track"]), "evictions_in_region": st["evictions"],
             "value": round(st["kv_bytes"] / elapsed / 1e9, 2), "unit": "GB/s",
             "us_per_step": round(elapsed * 1e6 / n_steps, 1),
             "pct_of_hbm_peak": round(100.0 * st["kv_bytes"] / elapsed / 1e9 / HBM_PEAK_GBPS, 2),
             "kv_bytes_per_step": st["kv_bytes"] // n_steps}
        r["_elapsed"], r["_kv_bytes"], r["_kernel_ms"], r["_launches"] = elapsed, st["kv_bytes"], kernel_ms, launches
        r["_t_first"], r["_t_last"] = t_first, st["t"]
        return r

    for _ in range(args.warmup):
        step(args.mode)
    # The timed region: exactly `steps` steps, nothing else on the stream.
    main_r = region(args.steps, args.mode)
    # The same region again with a pair of HIP events per attention launch (by default carried by the
    # kernel's own dispatch, so that they take its start and end): timing a launch costs stream time, so
    # this stays out of the region `value` comes from.
    roof_r = region(min(args.steps, 64), args.mode, time_kernel=True)
    other = "stack" if args.mode == "layer" else "layer"
    other_r = None if args.no_other_mode else region(min(args.steps, 32), other)
    untracked_r = None
    if tracked:
        set_track(False)
        untracked_r = region(args.steps, args.mode)
        set_track(True)

    launches = roof_r["_launches"]
    avg_launch_bytes = roof_r["_kv_bytes"] / max(1, launches)
    avg_launch_s = roof_r["_kernel_ms"] * 1e-3 / max(1, launches)
    achieved = avg_launch_bytes / avg_launch_s / 1e9 if launches else 0.0
    traffic = read_traffic(w.name, args.mode, tracked) if not (args.keep_pct or args.interval or args.chunk) else None

    def public(r):
        return {k: v for k, v in r.items() if not k.startswith("_")}

    row = {
        "workload": f"{w.name}: {w.L} layers x {w.Hkv} KV heads (G={w.G}), D={w.D}, batch {w.batch}, context {w.ctx}, "
                    f"keep {w.keep_pct}% ({sum(budgets) * w.batch} cached tokens)",
        "n_caches": arena.n_caches,
        "timed": public(main_r),
        "roofline": {
            "bound": "hbm", "kernel": "decode_partial_mfma" + ("<score tracking>" if tracked else ""),
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
            "launches": int(launches), "avg_launch_us": round(avg_launch_s * 1e6, 2),
            "timed_with": "HIP events carried by the kernel's dispatch" if args.event_mode == 2
                          else "HIP events recorded on the stream before and after each launch",
            "algorithmic_bytes_per_launch": int(avg_launch_bytes),
        },
    }
    if traffic is None:
        row["roofline"]["traffic_note"] = "no committed counter summary for this workload, launch mode and tracking state"
    if other_r is not None:
        row["other_launch_mode"] = public(other_r)
    if untracked_r is not None:
        row["score_tracking_off"] = public(untracked_r)

    if interval:
        # Evictions as they come in the decode loop (every `interval` steps, scores as the loop left them),
        # timed with events around baklava_compact (which first adds the weights still on record).  The
        # first evictions after the synthetic start remove rows from anywhere in a cache; once the rows
        # the loop itself appended are the ones with the least accumulated attention, the evictions
        # settle.  The loop runs on until `--evictions` of them have been timed; `us` is the median of
        # the last three, the whole series is listed.
        def good():
            return [e for e in eviction_events if e[1] or not tracked]
        while len(good()) < args.evictions and st["t"] < (args.evictions + 8) * interval + 8 * args.steps:
            step(args.mode)
        torch.cuda.synchronize()
        series = [(e[0], round(e[2].elapsed_time(e[3]) * 1e3, 1)) for e in good()]
        if series:
            tail = sorted(us for _, us in series[-3:])
            med = tail[len(tail) // 2]
            # the step time without evictions: those that fell into the timed region are taken out again
            inside = sum(e[2].elapsed_time(e[3]) * 1e3 for e in eviction_events
                         if main_r["_t_first"] <= e[0] <= main_r["_t_last"])
            base_us = main_r["us_per_step"] - inside / main_r["steps"]
            per_step_us = base_us + med / interval
            row["eviction"] = {
                "us": med, "interval_steps": interval,
                "amortised_us_per_step": round(med / interval, 2),
                "us_per_step_without_eviction": round(base_us, 1),
                "value_with_eviction": round(main_r["kv_bytes_per_step"] / per_step_us / 1e3, 2), "unit": "GB/s",
                "us_per_step_with_eviction": round(per_step_us, 1),
                "pct_of_hbm_peak_with_eviction": round(100.0 * main_r["kv_bytes_per_step"] / per_step_us / 1e3 / HBM_PEAK_GBPS, 2),
                "series_step_us": series if len(series) <= 24 else series[:6] + series[-12:],
                "evictions_timed": len(series),
                "note": "baklava_compact as the decode loop reaches it on schedule"
                        + (", scores accumulated by the attention kernel on top of the synthetic prompt scores" if tracked else "")
                        + "; `us` = median of the last three of the series; which rows leave, and hence how many move, follows from the scores",
            }
    if interval and want_full_eviction:
        # One eviction in which nearly every row moves: all caches full, fresh random scores.
        arena.set_lengths(arena.cap_host)
        arena.score.copy_(torch.rand((arena.total_tokens,), generator=gen, device=dev, dtype=torch.float32))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        arena.compact(0, w.L)
        e1.record()
        torch.cuda.synchronize()
        kept_bytes = int(arena.lengths().astype(np.int64).sum()) * w.token_bytes
        ms = e0.elapsed_time(e1)
        row["full_eviction"] = {
            "us": round(ms * 1e3, 1), "kept_kv_bytes": kept_bytes,
            "moved_GBps_read_plus_write": round(2 * kept_bytes / ms / 1e6, 1),
            "amortised_us_per_step": round(ms * 1e3 / interval, 2),
            "note": "every cache at capacity, fresh U(0,1) scores: nearly every kept row moves (the upper end of what an eviction costs)",
        }
    return row, arena, w, q, main_r


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2502_13176_amd import binding as B
    from paper_2502_13176_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    row, arena, w, q, main_r = measure_workload(args, args.workload, torch, B, synth, np)
    if args.emit_row:
        arena.close()
        print(json.dumps(row))
        return
    timed = row["timed"]
    interval = 0 if args.no_compaction else w.interval
    result = {
        "metric": "decode-attn KV bytes read/s", "value": timed["value"], "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(main_r["_elapsed"] * 1e3 / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {
            "workload": row["workload"] + ": fused append + attention for every layer"
                        + (", attention weights accumulated per cached row (score tracking)" if timed["track_scores"] else "")
                        + f"; {timed['evictions_in_region']} evictions in the timed region"
                        + (f" (the loop evicts every {interval} steps, {args.policy} policy: see `eviction` for its cost per step)" if interval else ""),
            "launch_mode": args.mode, "n_caches": arena.n_caches, "kv_bytes_per_step": timed["kv_bytes_per_step"],
            "evictions_in_timed_region": timed["evictions_in_region"], "track_scores": timed["track_scores"],
        },
        "us_per_step": timed["us_per_step"],
        "pct_of_hbm_peak": timed["pct_of_hbm_peak"],
        "roofline": row["roofline"],
    }
    for key in ("score_tracking_off", "other_launch_mode", "eviction", "full_eviction"):
        if key in row:
            result[key] = row[key]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(arena, w, q, torch, args.cpu_seconds)
    arena.close()
    del arena, q
    torch.cuda.empty_cache()
    second = None if args.no_second_workload else {"llama32": "qwen"}.get(args.workload)
    if second:
        # The other model shape the benchmark definition names, same regions, in a child process of its
        # own once this one has given its arena back: an arena allocated after another one of 10+ GB
        # has been freed in the same process streams a few percent slower (measured), and either
        # workload should be timed as a process that runs it alone would see it.  Guarded: the line with
        # the main metric is printed whatever happens here.
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", second, "--emit-row", "--steps", str(args.steps),
               "--warmup", str(args.warmup), "--mode", args.mode, "--policy", args.policy, "--evictions", str(args.evictions)]
        for flag, on in (("--no-track", args.no_track), ("--no-compaction", args.no_compaction), ("--no-other-mode", args.no_other_mode)):
            if on:
                cmd.append(flag)
        try:
            res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
            lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
            result[second] = json.loads(lines[-1]) if res.returncode == 0 and lines else \
                {"error": f"exit status {res.returncode}: {res.stderr.strip()[-300:]}"}
        except Exception as exc:  # noqa: BLE001
            result[second] = {"error": f"{type(exc).__name__}: {exc}"}
    result["stream_probe"] = stream_probe(torch, B, torch.device("cuda:0"))
    if not args.no_profiling_row:
        dev0 = torch.device("cuda:0")
        for key, fn in (("profiling_kernel", lambda: profiling_row(torch, B, dev0, not args.no_cpu_baseline)),
                        ("prefill_scores", lambda: prefill_row(torch, B, synth, dev0, not args.no_cpu_baseline)),
                        ("layer_importance", lambda: layer_row(torch, B, synth, dev0, not args.no_cpu_baseline))):
            try:
                result[key] = fn()
            except Exception as exc:  # noqa: BLE001
                result[key] = {"error": f"{type(exc).__name__}: {exc}"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
