#!/usr/bin/env python3
"""Benchmark of the ragged per-head KV-cache decode path on one MI355X.

One "step" is one decode step of the whole model: for every layer append the new K/V row to each
cache and run single-query attention over the ragged caches; every `interval` steps evict every
cache back to its budget.  Inputs are synthetic and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is K/V bytes read by attention per second over the timed steps
(appends and evictions included in the time, not in the bytes).
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
    ap.add_argument("--warmup", type=int, default=8)
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
    ap.add_argument("--no-track", action="store_true", help="do not accumulate attention scores (long workload)")
    ap.add_argument("--track", action="store_true", help="accumulate attention scores whatever the workload")
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


def cpu_baseline(arena, w, q_dev, torch, target_seconds):
    """The fp64 oracle's decode attention timed on this machine's host cores over a bounded sample of
    the same caches (layer 0 first, then further layers until the time target is met)."""
    import numpy as np
    from oracle import baklava_oracle as O
    from paper_2502_13176_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    lens = arena.lengths()
    q_host = q_dev.view(torch.int16).cpu().numpy().view(np.uint16) if w.dtype == "bf16" else q_dev.cpu().numpy()
    q64 = synth.storage_to_f64(q_host, w.dtype)
    cpl = w.batch * w.Hkv
    # the library's answer on the same state, for the error of the sampled caches
    out_dev = torch.zeros((w.L, w.batch, w.Hq, w.D), dtype=torch.float32, device=arena.device)
    arena.decode_attn(0, w.L, q_dev, out_dev)
    torch.cuda.synchronize()
    out_host = out_dev.cpu().numpy().astype(np.float64)
    worst = 0.0
    t_used, bytes_done, n_done = 0.0, 0, 0
    for c in range(arena.n_caches):
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
        if t_used >= target_seconds:
            break
    return {
        "value": round(bytes_done / t_used / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
        "sample": f"fp64 oracle decode attention over the first {n_done} of {arena.n_caches} caches "
                  f"({bytes_done / 1e6:.1f} MB of K/V, {t_used:.1f} s), widening of the stored rows included",
        "max_abs_error_vs_oracle_on_sample": worst,
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
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
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
    e0.record()
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
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
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
                     "traffic": read_traffic(None, None, "layer_cosine_kernel_llama_32layers_T8192.txt")
                     if (n_layers, T, hidden) == (32, 8192, 4096) else None,
                     "algorithmic_bytes_per_launch": nbytes_alg},
    }
    if with_cpu_baseline:
        import time
        from oracle import baklava_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count() or 1
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


def read_traffic(workload, mode, name=None):
    """HBM bytes per launch of a kernel, from the committed counter summary (if any)."""
    path = os.path.join(ROOT, "profiles", name or f"decode_partial_mfma_{workload}_{mode}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


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
    w = synth.WORKLOADS[args.workload]
    if args.interval > 0:
        w = synth.shrink(w, interval=args.interval, slack=args.interval)
    if args.keep_pct > 0:
        w = synth.shrink(w, keep_pct=args.keep_pct)
    budgets = synth.budgets_for(w, B.alloc_proportional)
    track = (w.scores == "kernel" or args.track) and not args.no_track
    policy = B.POLICY_STREAMING if args.policy == "streaming" else B.POLICY_SCORE
    arena = B.Arena(w.L, w.Hq, w.Hkv, w.D, w.batch, w.dtype, budgets, w.slack, w.sink, w.recent,
                    policy, track)
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
    q = torch.randn((w.L, w.batch, w.Hq, w.D), generator=gen, device=arena.device, dtype=torch.float32).to(tdt)
    k_new = torch.randn((w.L, w.batch, w.Hkv, w.D), generator=gen, device=arena.device, dtype=torch.float32).to(tdt)
    v_new = torch.randn((w.L, w.batch, w.Hkv, w.D), generator=gen, device=arena.device, dtype=torch.float32).to(tdt)
    out = torch.zeros((w.L, w.batch, w.Hq, w.D), device=arena.device, dtype=torch.float32)
    torch.cuda.synchronize()

    state = {"t": 0, "kv_bytes": 0, "compactions": 0}
    interval = 0 if args.no_compaction else w.interval

    def step(mode):
        state["t"] += 1
        t = state["t"]
        if mode == "layer":
            for l in range(w.L):
                arena.append_decode_attn(l, 1, k_new[l], v_new[l], w.ctx + t, q[l], out[l])
        else:
            arena.append_decode_attn(0, w.L, k_new, v_new, w.ctx + t, q, out)
        state["kv_bytes"] += int(arena.lengths().astype(np.int64).sum()) * w.token_bytes
        if interval and t % interval == 0:
            arena.compact(0, w.L)
            state["compactions"] += 1
        elif not interval and (t % w.slack == 0):
            # appends only: start again from the budgets before a cache overflows
            arena.set_lengths(lens0)

    def region(n_steps, mode, time_kernel):
        """n_steps decode steps bracketed by synchronisation; with time_kernel every attention
        launch is also bracketed by HIP events on the launch stream."""
        arena.set_option(B.OPT_TIME_KERNEL, 1 if time_kernel else 0)
        state["kv_bytes"] = 0
        state["compactions"] = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_steps):
            step(mode)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms, launches = arena.profile_read() if time_kernel else (0.0, 0)
        arena.set_option(B.OPT_TIME_KERNEL, 0)
        return {"elapsed": elapsed, "kv_bytes": state["kv_bytes"], "compactions": state["compactions"],
                "kernel_ms": kernel_ms, "launches": launches, "steps": n_steps}

    for _ in range(args.warmup):
        step(args.mode)
    # The timed region: exactly `steps` steps, nothing else on the stream.
    main_r = region(args.steps, args.mode, time_kernel=False)
    # The same region again with event brackets around every attention launch: the brackets cost a
    # few microseconds of stream time each, so they stay out of the region `value` comes from.
    roof_r = region(min(args.steps, 64), args.mode, time_kernel=True)
    # Upper bound for comparison: all layers in one launch.
    other = "stack" if args.mode == "layer" else "layer"
    other_r = None if args.no_other_mode else region(min(args.steps, 32), other, time_kernel=False)

    elapsed = main_r["elapsed"]
    ms_per_step = elapsed * 1e3 / args.steps
    gbps = main_r["kv_bytes"] / elapsed / 1e9
    launches = roof_r["launches"]
    avg_launch_bytes = roof_r["kv_bytes"] / max(1, launches)
    avg_launch_s = roof_r["kernel_ms"] * 1e-3 / max(1, launches)
    achieved = avg_launch_bytes / avg_launch_s / 1e9 if launches else 0.0
    state["kv_bytes"] = main_r["kv_bytes"]
    state["compactions"] = main_r["compactions"]

    result = {
        "metric": "decode-attn KV bytes read/s", "value": round(gbps, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {w.L} layers x {w.Hkv} KV heads (G={w.G}), D={w.D}, batch {w.batch}, "
                        f"context {w.ctx}, keep {w.keep_pct}% ({sum(budgets) * w.batch} cached tokens), "
                        f"compaction every {interval} steps ({args.policy} policy)" if interval else
                        f"{w.name}: attention and appends only",
            "launch_mode": args.mode, "n_caches": arena.n_caches, "kv_bytes_per_step": state["kv_bytes"] // args.steps,
            "compactions_in_timed_region": state["compactions"], "track_scores": bool(track),
        },
        "us_per_step": round(ms_per_step * 1e3, 1),
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "roofline": {
            "bound": "hbm", "kernel": "decode_partial", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic(w.name, args.mode),
            "launches": int(launches), "avg_launch_us": round(avg_launch_s * 1e6, 2),
            "algorithmic_bytes_per_launch": int(avg_launch_bytes),
        },
    }
    if other_r is not None:
      result["other_launch_mode"] = {
          "launch_mode": other, "steps": other_r["steps"],
          "value": round(other_r["kv_bytes"] / other_r["elapsed"] / 1e9, 2), "unit": "GB/s",
          "us_per_step": round(other_r["elapsed"] * 1e6 / other_r["steps"], 1),
          "pct_of_hbm_peak": round(100.0 * other_r["kv_bytes"] / other_r["elapsed"] / 1e9 / HBM_PEAK_GBPS, 2),
      }
    if not args.no_compaction:
        # One eviction in which nearly every row moves: all caches full, fresh random scores.
        arena.set_lengths(arena.cap_host)
        arena.score.copy_(torch.rand((arena.total_tokens,), generator=gen, device=arena.device, dtype=torch.float32))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        arena.compact(0, w.L)
        e1.record()
        torch.cuda.synchronize()
        kept_bytes = int(arena.lengths().astype(np.int64).sum()) * w.token_bytes
        ms = e0.elapsed_time(e1)
        result["full_eviction"] = {
            "us": round(ms * 1e3, 1), "kept_kv_bytes": kept_bytes,
            "moved_GBps_read_plus_write": round(2 * kept_bytes / ms / 1e6, 1),
            "note": "every cache at capacity, fresh U(0,1) scores: nearly every kept row moves",
        }
    result["stream_probe"] = stream_probe(torch, B, arena.device)
    if not args.no_profiling_row:
        # the next row of the path after the decode loop's own: the one-time profiling kernel
        # (each guarded: the line with the main metric is printed whatever happens to these)
        for key, fn in (("profiling_kernel", lambda: profiling_row(torch, B, arena.device, not args.no_cpu_baseline)),
                        ("prefill_scores", lambda: prefill_row(torch, B, synth, arena.device, not args.no_cpu_baseline)),
                        ("layer_importance", lambda: layer_row(torch, B, synth, arena.device, not args.no_cpu_baseline))):
            try:
                result[key] = fn()
            except Exception as exc:  # noqa: BLE001
                result[key] = {"error": f"{type(exc).__name__}: {exc}"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(arena, w, q, torch, args.cpu_seconds)
    arena.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
