#!/usr/bin/env python3
"""Benchmark of the PRESERVE decode step on one MI355X.

A "step" is one pass of the whole hot path (all layers: norms, QKV, RoPE + KV append, decode attention, O, comm
window #1 || prefetch, gate/up + SwiGLU, down, comm window #2 || prefetch) over one batch of synthetic input that is
already resident in HBM.  The default workload is c2, one TP=8 shard of a Llama-3-8B-shaped model (the configuration
the metric is quoted on).  Prints ONE JSON line.

Protocol (per mode: prefetch off, prefetch on into the memory-side cache only, prefetch on with the policy's
`prelaunch` extension):
  * W untimed steps, then exactly K steps between two full synchronisations -> mean us/layer (`value`,
    `us_per_layer_prefetch_off`, `us_per_layer_cache_only`);
  * K more steps, each bracketed by a pair of events on the caller's stream -> median, p10 and p90 per step;
  * when a step moves less than the memory-side cache holds (the small workload), the same K event-timed steps again
    with 1 GiB streamed through the GPU before each one, outside the timed region, so that the step starts from HBM
    as a multi-GB model would ("cold"); the back-to-back numbers are then the "hot" ones.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--budget-mb 64] ...
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
CACHE_BYTES = 256 << 20          # memory-side cache of the device
FLUSH_BYTES = 1 << 30


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--layers", type=int, default=0, help="materialise only the first N layers (0 = all)")
    ap.add_argument("--budget-mb", type=float, default=0.0,
                    help="Algorithm 1's capacity C; 0 = what the prefetch kernel can pull inside one window "
                         "(window us x 4.5 MB/us), capped at 192 MB of the 256 MB Infinity Cache")
    ap.add_argument("--chunk-mb", type=float, default=0.0)
    ap.add_argument("--cu-budget", type=int, default=256)
    ap.add_argument("--partial", type=int, default=1,
                    help="1 = an operator that does not fit the rest of the budget is prefetched in part (policy extension; a KV "
                         "cache or a wide projection can exceed any budget); 0 = whole operators only, as in Algorithm 1")
    ap.add_argument("--join", type=int, default=0)
    ap.add_argument("--prelaunch", type=int, default=1,
                    help="1 = the first operator after a window is launched at the window's start and holds its weights in "
                         "registers until the window ends (policy extension; at batch 3-32 the gate/up projection only, "
                         "above that none)")
    ap.add_argument("--targets", type=int, default=3)
    ap.add_argument("--window-us", type=float, nargs=2, default=None)
    ap.add_argument("--tune", type=int, default=0,
                    help="1 = let the library time its candidate attention splits on layer 0 first (psv_tune_attention); "
                         "the default split is within ~1 %% of the tuned one on the five workloads")
    ap.add_argument("--fused", type=int, default=-1,
                    help="kernels of the batch-1 path (psv_set_fused_kernels): 0 = one per operator, 1 = one per inter-window "
                         "segment, 2 = the whole step as one kernel, -1 (default) = the library chooses by shape")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=0, help="layers the oracle is timed on (0 = auto)")
    ap.add_argument("--seed", type=int, default=2501)
    ap.add_argument("--contiguous", action="store_true", help="force a contiguous (unpaged) KV cache")
    ap.add_argument("--format", default="bf16", choices=["bf16", "int8", "w8", "kv8"],
                    help="storage format of weights and KV-cache: bf16 (the benchmark's), int8 (both, the paper's "
                         "measurement precision), w8 / kv8 (only the weights / only the cache in int8)")
    ap.add_argument("--weight-layout", default="", choices=["", "row", "tiled"],
                    help="storage order of the projection matrices: row-major, or the tiled order of the matrix-core "
                         "projections (default: the workload's own)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="also launch one plain copy kernel of this size (known bytes, to scale hardware counters)")
    ap.add_argument("--skip-kernel-table", action="store_true", help="omit the per-operator event timing passes")
    ap.add_argument("--skip-cold", action="store_true", help="omit the cold-cache pass of small workloads")
    ap.add_argument("--also", default="c1,c3,c4,c5",
                    help="other workloads measured by the same code on their first layers (real shapes; default policy) and "
                         "reported under other_workloads; empty = none")
    ap.add_argument("--also-layers", type=int, default=4)
    return ap.parse_args()


def time_steps(sess, steps, warmup):
    """W untimed steps, then exactly K steps between two full synchronisations.  Returns ms per step."""
    import torch
    for _ in range(warmup):
        sess.step()
    sess.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        sess.step()
    sess.sync()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def event_steps(sess, steps, flush=None):
    """K steps, each between two events on the caller's (main) stream; `flush` (a device buffer) is streamed through the
    GPU before each step, outside the timed region.  Returns the sorted step times in us."""
    import torch
    from paper_2501_08192_amd import binding as psv
    pairs = []
    for _ in range(steps):
        if flush is not None:
            psv.psv_prefetch_region(flush, flush.numel(), 1024, sess.main)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(sess.main)
        sess.step()
        e1.record(sess.main)
        pairs.append((e0, e1))
    sess.sync()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)


def spread(us_sorted, layers):
    n = len(us_sorted)
    pick = lambda q: us_sorted[min(n - 1, max(0, int(round(q * (n - 1)))))] / layers
    return {"median": round(pick(0.5), 3), "p10": round(pick(0.1), 3), "p90": round(pick(0.9), 3)}


def profile_op(sess, op, steps):
    """Average duration (us) of one operator's kernel, bracketed by HIP events on the main stream."""
    from paper_2501_08192_amd import binding as psv
    psv.psv_set_profile_op(sess.ctx, op)
    for _ in range(steps):
        sess.step()
    ms, n = psv.psv_get_profile(sess.ctx)
    psv.psv_set_profile_op(sess.ctx, -1)
    return (ms * 1e3 / n if n else 0.0), n


def cpu_baseline(sess, n_layers, target_s=10.0, max_reps=40):
    """The CPU oracle, as it stands, on the first n_layers of the same workload (host cores of this machine),
    repeated until about target_s seconds of CPU work have been timed."""
    import numpy as np
    import oracle
    w = sess.w
    m = oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, 16, w.rms_eps, w.rope_theta)
    x0 = sess.x_in.cpu().numpy().astype(np.float64)
    pt = sess.page_table_host.numpy() if w.paged else None
    lens = sess.seq_lens_host.numpy()
    host = [(sess.host_layer(l), *sess.host_pools(l)) for l in sess.layers[:n_layers]]
    reps, total = 0, 0.0
    while reps < max_reps and (total < target_s or reps < 1):
        x = x0
        t0 = time.perf_counter()
        for lw, kp, vp in host:
            x = oracle.decode_layer_x(m, lw, kp, vp, pt, w.blocks_per_seq, lens, x)
        total += time.perf_counter() - t0
        reps += 1
    return total * 1e6 / (reps * len(host)), len(host), reps, oracle.num_threads()


def other_workload(name, n_layers, steps, warmup, seed):
    """The same three modes on the first layers of another workload (its real shape; more layers would only repeat
    them).  Each of these moves far more per step than the memory-side cache holds, except the small c1, which is
    measured whole, hot and cold."""
    import torch
    from paper_2501_08192_amd import binding as psv
    from paper_2501_08192_amd import synth
    from paper_2501_08192_amd.harness import Session, default_policy
    w = synth.WORKLOADS[name]
    L = min(n_layers, w.n_layers)
    with Session(w, seed=seed, layers=list(range(L))) as sess:
        modes = {"off": psv.prefetch_policy(mode=0), "cache_only": default_policy(w, prelaunch=0), "on": default_policy(w)}
        flush = None
        if w.layer_bytes * L < CACHE_BYTES * 2:
            flush = torch.empty(FLUSH_BYTES, dtype=torch.uint8, device="cuda").zero_()
        res = {"layers_run": L, "layers_total": w.n_layers, "layer_bytes": w.layer_bytes, "us_per_layer": {}, "step_us_per_layer": {}}
        outs = {}
        for mode, pol in modes.items():
            sess.set_policy(pol)
            outs[mode] = sess.run().clone()
            res["us_per_layer"][mode] = round(time_steps(sess, steps, warmup) * 1e3 / L, 3)
            res["step_us_per_layer"][mode] = spread(event_steps(sess, steps), L)
            if flush is not None:
                res.setdefault("cold_step_us_per_layer", {})[mode] = spread(event_steps(sess, steps, flush), L)
        u = res["us_per_layer"]
        res["speedup_cache_only"] = round(u["off"] / u["cache_only"], 4)
        res["speedup_prelaunch"] = round(u["off"] / u["on"], 4)
        if flush is not None:
            cs = res["cold_step_us_per_layer"]
            res["cold_speedup_cache_only"] = round(cs["off"]["median"] / cs["cache_only"]["median"], 4)
            res["cold_speedup_prelaunch"] = round(cs["off"]["median"] / cs["on"]["median"], 4)
        win = sum(w.window_us)
        res["hbm_frac_outside_windows"] = {m: round(w.layer_bytes / max(1e-9, u[m] - win) / 1e3 / HBM_PEAK_GBPS, 4) for m in ("off", "on")}
        res["on_off_bit_identical"] = bool(torch.equal(outs["off"], outs["on"]) and torch.equal(outs["off"], outs["cache_only"]))
    del flush
    torch.cuda.empty_cache()
    return res


def per_operator_leg(w, layers, steps, warmup, seed, policies, gate_bytes):
    """The same workload with one kernel per operator (psv_set_fused_kernels 0), for a record whose timed path runs the
    per-segment kernels: the three modes and the gate/up kernel's own bandwidth with prefetching off."""
    from paper_2501_08192_amd import binding as psv
    from paper_2501_08192_amd.harness import Session
    with Session(w, seed=seed, layers=layers, fused=0) as sess:
        L = len(sess.layers)
        res = {"us_per_layer": {}}
        for mode, pol in policies.items():
            sess.set_policy(pol)
            sess.run()
            res["us_per_layer"][mode] = round(time_steps(sess, steps, warmup) * 1e3 / L, 3)
        sess.set_policy(policies["off"])
        t, n = profile_op(sess, psv.PSV_OP_GATE, max(3, min(steps, 10)))
        res["roofline_gate_up"] = {"kernel": "gate/up projection + SwiGLU (prefetch off), not in the timed path of this record",
                                   "bytes_per_launch": gate_bytes, "avg_us": round(t, 3), "launches": n,
                                   "achieved": round(gate_bytes / t / 1e3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                   "frac": round(gate_bytes / t / 1e3 / HBM_PEAK_GBPS, 4)}
    return res


def stored_traffic(workload, kernel):
    """HBM bytes per launch of a kernel as recorded in the committed rocprofv3 counter summary of this workload:
    (bytes, path of the summary) or (None, None).  A stored figure from an earlier profiler run, not a measurement
    of this run -- hardware counters cannot be read from inside the benchmark."""
    import re
    rel = os.path.join("profiles", "%s_pmc_hbm_traffic.md" % workload)
    try:
        m = re.search(r"traffic_bytes_per_launch\[%s,%s\]\s*=\s*(\d+)" % (workload, kernel), open(os.path.join(ROOT, rel)).read())
        return (int(m.group(1)), rel) if m else (None, None)
    except OSError:
        return None, None


def main():
    a = parse()
    if a.gpus != 1:
        sys.stderr.write("bench.py: this build measures one GPU's shard only (no collectives are part of it); "
                         "run with --gpus 1\n")
        sys.exit(2)
    import torch
    from paper_2501_08192_amd import binding as psv
    from paper_2501_08192_amd import synth
    from paper_2501_08192_amd.harness import Session, default_policy

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU\n")
        sys.exit(1)
    w = synth.WORKLOADS[a.workload]
    if a.window_us is not None:
        w = w.scaled(window_us=tuple(a.window_us))
    if a.contiguous:
        w = w.scaled(paged=False)
    if a.format != "bf16":
        w = w.scaled(weight_format="int8" if a.format in ("int8", "w8") else "bf16",
                     kv_format="int8" if a.format in ("int8", "kv8") else "bf16")
    if a.weight_layout:
        w = w.scaled(weight_layout=a.weight_layout)
    layers = list(range(a.layers)) if a.layers else None
    sess = Session(w, seed=a.seed, layers=layers, fused=None if a.fused < 0 else a.fused)
    L = len(sess.layers)
    MB = 1 << 20
    if a.budget_mb <= 0:
        a.budget_mb = min(192.0, max(w.window_us) * 4.5)
    # with no flags `on` is harness.default_policy(w), the configuration the full-size parity tests run
    kw = dict(targets=a.targets, budget_bytes=int(a.budget_mb * MB), chunk_bytes=int(a.chunk_mb * MB),
              cu_budget=a.cu_budget, partial=a.partial, join=a.join)
    modes = {"off": psv.prefetch_policy(mode=0),
             "cache_only": default_policy(w, prelaunch=0, **kw),        # the paper's scheme: every prefetch goes to the cache
             "on": default_policy(w, prelaunch=a.prelaunch, **kw)}

    attn_chunk = sess.tune_attention() if a.tune else 0
    step_bytes = w.layer_bytes * L
    flush = None
    if step_bytes < CACHE_BYTES * 2 and not a.skip_cold:      # the whole step (nearly) fits the memory-side cache
        flush = torch.empty(FLUSH_BYTES, dtype=torch.uint8, device="cuda").zero_()

    ms, hot, cold, outputs = {}, {}, {}, {}
    for name, pol in modes.items():
        sess.set_policy(pol)
        outputs[name] = sess.run().clone()
        ms[name] = time_steps(sess, a.steps, a.warmup)
        hot[name] = spread(event_steps(sess, a.steps), L)
        if flush is not None:
            cold[name] = spread(event_steps(sess, max(10, min(a.steps, 60)), flush), L)
    identical = bool(torch.equal(outputs["off"], outputs["on"]) and torch.equal(outputs["off"], outputs["cache_only"]))
    stats = psv.psv_get_stats(sess.ctx)
    sess.set_policy(modes["on"])
    sess.run()
    n_prelaunched = psv.psv_debug_last_step_prelaunches(sess.ctx)     # consumers the `on` step launched into their windows
    prelaunch_active = n_prelaunched > 0
    vector_path = w.weight_layout != "tiled" and (w.batch == 1 or (w.batch == 2 and w.hidden <= 4096))
    prelaunched_ops = ("qkv", "gate_up") if vector_path else ("gate_up",)      # matrix-core path: the gate/up GEMM only

    us = {k: v * 1e3 / L for k, v in ms.items()}
    win = sum(w.window_us)
    layer_bytes = stats["weight_bytes_per_layer"] + stats["kv_bytes_per_layer"]
    eff = {k: layer_bytes / max(1e-9, (v - win)) / 1e3 for k, v in us.items()}          # GB/s outside the windows

    # per-operator kernel durations (events attached to the kernel dispatches: end of the previous kernel on the stream
    # to the end of this one), prefetch off and on; the dominant kernel -- gate/up projection + SwiGLU, HBM-bound --
    # carries the roofline entry
    qkv_rows = (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim
    wb = 1 if w.weight_format == "int8" else 2          # bytes per weight
    op_bytes = {"qkv": wb * qkv_rows * w.hidden, "attn": stats["kv_bytes_per_layer"],
                "o": wb * w.hidden * w.n_q_heads * w.head_dim, "gate_up": wb * 2 * w.ffn * w.hidden,
                "down": wb * w.hidden * w.ffn}
    op_ids = {"qkv": psv.PSV_OP_QKV, "attn": psv.PSV_OP_ATTN, "o": psv.PSV_OP_O, "gate_up": psv.PSV_OP_GATE,
              "down": psv.PSV_OP_DOWN}
    n_prof = max(3, min(a.steps, 10))
    kernels = {}
    if a.calibrate_copy_mb > 0:
        nb = a.calibrate_copy_mb << 20
        src = torch.empty(nb, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        psv.psv_copy_bytes(dst, src, nb, sess.main)
        sess.sync()
    path = psv.psv_debug_last_step_path(sess.ctx)   # 0 one kernel per operator, 1 one per segment, 2 one per step
    fused_on = path >= 1
    whole_step = path == 2                          # the step is one kernel: no per-operator table
    step_kernel = None
    if whole_step:
        # the kernel's own duration without windows, prefetch off: all the step's bytes over that time is its bandwidth
        sess.set_policy(modes["off"])
        sess.set_windows(0.0, 0.0)
        sess.run()
        t_k, n_k = profile_op(sess, psv.PSV_OP_QKV, n_prof)
        sess.set_windows(*w.window_us)
        step_kernel = {"us": round(t_k, 3), "launches": n_k, "bytes": int(layer_bytes * L),
                       "gbps": round(layer_bytes * L / t_k / 1e3, 1), "us_per_layer": round(t_k / L, 3)}
    for mode_name in ("off", "on"):
        if whole_step or (a.skip_kernel_table and mode_name == "on"):
            break
        sess.set_policy(modes[mode_name])
        for name, op in op_ids.items():
            t, n = profile_op(sess, op, n_prof)
            k = kernels.setdefault(name, {"bytes": op_bytes[name]})
            k["launches"] = n
            if n == 0:                      # fused into the kernel of the operator that opens its segment
                k["us_" + mode_name] = None
                continue
            k["us_" + mode_name] = round(t, 3)
            launched_into_window = mode_name == "on" and prelaunch_active and name in prelaunched_ops
            if launched_into_window:
                # its weights were requested while the window ran: the time left after the window is no bandwidth figure
                k["us_after_window_on"] = round(t, 3)
                del k["us_on"]
            elif not fused_on:
                k["gbps_" + mode_name] = round(op_bytes[name] / t / 1e3, 1)
    if whole_step:
        gate_us, gate_n, gate_bytes = step_kernel["us"], step_kernel["launches"], step_kernel["bytes"]
    else:
        gate_us, gate_n = kernels["gate_up"]["us_off"], kernels["gate_up"]["launches"]
        gate_bytes = op_bytes["gate_up"] + (op_bytes["down"] if fused_on and kernels["down"]["launches"] == 0 else 0)
    achieved = gate_bytes / gate_us / 1e3
    traffic, traffic_src = (stored_traffic(w.name, "mlp_fused" if fused_on else "gate_up")
                            if (a.format == "bf16" and not whole_step) else (None, None))

    out = {
        "metric": "decode_step_latency_us_per_layer_prefetch_on",
        "value": round(us["on"], 3),
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms["on"], 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if a.format == "bf16" else "%s (storage: %s weights, %s KV; fp32 accumulation)" % (
            a.format, w.weight_format, w.kv_format),
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, hidden %d, %d q / %d kv heads x 128, ffn %d, batch %d, context %d, %s KV, "
                               "%s weights, windows %g/%g us" % (w.name, L, w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn, w.batch,
                                                      w.context, "paged" if w.paged else "contiguous",
                                                      "tiled" if w.weight_layout == "tiled" else "row-major", *w.window_us),
                   "prefetch_budget_mb": a.budget_mb, "cu_budget": a.cu_budget, "chunk_mb": a.chunk_mb,
                   "partial": a.partial, "join": a.join, "prelaunch": a.prelaunch, "prelaunch_active": prelaunch_active, "prelaunched_per_step": n_prelaunched,
                   "targets": a.targets, "fused_kernels": "by shape" if a.fused < 0 else int(a.fused), "kernel_path": path, "streams_overlap": bool(sess.overlap),
                   "attn_tokens_per_workgroup": attn_chunk if a.tune else "default"},
        "us_per_layer_prefetch_off": round(us["off"], 3),
        "us_per_layer_cache_only": round(us["cache_only"], 3),
        "prefetch_speedup": round(us["off"] / us["on"], 4),
        "speedup_cache_only": round(us["off"] / us["cache_only"], 4),          # the paper's method alone
        "speedup_prelaunch": round(us["off"] / us["on"], 4),                   # with the first consumer launched into the window
        "step_us_per_layer": {k: hot[k] for k in ("off", "cache_only", "on")},    # per-step event pairs: median, p10, p90
        "on_off_bit_identical": identical,
        "layer_bytes": layer_bytes,
        "planned_prefetch_bytes_per_step": stats["planned_prefetch_bytes"],
        "effective_hbm_gbps_outside_windows": {"prefetch_off": round(eff["off"], 1), "prefetch_on": round(eff["on"], 1),
                                                "peak": HBM_PEAK_GBPS,
                                                "frac_off": round(eff["off"] / HBM_PEAK_GBPS, 4),
                                                "frac_on": round(eff["on"] / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "kernel": ("the whole step as one kernel, windows of 0 us, prefetch off" if whole_step else
                                                "gate/up + SwiGLU + down, fused (prefetch off)" if gate_bytes != op_bytes["gate_up"]
                                                else "gate/up projection + SwiGLU (prefetch off)"),
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_source": ("stored: %s (rocprofv3 counters of an earlier run of this kernel; not measured by this run)"
                                        % traffic_src) if traffic is not None else None,
                     "bytes_per_launch": gate_bytes, "avg_us": round(gate_us, 3), "launches": gate_n},
    }
    if cold:
        out["cold_cache"] = {"rule": "%d MiB streamed through the GPU before every timed step, outside the timed region"
                                     % (FLUSH_BYTES >> 20),
                             "step_us_per_layer": cold,
                             "speedup_cache_only": round(cold["off"]["median"] / cold["cache_only"]["median"], 4),
                             "speedup_prelaunch": round(cold["off"]["median"] / cold["on"]["median"], 4)}
        out["hot_cache_note"] = "back-to-back steps of this workload run from the memory-side cache: step_us_per_layer and value are hot numbers"
    out["kernels"] = kernels
    if step_kernel is not None:
        out["step_kernel"] = step_kernel
    if not a.no_cpu_baseline:
        # whole step when a layer is cheap; otherwise the first layers whose oracle cost is ~10-30 s
        n_cpu = a.cpu_layers or max(1, min(L, int(6.0e10 / max(1, (stats["weight_bytes_per_layer"] +
                                                                   8 * stats["kv_bytes_per_layer"]) * w.batch))))
        cpu_us, n_done, reps, threads = cpu_baseline(sess, n_cpu)
        out["cpu_baseline"] = {"value": round(cpu_us, 1), "unit": "us/layer", "cores": threads, "kind": "oracle",
                               "sample": "fp64 C oracle, first %d of %d layers of the same workload, %d repetitions"
                                         % (n_done, L, reps)}
    sess.close()
    del sess, flush
    torch.cuda.empty_cache()
    if path == 1 and a.fused < 0:
        # the library chose the per-segment kernels for this shape: the record also carries the per-operator kernels
        out["per_operator_kernels"] = per_operator_leg(w, layers, max(10, min(a.steps, 50)), min(a.warmup, 10), a.seed, modes,
                                                       op_bytes["gate_up"])
        best_off = min(out["us_per_layer_prefetch_off"], out["per_operator_kernels"]["us_per_layer"]["off"])
        out["speedup_vs_fastest_off"] = round(best_off / out["value"], 4)
    others = [n for n in a.also.split(",") if n and n != a.workload]
    if others and a.format == "bf16" and a.fused < 0 and a.window_us is None:
        out["other_workloads"] = {n: other_workload(n, a.also_layers, max(10, min(a.steps, 50)), min(a.warmup, 10), a.seed)
                                  for n in others}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
