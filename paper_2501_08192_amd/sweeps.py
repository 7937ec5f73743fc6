"""Measurement drivers around the C-ABI library (GPU needed): the batch x context speedup map on 70B-shaped
shards and the window / budget / chunk / workgroup sweeps on one of the benchmark workloads.  They only set
policies, run decode steps and time them; every step of the path runs in the library's kernels.

    python -m paper_2501_08192_amd.sweeps map tp4            # Section 4, "Impact of batch size and sequence length"
    python -m paper_2501_08192_amd.sweeps map tp8
    python -m paper_2501_08192_amd.sweeps sweep c5 --layers 4 --which window,budget,chunk,cu,targets
    python -m paper_2501_08192_amd.sweeps calibrate          # fits the analytic model's constants -> machine_mi355x.json
    python -m paper_2501_08192_amd.sweeps record             # measured rows the model is tested against -> tests/golden/

The map stands in for the paper's sweep over batch size and sequence length (its Figure on the speedup across
batch sizes and sequence lengths); the sweeps for its remark that the prefetch should take about as long as the
allreduce it hides behind (appendix on the optimal cache size).
"""
import argparse
import json
import os
import time

import torch

from . import binding as psv
from . import model, synth
from .harness import Session, default_policy

MB = 1 << 20
SHAPES = {                      # hidden, local q heads, local kv heads, local FFN width
    "tp4": (8192, 16, 2, 7168),  # 70B-shaped model on 4 devices: 2 local kv heads
    "tp8": (8192, 8, 1, 3584),   # ... on 8 devices: 1 local kv head
}


def timed(sess, n_layers, steps=20, warmup=5, reps=3):
    """Median over `reps` of the time per layer of `steps` back-to-back decode steps (us)."""
    for _ in range(warmup):
        sess.step()
    sess.sync()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        t0 = time.perf_counter()
        for _ in range(steps):
            sess.step()
        sess.sync()
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e6 / steps / n_layers)
    return sorted(ts)[len(ts) // 2]


def speed_map(shape, batches, contexts, layers=4, window=20.0, out=print, kv_layout="head", weight_layout="row"):
    """off / on us per layer and speedup for every (batch, context), beside the analytic model's prediction.
    The budget is the one the model picks; the rest of the policy is bench.py's default."""
    hidden, nq, nkv, ffn = SHAPES[shape]
    mach = model.Machine.load()
    out("shape %s: hidden %d, %d q / %d kv heads, ffn %d, windows %g us, %d layers materialised, %s-major KV, %s weights"
        % (shape, hidden, nq, nkv, ffn, window, layers, kv_layout, "tiled" if weight_layout == "tiled" else "row-major"))
    out("%5s %7s | %9s %9s %8s | %9s %9s %8s | budget" % ("batch", "context", "off", "on", "speedup", "m.off", "m.on", "m.spd"))
    rows = []
    for B in batches:
        for T in contexts:
            w = synth.Workload("map", 80, hidden, nq, nkv, 128, ffn, B, T, False, (window, window), kv_layout=kv_layout,
                               weight_layout=weight_layout)
            if w.kv_bytes_per_layer * layers > 60e9:
                continue
            b = model.op_bytes(hidden, nq, nkv, ffn, B, T, weight_layout=weight_layout)
            path = model.path_of(B, hidden, weight_layout)
            hold = model.mm_hold(B, hidden, ffn, weight_layout=weight_layout) if path != "vec" else 0.0
            budget = model.best_budget(b, (window, window), mach, path=path)
            with Session(w, layers=list(range(layers))) as s:
                s.set_policy(psv.prefetch_policy(mode=0))
                x_off = s.run().clone()
                off = timed(s, layers)
                s.set_policy(default_policy(w, budget_bytes=int(budget), partial=1))
                x_on = s.run().clone()
                on = timed(s, layers)
                if not torch.equal(x_off, x_on):
                    raise AssertionError("prefetch on/off outputs differ at batch %d context %d" % (B, T))
            m_off = model.layer_time(b, (window, window), mach, 0.0, path=path)
            m_on = model.layer_time(b, (window, window), mach, budget, prelaunch=True, path=path, hold_mm=hold)
            rows.append((B, T, off, on, m_off, m_on, budget))
            out("%5d %7d | %9.1f %9.1f %8.3f | %9.1f %9.1f %8.3f | %d MB"
                % (B, T, off, on, off / on, m_off, m_on, m_off / m_on, budget / 1e6))
            torch.cuda.empty_cache()
    return rows


def policy_sweeps(name, layers=4, steps=30, which=("window", "budget", "chunk", "cu", "targets"), out=print):
    """Speedup of one benchmark workload as the window, the budget C, the chunk size, the prefetch kernel's
    workgroup budget and the targets vary (all other policy fields fixed, no pre-launched consumers: the sweeps
    isolate the cache prefetch)."""
    w = synth.WORKLOADS[name]
    with Session(w, layers=list(range(layers))) as s:
        def run(win, budget_mb, chunk_mb=0, cu=256, partial=1, targets=3, join=0):
            s.set_windows(win, win)
            s.set_policy(psv.prefetch_policy(mode=0))
            off = timed(s, layers, steps)
            s.set_policy(psv.prefetch_policy(mode=1, targets=targets, budget_bytes=int(budget_mb * MB),
                                             chunk_bytes=int(chunk_mb * MB), cu_budget=cu, partial=partial, join=join))
            on = timed(s, layers, steps)
            planned = psv.psv_get_stats(s.ctx)["planned_prefetch_bytes"] / max(1, w.n_layers) / 1e6   # the plan spans all layers
            out("win %5.1f budget %6.1f MB chunk %5.1f MB cu %4d targets %d join %d : off %8.2f on %8.2f us/layer "
                "speedup %.4f  planned %.1f MB/layer" % (win, budget_mb, chunk_mb, cu, targets, join, off, on, off / on, planned))
            return off / on

        base_win = w.window_us[0]
        if "window" in which:
            out("== window sweep (budget 192 MB)")
            for win in (0.0, 5.0, 10.0, 20.0, 50.0):
                run(win, 192)
        if "budget" in which:
            out("== budget sweep (window %g and 50 us)" % base_win)
            for win in (base_win, 50.0):
                for b in (8, 16, 32, 64, 128, 192, 256, 384, 600):
                    run(win, b)
        if "chunk" in which:
            out("== chunk sweep (window 50 us, budget 256 MB)")
            for c in (0, 1, 2, 4, 8, 16, 32, 64):
                run(50.0, 256, chunk_mb=c)
        if "cu" in which:
            out("== workgroup budget sweep (window %g us, budget 64 MB)" % base_win)
            for cu in (16, 32, 64, 128, 256, 512, 1024):
                run(base_win, 64, cu=cu)
        if "targets" in which:
            out("== targets (window %g us, budget 192 MB)" % base_win)
            for t in (1, 2, 3):
                run(base_win, 192, targets=t)
            run(base_win, 192, join=1)


# ---- calibration of the analytic model ---------------------------------------------------------------------

# Shapes the constants are fitted on: none of them is a benchmark workload or a cell of the speedup map.
CAL_SHAPES = {   # hidden, q heads, kv heads, ffn, batch, context, weight layout
    "v1": (2048, 16, 2, 5632, 1, 1024, "row"), "v2": (8192, 8, 1, 3584, 1, 512, "row"), "v3": (4096, 8, 2, 2816, 1, 3072, "row"),
    "m1": (2048, 16, 2, 5632, 8, 2048, "row"), "m2": (8192, 8, 1, 3584, 12, 2048, "row"), "m3": (4096, 8, 2, 2816, 48, 4096, "row"),
    "m4": (8192, 8, 1, 3584, 24, 12288, "row"),     # a KV-dominated layer (151 MB of cache): sets the attention's streaming rate
    "m5": (4096, 8, 2, 2816, 6, 2048, "row"),
    "m6": (8192, 8, 1, 3584, 20, 40960, "row"),      # 419 MB of cache per layer: the attention at its streaming rate
    "t1": (2048, 16, 2, 5632, 8, 2048, "tiled"), "t2": (8192, 8, 1, 3584, 12, 2048, "tiled"), "t3": (4096, 8, 2, 2816, 48, 4096, "tiled"),
    "t4": (8192, 8, 1, 3584, 24, 12288, "tiled"), "t5": (4096, 8, 2, 2816, 6, 2048, "tiled"),
}
OPS = {"qkv": psv.PSV_OP_QKV, "attn": psv.PSV_OP_ATTN, "o": psv.PSV_OP_O, "gate_up": psv.PSV_OP_GATE, "down": psv.PSV_OP_DOWN}


def op_times(sess, steps=8):
    out = {}
    for name, op in OPS.items():
        psv.psv_set_profile_op(sess.ctx, op)
        for _ in range(steps):
            sess.step()
        ms, n = psv.psv_get_profile(sess.ctx)
        out[name] = ms * 1e3 / max(1, n)
    psv.psv_set_profile_op(sess.ctx, -1)
    return out


def slope_through(points, icpt):
    """bytes per us of t = icpt + bytes / bw with the intercept given (least squares)."""
    num = sum(p[0] * p[0] for p in points)
    den = sum(p[0] * (p[1] - icpt) for p in points)
    return num / den


def calibrate(path, window=50.0, layers=4, out=print):
    pts = {"vec": [], "vec_hit": [], "mm": [], "mm_hit": [], "mmt": [], "mmt_hit": [], "attn": [], "attn_hit": [], "pre": [], "pre_mm": []}
    raw, resid = {}, {}
    big = 192 * MB
    for name, (H, nq, nkv, F, B, T, layout) in CAL_SHAPES.items():
        w = synth.Workload(name, 80, H, nq, nkv, 128, F, B, T, False, (window, window), weight_layout=layout)
        b = model.op_bytes(H, nq, nkv, F, B, T, weight_layout=layout)
        nb = {"qkv": b["qkv"], "attn": b["attn"], "o": b["o"], "gate_up": b["gate"] + b["up"], "down": b["down"]}
        part = {op: b["p_" + op] for op in ("qkv", "o", "gate_up", "down")}      # split-K partials: traffic of the projection too
        cls = model.path_of(B, H, layout)
        hold = model.mm_hold(B, H, F, weight_layout=layout) if cls != "vec" else 0.0
        with Session(w, layers=list(range(layers))) as s:
            # windows long enough for the whole budget to arrive inside them; whole-layer timing first (it warms up)
            s.set_policy(psv.prefetch_policy(mode=0))
            off = timed(s, layers)
            off_ops = op_times(s)
            s.set_policy(default_policy(w, budget_bytes=big, prelaunch=0, partial=1))
            hit = timed(s, layers)
            hit_ops = op_times(s)
            pre_ops = None
            if cls == "vec" or hold > 0:
                s.set_policy(default_policy(w, budget_bytes=big, partial=1))
                timed(s, layers, steps=5, reps=1)
                if (psv.psv_debug_last_step_prelaunches(s.ctx) > 0) != (cls == "vec" or hold > 0):
                    raise AssertionError("%s: the model's rule for launching into windows is not the library's" % name)
                pre_ops = op_times(s)
        raw[name] = {"bytes": nb, "us_off": off_ops, "us_cache_only": hit_ops, "us_prelaunch": pre_ops, "layer_off": off, "layer_cache_only": hit}
        for op in ("qkv", "o", "gate_up", "down"):
            pts[cls].append((nb[op] + part[op], off_ops[op]))
            pts[cls + "_hit"].append((nb[op] + part[op], hit_ops[op]))
        pts["attn"].append((nb["attn"], off_ops["attn"]))
        pts["attn_hit"].append((nb["attn"], hit_ops["attn"]))
        if pre_ops and cls == "vec":
            pts["pre"] += [(nb["qkv"], pre_ops["qkv"]), (nb["gate_up"], pre_ops["gate_up"])]
        elif pre_ops:       # (class, bytes it does not hold, us after the window) of the gate/up GEMM launched into its window
            pts["pre_mm"].append((cls, (1.0 - hold) * nb["gate_up"] + part["gate_up"], pre_ops["gate_up"]))
        resid[name] = off - sum(off_ops.values()) - 2 * window       # what the five operator kernels and the windows leave
        out("%s: layer off %.1f cache-only %.1f; ops off %s" % (name, off, hit, {k: round(v, 2) for k, v in off_ops.items()}))
        torch.cuda.empty_cache()
    d = model.Machine()
    t_fixed, bw_hbm = model.fit_line(pts["vec"])
    t_fixed_mm, bw_mm = model.fit_line(pts["mm"])
    t_fixed_mmt, bw_mmt = model.fit_line(pts["mmt"])
    bw_mm_cache, bw_mmt_cache = slope_through(pts["mm_hit"], t_fixed_mm), slope_through(pts["mmt_hit"], t_fixed_mmt)
    t_fixed_attn, bw_attn = model.fit_line(pts["attn"])
    w_extra = sum(resid[n] for n in ("v1", "v2", "v3")) / 3 / 2      # per window: its kernel overruns the request, plus its dispatch gap
    mm_names = [n for n in CAL_SHAPES if n[0] in "mt"]
    t_small = sum(resid[n] - 2 * w_extra for n in mm_names) / len(mm_names) / d.n_small
    # a projection launched into its window: what is left after the window against the bytes it holds
    pre_pts = [(min(nb, d.reg_bytes), us - max(0.0, nb - d.reg_bytes) / bw_hbm) for nb, us in pts["pre"]]
    try:
        t_post, bw_reg = model.fit_line(pre_pts)
    except ValueError:      # no measurable slope: working through the held weights costs nothing beyond the fixed part
        t_post, bw_reg = sum(us for _, us in pre_pts) / len(pre_pts), 1e9
    # the gate/up GEMM launched into its window: what is left after the window beyond streaming the part it does not hold
    # (from the cache: the calibration budget covers the whole matrix)
    t_post_mm = sum(us - rest / (bw_mmt_cache if cls == "mmt" else bw_mm_cache) for cls, rest, us in pts["pre_mm"]) / len(pts["pre_mm"])
    # the prefetch kernel alone on cold regions of three sizes: 1 GiB is read through the GPU before every sample (read, not
    # written: dirty lines in the memory-side cache would have to be written back under the measurement and halve the rate),
    # the fastest of three samples per size counts
    pf = []
    stream = torch.cuda.Stream()
    flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
    for mb in (16, 64, 192):
        buf = torch.empty(mb * MB, dtype=torch.uint8, device="cuda").random_()
        best = None
        for _ in range(4):
            torch.cuda.synchronize()
            psv.psv_prefetch_region(flush, 1 << 30, 256, stream)
            psv.psv_prefetch_region(flush, 1 << 30, 256, stream)      # twice: the first pass writes back what was dirty
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            psv.psv_prefetch_region(buf, mb * MB, 256, stream)
            e1.record(stream)
            stream.synchronize()
            us = e0.elapsed_time(e1) * 1e3
            best = us if best is None else min(best, us)
        pf.append((mb * MB, best))
        del buf
    del flush
    _, bw_prefetch = model.fit_line(pf)
    mach = {"t_fixed": t_fixed, "bw_hbm": bw_hbm, "bw_cache": slope_through(pts["vec_hit"], t_fixed),
            "t_fixed_mm": t_fixed_mm, "bw_mm": bw_mm, "bw_mm_cache": bw_mm_cache,
            "t_fixed_mmt": t_fixed_mmt, "bw_mmt": bw_mmt, "bw_mmt_cache": bw_mmt_cache, "t_post_mm": t_post_mm,
            "t_fixed_attn": t_fixed_attn, "bw_attn": bw_attn, "bw_attn_cache": slope_through(pts["attn_hit"], t_fixed_attn),
            "t_small": t_small, "t_window_extra": w_extra, "bw_prefetch": bw_prefetch, "t_post": t_post, "bw_reg": bw_reg}
    mach = {k: round(float(v), 4) for k, v in mach.items()}
    json.dump({"command": "python -m paper_2501_08192_amd.sweeps calibrate", "shapes": CAL_SHAPES, "window_us": window,
               "machine": mach, "measured": raw, "prefetch_kernel": pf}, open(path, "w"), indent=1, sort_keys=True)
    out("machine: %s" % mach)
    return mach


# ---- measured records the model is tested against ----------------------------------------------------------

def record(path, layers=4, out=print):
    """us per layer of the five benchmark workloads (their first layers) and of cells of the speedup map, prefetch off,
    cache only and with the default policy, plus the c5 budget sweep at two windows: the rows tests/test_model.py holds
    the analytic model to."""
    rows = []

    def measure(name, w, n_layers, budget=None):
        with Session(w, layers=list(range(n_layers))) as s:
            kw = {} if budget is None else {"budget_bytes": int(budget)}
            s.set_policy(psv.prefetch_policy(mode=0))
            off = timed(s, n_layers)
            s.set_policy(default_policy(w, prelaunch=0, **kw))
            cache = timed(s, n_layers)
            pol = default_policy(w, **kw)
            s.set_policy(pol)
            pre = timed(s, n_layers)
            kernel_path = psv.psv_debug_last_step_path(s.ctx)      # 0: one kernel per operator, 1: one per segment
            prelaunched = psv.psv_debug_last_step_prelaunches(s.ctx)
        rows.append({"name": name, "weight_layout": w.weight_layout, "prelaunched": prelaunched, "hidden": w.hidden, "n_q": w.n_q_heads, "n_kv": w.n_kv_heads, "ffn": w.ffn, "batch": w.batch,
                     "context": w.context, "windows": list(w.window_us), "budget": int(pol.budget_bytes), "partial": int(pol.partial),
                     "us_off": round(off, 2), "us_cache_only": round(cache, 2), "us_default": round(pre, 2), "kernel_path": kernel_path})
        out(str(rows[-1]))
        torch.cuda.empty_cache()

    for name in ("c1", "c2", "c3", "c4", "c5"):
        w = synth.WORKLOADS[name]
        measure(name, w, min(layers, w.n_layers) if name != "c2" else 8)
    for shape, layout, cells in (("tp8", "row", ((1, 1024), (1, 16384), (4, 4096), (16, 4096), (64, 4096), (16, 16384))),
                                 ("tp4", "row", ((1, 4096), (16, 4096), (64, 16384))),
                                 ("tp8", "tiled", ((4, 4096), (8, 16384), (16, 4096))), ("tp4", "tiled", ((8, 4096),))):
        H, nq, nkv, F = SHAPES[shape]
        for B, T in cells:
            measure("%s_b%d_t%d%s" % (shape, B, T, "_tiled" if layout == "tiled" else ""),
                    synth.Workload("map", 80, H, nq, nkv, 128, F, B, T, False, (20.0, 20.0), weight_layout=layout), 4, budget=96e6)
    sweep = []
    w = synth.WORKLOADS["c5"]
    with Session(w, layers=list(range(layers))) as s:
        for win in (20.0, 50.0):
            s.set_windows(win, win)
            s.set_policy(psv.prefetch_policy(mode=0))
            off = timed(s, layers)
            for mb in (16, 64, 128, 192, 256, 384, 600):
                s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=mb * MB, cu_budget=256, partial=1))
                on = timed(s, layers)
                sweep.append({"window": win, "budget_mb": mb, "us_off": round(off, 2), "us_on": round(on, 2)})
                out(str(sweep[-1]))
    json.dump({"command": "python -m paper_2501_08192_amd.sweeps record", "rows": rows, "c5_budget_sweep": sweep},
              open(path, "w"), indent=1)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    m = sub.add_parser("map")
    m.add_argument("shape", choices=sorted(SHAPES))
    m.add_argument("--batches", default="1,4,16,64")
    m.add_argument("--contexts", default="1024,4096,16384,65536")
    m.add_argument("--layers", type=int, default=4,
                   help="layers materialised; an even count, so that every window that can be launched into is (the chain has to end on the main stream)")
    m.add_argument("--window", type=float, default=20.0)
    m.add_argument("--kv-layout", default="head", choices=["head", "token"],
                   help="token: both pools [block, token, kv head, channel] -- one head's reads are strided when the shard has "
                        "several local kv heads")
    m.add_argument("--weight-layout", default="row", choices=["row", "tiled"],
                   help="tiled: projection matrices in the order of the matrix-core projections (which then run at every batch)")
    sw = sub.add_parser("sweep")
    sw.add_argument("workload", choices=sorted(synth.WORKLOADS))
    sw.add_argument("--layers", type=int, default=4)
    sw.add_argument("--steps", type=int, default=30)
    sw.add_argument("--which", default="window,budget,chunk,cu,targets")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    ca = sub.add_parser("calibrate")
    ca.add_argument("--out", default=model.MACHINE_FILE)
    rc = sub.add_parser("record")
    rc.add_argument("--out", default=os.path.join(root, "tests", "golden", "measured_mi355x.json"))
    a = ap.parse_args(argv)

    def out(line):
        print(line, flush=True)

    if a.cmd == "calibrate":
        calibrate(a.out, out=out)
    elif a.cmd == "record":
        record(a.out, out=out)
    elif a.cmd == "map":
        speed_map(a.shape, [int(x) for x in a.batches.split(",")], [int(x) for x in a.contexts.split(",")],
                  a.layers, a.window, out, kv_layout=a.kv_layout, weight_layout=a.weight_layout)
    else:
        policy_sweeps(a.workload, a.layers, a.steps, tuple(a.which.split(",")), out)


if __name__ == "__main__":
    main()
