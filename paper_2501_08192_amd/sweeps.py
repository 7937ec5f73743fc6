"""Measurement drivers around the C-ABI library (GPU needed): the batch x context speedup map on 70B-shaped
shards and the window / budget / chunk / workgroup sweeps on one of the benchmark workloads.  They only set
policies, run decode steps and time them; every step of the path runs in the library's kernels.

    python -m paper_2501_08192_amd.sweeps map tp4            # Section 4, "Impact of batch size and sequence length"
    python -m paper_2501_08192_amd.sweeps map tp8
    python -m paper_2501_08192_amd.sweeps sweep c5 --layers 4 --which window,budget,chunk,cu,targets

The map stands in for the paper's sweep over batch size and sequence length (its Figure on the speedup across
batch sizes and sequence lengths); the sweeps for its remark that the prefetch should take about as long as the
allreduce it hides behind (appendix on the optimal cache size).
"""
import argparse
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


def speed_map(shape, batches, contexts, layers=3, window=20.0, out=print, kv_layout="head"):
    """off / on us per layer and speedup for every (batch, context), beside the analytic model's prediction.
    The budget is the one the model picks; the rest of the policy is bench.py's default."""
    hidden, nq, nkv, ffn = SHAPES[shape]
    mach = model.Machine()
    out("shape %s: hidden %d, %d q / %d kv heads, ffn %d, windows %g us, %d layers materialised, %s-major KV"
        % (shape, hidden, nq, nkv, ffn, window, layers, kv_layout))
    out("%5s %7s | %9s %9s %8s | %9s %9s %8s | budget" % ("batch", "context", "off", "on", "speedup", "m.off", "m.on", "m.spd"))
    rows = []
    for B in batches:
        for T in contexts:
            w = synth.Workload("map", 80, hidden, nq, nkv, 128, ffn, B, T, False, (window, window), kv_layout=kv_layout)
            if w.kv_bytes_per_layer * layers > 60e9:
                continue
            b = model.op_bytes(hidden, nq, nkv, ffn, B, T)
            budget = model.best_budget(b, (window, window), mach)
            with Session(w, layers=list(range(layers))) as s:
                s.set_policy(psv.prefetch_policy(mode=0))
                x_off = s.run().clone()
                off = timed(s, layers)
                s.set_policy(default_policy(w, budget_bytes=int(budget), partial=1))
                x_on = s.run().clone()
                on = timed(s, layers)
                if not torch.equal(x_off, x_on):
                    raise AssertionError("prefetch on/off outputs differ at batch %d context %d" % (B, T))
            m_off = model.layer_time(b, (window, window), mach, 0.0)
            m_on = model.layer_time(b, (window, window), mach, budget)
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


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    m = sub.add_parser("map")
    m.add_argument("shape", choices=sorted(SHAPES))
    m.add_argument("--batches", default="1,4,16,64")
    m.add_argument("--contexts", default="1024,4096,16384,65536")
    m.add_argument("--layers", type=int, default=3)
    m.add_argument("--window", type=float, default=20.0)
    m.add_argument("--kv-layout", default="head", choices=["head", "token"],
                   help="token: both pools [block, token, kv head, channel] -- one head's reads are strided when the shard has "
                        "several local kv heads")
    sw = sub.add_parser("sweep")
    sw.add_argument("workload", choices=sorted(synth.WORKLOADS))
    sw.add_argument("--layers", type=int, default=4)
    sw.add_argument("--steps", type=int, default=30)
    sw.add_argument("--which", default="window,budget,chunk,cu,targets")
    a = ap.parse_args(argv)

    def out(line):
        print(line, flush=True)

    if a.cmd == "map":
        speed_map(a.shape, [int(x) for x in a.batches.split(",")], [int(x) for x in a.contexts.split(",")],
                  a.layers, a.window, out, kv_layout=a.kv_layout)
    else:
        policy_sweeps(a.workload, a.layers, a.steps, tuple(a.which.split(",")), out)


if __name__ == "__main__":
    main()
