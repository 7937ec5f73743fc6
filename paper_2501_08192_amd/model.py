"""Analytic latency model of one decode layer with and without prefetching, in the spirit of the paper's
design-space model (Section 5, "Performance & cost model": memory time linear in bytes over the bandwidth of
the level that serves them, communication as a fixed latency), re-parameterised for MI355X.  Pure Python; used to
predict the speedup map and to pick a prefetch budget.

Per kernel:  t = t_fixed + hit_bytes / bw_cache + miss_bytes / bw_hbm, with one (t_fixed, bw_hbm, bw_cache) triple
per kernel class: the vector-ALU projections of batch 1-2, the matrix-core projections of larger batches (on row-major
and on tiled weights), the decode attention, and the small kernels the matrix-core path adds (residual sums, split-K
reductions, attention merge).
Per window:  t = max(window, t_fork + prefetch_bytes / bw_prefetch)   (the prefetch may outlast the window),
and whatever part of a prefetch is still running after the window competes with its consumer for HBM.

The constants are not fitted to the workloads the model is used to predict: `sweeps.py calibrate` measures the
per-operator kernel times of a dozen calibration shapes that are none of the benchmark workloads nor cells of the
speedup map, fits the triples by least squares and writes machine_mi355x.json next to this file; Machine.load()
reads it.  tests/test_model.py holds the model to the measured records in tests/golden/measured_mi355x.json
(written by `sweeps.py record`) within a stated tolerance.
"""
import json
import os
from dataclasses import dataclass, fields, replace

HERE = os.path.dirname(os.path.abspath(__file__))
MACHINE_FILE = os.path.join(HERE, "machine_mi355x.json")


@dataclass(frozen=True)
class Machine:
    # vector-ALU projections (batch 1; batch 2 up to hidden 4096)
    t_fixed: float = 3.5         # us per dependent kernel: dispatch gap, first byte, reduction, drain
    bw_hbm: float = 4.5e6        # bytes/us streamed from HBM
    bw_cache: float = 5.5e6      # bytes/us streamed when the bytes were prefetched into the Infinity Cache
    # matrix-core projections (split-K GEMM)
    t_fixed_mm: float = 4.0
    bw_mm: float = 4.2e6
    bw_mm_cache: float = 5.0e6
    # ... on tiled weights
    t_fixed_mmt: float = 4.0
    bw_mmt: float = 4.9e6
    bw_mmt_cache: float = 5.6e6
    # decode attention
    t_fixed_attn: float = 4.5
    bw_attn: float = 4.8e6
    bw_attn_cache: float = 5.5e6
    # small kernels of the matrix-core path (2 residual sums, 2 split-K reductions, attention merge)
    t_small: float = 3.7
    n_small: int = 5
    # prefetch kernel
    bw_prefetch: float = 5.0e6   # bytes/us with >= 128 workgroups
    t_fork: float = 2.5          # us from window start to the first prefetch load (gate kernel + dispatch)
    t_window_extra: float = 0.8  # us a window costs beyond its length (the stand-in kernel's overrun and its dispatch gap)
    cache_bytes: float = 192e6   # usable part of the 256 MB Infinity Cache
    # a projection launched into its window (policy.prelaunch, vector path)
    reg_bytes: float = 32e6      # weights its first pass holds in registers
    t_post: float = 3.0          # us it still needs after the window (poll, activations, reduce, drain)
    bw_reg: float = 24e6         # bytes/us at which it works through the weights it holds
    # the gate/up GEMM launched into its window (policy.prelaunch, matrix-core path, batch <= 32)
    t_post_mm: float = 6.0       # us after the window until it has worked through what it holds, the residual kernel it
                                 #   waits for included

    @classmethod
    def load(cls, path=MACHINE_FILE):
        """The calibrated constants if the calibration file exists, else the defaults above."""
        try:
            data = json.load(open(path))
        except OSError:
            return cls()
        names = {f.name for f in fields(cls)}
        return replace(cls(), **{k: v for k, v in data.get("machine", {}).items() if k in names})


def path_of(batch, hidden, weight_layout="row"):
    """Which projections a step runs: "vec" (vector ALU), "mm" (matrix cores) or "mmt" (matrix cores on tiled weights,
    at every batch) -- the library's own rule."""
    if weight_layout == "tiled":
        return "mmt"
    return "vec" if batch == 1 or (batch == 2 and hidden <= 4096) else "mm"


def sk_splits(batch, n_rows, k, weight_bytes=2.0, tiled=False):
    """K splits of the split-K GEMM: the library's cost model (0.6 us per slab step, 512 resident workgroups, weights and
    partials at 4 TB/s)."""
    n_slabs = k // 64
    row_groups = (n_rows + 127) // 128
    w_bytes, part_bytes = weight_bytes * n_rows * k, 8.0 * batch * n_rows
    best, best_cost, best1, best1_cost = 1, 1e30, 0, 1e30
    ks = 1
    while ks <= 16 and ks * 2 <= n_slabs:
        spb = (n_slabs + ks - 1) // ks
        if (n_slabs + spb - 1) // spb == ks:
            rounds = (row_groups * ks + 511) // 512
            cost = rounds * spb * 0.6 + (w_bytes + ks * part_bytes) / 4.0e6
            if cost < best_cost - 1e-9:
                best, best_cost = ks, cost
            if rounds == 1 and cost < best1_cost - 1e-9:
                best1, best1_cost = ks, cost
        ks += 1
    if tiled and best1 and best1_cost <= 1.02 * best_cost:      # tiled weights: within 2 %, one round of workgroups wins
        best = best1
    return best


def mm_hold(batch, hidden, ffn, weight_format="bf16", cus=256, weight_layout="row"):
    """Fraction of the gate/up weights that the GEMM launched into its window keeps on chip, or 0.0 where the library does
    not launch it that way: its own copy of the library's rule.  Slabs kept per workgroup: bf16 weights 12 (6 if the range
    is shorter) at batch <= 16 and 8 (6) at batch 17-32; int8 weights 12 (8) at batch <= 16.  Not launched if that is
    less than a third of the range, with fewer than 128 workgroups, or with more than stay resident beside the kernel it
    waits for."""
    w8 = weight_format == "int8"
    if not (1 <= batch <= (16 if w8 else 32)) or hidden % 512 or batch * (hidden // 512) > 1024:
        return 0.0
    nb = (batch + 15) // 16
    n_rows = 2 * ffn
    splits = sk_splits(batch, n_rows, hidden, 1.0 if w8 else 2.0, weight_layout == "tiled")
    spb = (hidden // 64 + splits - 1) // splits
    grid = (n_rows + 127) // 128 * splits
    big = spb >= (12 if nb == 1 else 8)
    held = (12 if big else 8) if w8 else ((8 if big else 6) if nb == 2 else (12 if big else 6))
    if held * 3 < spb or grid < 128:
        return 0.0
    if w8 or (nb == 1 and not big):        # three resident workgroups per compute unit, a quarter of the slots kept free
        ok = grid + cus // 4 <= 3 * cus
    else:                                  # two per compute unit, the producer's waves fit beside them
        ok = grid <= 2 * cus
    return min(1.0, held / spb) if ok else 0.0


def op_bytes(hidden, n_q, n_kv, ffn, batch, context, head_dim=128, weight_format="bf16", kv_format="bf16",
             weight_layout="row"):
    """Algorithmic bytes of the operators of one layer: bf16, or the int8 formats (1 byte per weight; per cached
    token and kv head 128 code bytes + a 4-byte scale, for K and for V).  Under "p_qkv", "p_o", "p_gate_up", "p_down": the
    split-K partial results a matrix-core projection writes and its reducing kernel reads back, 8 * splits * batch * rows
    bytes (zero on the vector path) -- never prefetched, but a third of the traffic of a small projection at batch 64."""
    wb = 1 if weight_format == "int8" else 2
    kv_token = 2 * (head_dim + 4) if kv_format == "int8" else 2 * 2 * head_dim
    qkv_rows = (n_q + 2 * n_kv) * head_dim
    out = {"qkv": qkv_rows * hidden * wb, "attn": batch * context * n_kv * kv_token, "o": hidden * n_q * head_dim * wb,
           "gate": ffn * hidden * wb, "up": ffn * hidden * wb, "down": hidden * ffn * wb}
    mm = path_of(batch, hidden, weight_layout) != "vec"
    for name, rows, k in (("qkv", qkv_rows, hidden), ("o", hidden, n_q * head_dim), ("gate_up", 2 * ffn, hidden), ("down", hidden, ffn)):
        out["p_" + name] = 8.0 * sk_splits(batch, rows, k, float(wb), weight_layout == "tiled") * batch * rows if mm else 0.0
    return out


def plan_windows(b, budget):
    """Algorithm 1 with the `partial` extension on the layer chain: bytes per operator prefetched in
    window 1 (gate, up, down) and window 2 (qkv, attn, o of the next layer)."""
    out = {}
    for ops in (("gate", "up", "down"), ("qkv", "attn", "o")):
        total = 0.0
        for op in ops:
            take = min(b[op], max(0.0, budget - 1 - total))
            out[op] = take
            total += b[op]
            if total >= budget:
                break
    return out


def prelaunched(b, windows, budget):
    """Which first consumers the `prelaunch` policy launches into their window: gate/up after window 1, the next
    layer's QKV after window 2, each only if the plan hands that window the whole operator (the gate matrix for
    the pair).  Vector path; for the matrix-core paths see mm_hold and layer_time."""
    planned = plan_windows(b, budget) if budget > 0 else {}
    return {"gate_up": windows[0] > 0 and planned.get("gate", 0.0) >= b["gate"],
            "qkv": windows[1] > 0 and planned.get("qkv", 0.0) >= b["qkv"]}


def kernel_time(m: Machine, name, nbytes, hit, path="vec", extra=0.0):
    """One kernel of class `name` ("attn", or a projection on `path`) moving nbytes, `hit` of them prefetched, and
    `extra` bytes of split-K partial results (matrix-core paths)."""
    if name == "attn":
        return m.t_fixed_attn + hit / m.bw_attn_cache + (nbytes - hit) / m.bw_attn
    if path == "mm":
        return m.t_fixed_mm + hit / m.bw_mm_cache + (nbytes - hit + extra) / m.bw_mm
    if path == "mmt":
        return m.t_fixed_mmt + hit / m.bw_mmt_cache + (nbytes - hit + extra) / m.bw_mmt
    return m.t_fixed + hit / m.bw_cache + (nbytes - hit) / m.bw_hbm


def layer_time(b, windows, m: Machine, budget=0.0, prelaunch=False, path="vec", hold_mm=0.0):
    """us per layer.  budget = 0: prefetch off.  A window of 0 us launches no prefetch; a window's plan larger
    than the cache keeps only cache_bytes / planned of itself resident.  prelaunch (vector path): the first consumer
    of a window that the plan covers whole is launched into the window; it is not prefetched a second time, holds
    up to reg_bytes of its weights in registers when the window ends and streams the rest.  prelaunch (matrix-core
    paths, hold_mm = mm_hold(...) > 0): the gate/up GEMM is launched into window 1 if the plan gives it anything, keeps
    hold_mm of its weights on chip and streams the rest; the residual kernel ahead of it is part of t_post_mm."""
    groups = (("gate", "up", "down"), ("qkv", "attn", "o"))
    planned = plan_windows(b, budget) if budget > 0 else {}
    pre = prelaunched(b, windows, budget) if (prelaunch and path == "vec") else {"gate_up": False, "qkv": False}
    if pre["gate_up"]:
        planned["gate"] = planned["up"] = 0.0
    if pre["qkv"]:
        planned["qkv"] = 0.0
    hit = {}
    for w, ops in zip(windows, groups):
        tot = sum(planned.get(op, 0.0) for op in ops)
        keep = 0.0 if (w <= 0 or tot <= 0) else min(1.0, m.cache_bytes / tot)
        for op in ops:
            hit[op] = planned.get(op, 0.0) * keep
    kernels = [("qkv", b["qkv"], hit["qkv"]), ("attn", b["attn"], hit["attn"]), ("o", b["o"], hit["o"]),
               ("gate_up", b["gate"] + b["up"], hit["gate"] + hit["up"]), ("down", b["down"], hit["down"])]
    mm = path in ("mm", "mmt")
    pre_mm = mm and prelaunch and hold_mm > 0 and windows[0] > 0 and planned.get("gate", 0.0) > 0
    t = m.t_small * (m.n_small - (1 if pre_mm else 0)) if mm else 0.0
    for name, nbytes, h in kernels:
        if pre_mm and name == "gate_up":
            rest, hit_rest = (1.0 - hold_mm) * nbytes, (1.0 - hold_mm) * h
            bw, bwc = (m.bw_mmt, m.bw_mmt_cache) if path == "mmt" else (m.bw_mm, m.bw_mm_cache)
            t += m.t_post_mm + hit_rest / bwc + (rest - hit_rest + b.get("p_gate_up", 0.0)) / bw
        elif pre.get(name):
            t += m.t_post + min(nbytes, m.reg_bytes) / m.bw_reg + max(0.0, nbytes - m.reg_bytes) / m.bw_hbm
        else:
            t += kernel_time(m, name, nbytes, h, path, b.get("p_" + name, 0.0) if mm else 0.0)
    for w, ops in zip(windows, groups):
        if w <= 0:
            continue
        pf = sum(planned.get(op, 0.0) for op in ops)
        t_pf = m.t_fork + pf / m.bw_prefetch if pf > 0 else 0.0
        t += w + m.t_window_extra
        if t_pf > w:                       # the tail of the prefetch shares HBM with the consumer
            t += (t_pf - w) * 0.5
    return t


def best_budget(b, windows, m: Machine, candidates=(8e6, 16e6, 32e6, 64e6, 96e6, 128e6, 192e6, 256e6), path="vec"):
    return min(candidates, key=lambda c: layer_time(b, windows, m, c, path=path))


def speedup(b, windows, m: Machine, budget, prelaunch=False, path="vec", hold_mm=0.0):
    return layer_time(b, windows, m, 0.0, path=path) / layer_time(b, windows, m, budget, prelaunch, path=path, hold_mm=hold_mm)


def fit_line(points):
    """Least-squares (t_fixed, bytes_per_us) of t = t_fixed + bytes / bw over (bytes, us) points."""
    n = len(points)
    sx = sum(p[0] for p in points); sy = sum(p[1] for p in points)
    sxx = sum(p[0] * p[0] for p in points); sxy = sum(p[0] * p[1] for p in points)
    den = n * sxx - sx * sx
    if n < 2 or den <= 0:
        raise ValueError("need at least two distinct sizes")
    slope = (n * sxy - sx * sy) / den
    icpt = (sy - slope * sx) / n
    if slope <= 0:
        raise ValueError("times do not grow with bytes")
    return icpt, 1.0 / slope
