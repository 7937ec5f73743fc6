"""Analytic latency model of one decode layer with and without prefetching, in the spirit of the paper's
design-space model (Section 5, "Performance & cost model": memory time linear in bytes over the bandwidth of
the level that serves them, communication as a fixed latency), re-parameterised with what was measured on
MI355X.  Pure Python; used to predict the speedup map and to pick a prefetch budget.

Per kernel:  t = t_fixed + hit_bytes / bw_cache + miss_bytes / bw_hbm.
Per window:  t = max(window, t_fork + prefetch_bytes / bw_prefetch)   (the prefetch may outlast the window),
and whatever part of a prefetch is still running after the window competes with its consumer for HBM.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class Machine:
    bw_hbm: float = 4.5e6        # bytes/us a consumer kernel streams from HBM (incremental rate measured on GEMV/GEMM)
    bw_cache: float = 5.5e6      # bytes/us a consumer kernel streams prefetched (Infinity-Cache resident) data
    bw_prefetch: float = 5.0e6   # bytes/us of the prefetch kernel with >= 128 workgroups
    t_fixed: float = 3.5         # us per dependent kernel: dispatch, first byte, reduction, drain
    t_fork: float = 2.5          # us from window start to the first prefetch load (gate kernel + dispatch)
    cache_bytes: float = 192e6   # usable part of the 256 MB Infinity Cache
    small_kernels: float = 0.0   # extra us per layer for merge / reduce / norm launches (matrix-core path)
    reg_bytes: float = 32e6      # weights the first pass of a GEMV launched into a window holds in registers
    t_post: float = 3.0          # us such a kernel still needs after the window (poll, activations, reduce, drain)
    bw_reg: float = 24e6         # bytes/us at which it works through the weights it holds (c2: QKV 3.3 us, gate/up 4.3 us)


def op_bytes(hidden, n_q, n_kv, ffn, batch, context, head_dim=128, weight_format="bf16", kv_format="bf16"):
    """Algorithmic bytes of the operators of one layer: bf16, or the int8 formats (1 byte per weight; per cached
    token and kv head 128 code bytes + a 4-byte scale, for K and for V)."""
    wb = 1 if weight_format == "int8" else 2
    kv_token = 2 * (head_dim + 4) if kv_format == "int8" else 2 * 2 * head_dim
    qkv = (n_q + 2 * n_kv) * head_dim * hidden * wb
    return {"qkv": qkv, "attn": batch * context * n_kv * kv_token, "o": hidden * n_q * head_dim * wb,
            "gate": ffn * hidden * wb, "up": ffn * hidden * wb, "down": hidden * ffn * wb}


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
    the pair).  Batch 1-2 only: the matrix-core path has no such launch."""
    planned = plan_windows(b, budget) if budget > 0 else {}
    return {"gate_up": windows[0] > 0 and planned.get("gate", 0.0) >= b["gate"],
            "qkv": windows[1] > 0 and planned.get("qkv", 0.0) >= b["qkv"]}


def layer_time(b, windows, m: Machine, budget=0.0, prelaunch=False):
    """us per layer.  budget = 0: prefetch off.  A window of 0 us launches no prefetch; a window's plan larger
    than the cache keeps only cache_bytes / planned of itself resident.  prelaunch: the first consumer of a window
    that the plan covers whole is launched into the window; it is not prefetched a second time, holds up to
    reg_bytes of its weights in registers when the window ends and streams the rest."""
    groups = (("gate", "up", "down"), ("qkv", "attn", "o"))
    planned = plan_windows(b, budget) if budget > 0 else {}
    pre = prelaunched(b, windows, budget) if prelaunch else {"gate_up": False, "qkv": False}
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
    t = m.small_kernels
    for name, nbytes, h in kernels:
        if pre.get(name):
            t += m.t_post + min(nbytes, m.reg_bytes) / m.bw_reg + max(0.0, nbytes - m.reg_bytes) / m.bw_hbm
        else:
            t += m.t_fixed + h / m.bw_cache + (nbytes - h) / m.bw_hbm
    for w, ops in zip(windows, groups):
        if w <= 0:
            continue
        pf = sum(planned.get(op, 0.0) for op in ops)
        t_pf = m.t_fork + pf / m.bw_prefetch if pf > 0 else 0.0
        t += w
        if t_pf > w:                       # the tail of the prefetch shares HBM with the consumer
            t += (t_pf - w) * 0.5
    return t


def best_budget(b, windows, m: Machine, candidates=(8e6, 16e6, 32e6, 64e6, 96e6, 128e6, 192e6, 256e6)):
    return min(candidates, key=lambda c: layer_time(b, windows, m, c))


def speedup(b, windows, m: Machine, budget, prelaunch=False):
    return layer_time(b, windows, m, 0.0) / layer_time(b, windows, m, budget, prelaunch)
