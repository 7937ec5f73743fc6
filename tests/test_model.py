"""The analytic latency model (paper Section 5, re-parameterised): consistency with the library's planner and
the qualitative behaviour the paper and the measurements show.  CPU only."""
import pytest

from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import model, synth


def _bytes(w):
    return model.op_bytes(w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn, w.batch, w.context, weight_layout=w.weight_layout)


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
@pytest.mark.parametrize("budget_mb", [8, 64, 192])
def test_model_plan_matches_library_planner(name, budget_mb):
    w = synth.WORKLOADS[name].scaled(n_layers=2)
    b = _bytes(w)
    # the library counts the read-only span (context - 1); feed the model the same number
    b["attn"] = w.batch * (w.context - 1) * w.n_kv_heads * w.head_dim * 4
    budget = budget_mb << 20
    d = psv.model_desc(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn, w.batch, w.context)
    plan = psv.psv_plan_chain(d, w.batch, w.context, psv.prefetch_policy(mode=1, budget_bytes=budget, partial=1))
    lib = {psv.OP_NAMES[e["target_op"]]: e["bytes"] for e in plan if e["layer"] == 0}
    mod = {k: v for k, v in model.plan_windows(b, budget).items() if v > 0}
    assert lib == {k: int(v) for k, v in mod.items()}


def test_prefetch_off_is_the_plain_sum():
    w = synth.WORKLOADS["c2"]
    b, m = _bytes(w), model.Machine()
    proj = b["qkv"] + b["o"] + b["gate"] + b["up"] + b["down"]
    want = (4 * m.t_fixed + proj / m.bw_hbm + m.t_fixed_attn + b["attn"] / m.bw_attn
            + sum(w.window_us) + 2 * m.t_window_extra)
    assert model.layer_time(b, w.window_us, m, 0.0) == pytest.approx(want)
    # the matrix-core path adds its five small kernels and uses its own projection constants
    mm = (4 * m.t_fixed_mm + proj / m.bw_mm + m.t_fixed_attn + b["attn"] / m.bw_attn + m.n_small * m.t_small
          + sum(w.window_us) + 2 * m.t_window_extra)
    assert model.layer_time(b, w.window_us, m, 0.0, path="mm") == pytest.approx(mm)
    assert model.path_of(1, 8192) == "vec" and model.path_of(2, 4096) == "vec" and model.path_of(2, 8192) == "mm" and model.path_of(8, 1024) == "mm"


def test_fit_line_recovers_a_line_and_refuses_nonsense():
    icpt, bw = model.fit_line([(1e6, 3.0 + 1e6 / 4e6), (8e6, 3.0 + 8e6 / 4e6), (30e6, 3.0 + 30e6 / 4e6)])
    assert icpt == pytest.approx(3.0) and bw == pytest.approx(4e6)
    with pytest.raises(ValueError):
        model.fit_line([(1e6, 5.0), (2e6, 4.0)])
    with pytest.raises(ValueError):
        model.fit_line([(1e6, 5.0)])


# ---- the calibrated model against measured records -----------------------------------------------------------
#
# machine_mi355x.json holds constants fitted (sweeps.py calibrate) on fourteen calibration shapes that are neither benchmark
# workloads nor cells of the speedup map; tests/golden/measured_mi355x.json holds measured us/layer (sweeps.py record) of
# the five workloads, thirteen map cells and the c5 budget sweep.  The model has to predict every row it was not fitted on.

import json
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "measured_mi355x.json")
TOL = 0.12      # relative error allowed per row and mode (worst: 9.2 %, batch 64 at 4k tokens; c1: 9.1 %)


def _golden():
    return json.load(open(GOLDEN))


def test_calibration_shapes_are_not_the_rows_being_predicted():
    cal = json.load(open(model.MACHINE_FILE))
    rows = {(r["hidden"], r["n_q"], r["n_kv"], r["ffn"], r["batch"], r["context"]) for r in _golden()["rows"]}
    assert len(cal["shapes"]) >= 12 and not rows & {tuple(v[:6]) for v in cal["shapes"].values()}
    assert set(cal["machine"]) >= {"t_fixed", "bw_hbm", "bw_cache", "t_fixed_mm", "bw_mm", "t_fixed_mmt", "bw_mmt", "t_fixed_attn",
                                   "bw_attn", "t_small", "t_window_extra", "bw_prefetch", "t_post", "bw_reg", "t_post_mm"}


def test_calibrated_model_predicts_every_measured_row():
    m = model.Machine.load()
    assert m != model.Machine()                       # the calibration file is in place
    worst = 0.0
    for r in _golden()["rows"]:
        b = model.op_bytes(r["hidden"], r["n_q"], r["n_kv"], r["ffn"], r["batch"], r["context"], weight_layout=r["weight_layout"])
        path, w = model.path_of(r["batch"], r["hidden"], r["weight_layout"]), tuple(r["windows"])
        hold = model.mm_hold(r["batch"], r["hidden"], r["ffn"], weight_layout=r["weight_layout"]) if path != "vec" else 0.0
        # the model's copy of the library's rule for launching the gate/up GEMM into its window agrees with what ran
        if path != "vec":
            assert (hold > 0) == (r["prelaunched"] > 0), r["name"]
        pred = {"us_off": model.layer_time(b, w, m, 0.0, path=path),
                "us_cache_only": model.layer_time(b, w, m, r["budget"], path=path),
                "us_default": model.layer_time(b, w, m, r["budget"], prelaunch=True, path=path, hold_mm=hold)}
        for k, v in pred.items():
            err = abs(v / r[k] - 1.0)
            worst = max(worst, err)
            assert err <= TOL, "%s %s: model %.1f measured %.1f" % (r["name"], k, v, r[k])
    assert worst > 0.0


def test_calibrated_model_ranks_the_modes_like_the_measurement_at_batch_one():
    """Where the first consumers are launched into their windows (vector path) the measured gain over the cache-only
    policy is 3-6 us per layer on the large shapes; the model has to see a gain of the same order.  Rows that the library
    runs with one kernel per inter-window segment (kernel_path 1: the 8B-shaped TP=8 shard) are left out: the model has
    no class for those kernels, whose gain from being launched into the window is about twice as large."""
    m = model.Machine.load()
    seen = 0
    for r in _golden()["rows"]:
        if model.path_of(r["batch"], r["hidden"], r["weight_layout"]) != "vec" or r["hidden"] < 4096 or r.get("kernel_path", 0) != 0:
            continue
        seen += 1
        b = model.op_bytes(r["hidden"], r["n_q"], r["n_kv"], r["ffn"], r["batch"], r["context"])
        w = tuple(r["windows"])
        gain_model = model.layer_time(b, w, m, r["budget"]) - model.layer_time(b, w, m, r["budget"], prelaunch=True)
        gain_meas = r["us_cache_only"] - r["us_default"]
        assert gain_meas > 1.0 and 0.4 * gain_meas < gain_model < 2.5 * gain_meas, (r["name"], gain_meas, gain_model)
    assert seen >= 3


def test_calibrated_model_finds_the_budget_knee_of_the_kv_dominated_workload():
    """c5 budget sweep: the best budget grows with the window (64 MB at 20 us, 192 MB at 50 us: prefetch time about equal
    to the window, the optimum the paper's appendix describes), budgets far beyond it lose; the model has to pick a
    budget whose measured speedup is within 1.5 % of the best measured one, and to agree on which budgets lose."""
    m = model.Machine.load()
    g = _golden()
    b = model.op_bytes(8192, 8, 1, 3584, 32, 32768, weight_layout="tiled")
    for win in (20.0, 50.0):
        pts = [s for s in g["c5_budget_sweep"] if s["window"] == win]
        meas = {s["budget_mb"]: s["us_off"] / s["us_on"] for s in pts}
        pred = {mb: model.speedup(b, (win, win), m, mb * 2 ** 20, path="mmt") for mb in meas}
        best_meas, best_pred = max(meas, key=meas.get), max(pred, key=pred.get)
        assert meas[best_pred] >= meas[best_meas] - 0.015, (win, best_meas, best_pred)
        for mb in meas:
            if meas[mb] < 0.95:
                assert pred[mb] < 1.0, (win, mb)
            # up to the 256 MB of the memory-side cache the model is within 0.02; budgets beyond it thrash the cache, which the
            # model does not know: it says 0.88 where 600 MB in a 20 us window measure 0.82 (worst: 0.064)
            tol = 0.03 if mb <= 256 else 0.08
            assert abs(pred[mb] - meas[mb]) < tol, (win, mb, pred[mb], meas[mb])
        # prefetch time of the model's pick ~ the window (within a factor of two: the budgets are a coarse grid)
        t_pf = m.t_fork + best_pred * 2 ** 20 / m.bw_prefetch
        assert 0.5 * win <= t_pf <= 2.0 * win, (win, best_pred, t_pf)
    best20 = max((s for s in g["c5_budget_sweep"] if s["window"] == 20.0), key=lambda s: s["us_off"] / s["us_on"])["budget_mb"]
    best50 = max((s for s in g["c5_budget_sweep"] if s["window"] == 50.0), key=lambda s: s["us_off"] / s["us_on"])["budget_mb"]
    assert best20 < best50


def test_speedup_has_a_knee_at_window_capacity_and_at_cache_capacity():
    w = synth.WORKLOADS["c5"]
    b, m = _bytes(w), model.Machine()
    short = [model.speedup(b, (5.0, 5.0), m, c * 1e6) for c in (16, 64, 192)]
    assert short[0] > short[2]                       # a short window is overrun by a large prefetch
    long_ = [model.speedup(b, (50.0, 50.0), m, c * 1e6) for c in (16, 64, 192, 600)]
    assert long_[0] < long_[1] < long_[2]            # a long window rewards a larger budget ...
    assert long_[3] <= long_[2]                      # ... up to the cache capacity
    assert model.speedup(b, (0.0, 0.0), m, 192e6) <= 1.0 + 1e-12    # nothing to hide behind


def test_best_budget_grows_with_the_window():
    w = synth.WORKLOADS["c5"]
    b, m = _bytes(w), model.Machine()
    picks = [model.best_budget(b, (x, x), m) for x in (5.0, 20.0, 50.0)]
    assert picks[0] <= picks[1] <= picks[2] and picks[0] < picks[2]


def test_int8_formats_halve_the_weight_bytes_and_shrink_the_cache_rows():
    b16 = model.op_bytes(8192, 8, 1, 3584, 32, 32768)
    b8 = model.op_bytes(8192, 8, 1, 3584, 32, 32768, weight_format="int8", kv_format="int8")
    for op in ("qkv", "o", "gate", "up", "down"):
        assert b16[op] == 2 * b8[op]
    assert b8["attn"] * 512 == b16["attn"] * 264          # (128 + 4) * 2 bytes per row against 128 * 2 * 2
    m = model.Machine()
    assert model.layer_time(b8, (20.0, 20.0), m) < model.layer_time(b16, (20.0, 20.0), m)


def test_prelaunch_takes_the_first_consumers_out_of_the_post_window_path():
    """c2, bench policy: both first consumers are covered whole by their windows' plans, fit the register budget and
    leave only their post-window part; measured 64.3 -> 59.9 us/layer, the model has to land within 2 us of that gain.
    A budget that does not cover the gate matrix leaves gate/up where it was."""
    w = synth.WORKLOADS["c2"]
    b, m = _bytes(w), model.Machine()
    budget = 67.5 * (1 << 20)
    assert model.prelaunched(b, w.window_us, budget) == {"gate_up": True, "qkv": True}
    plain = model.layer_time(b, w.window_us, m, budget)
    pre = model.layer_time(b, w.window_us, m, budget, prelaunch=True)
    assert 2.4 < plain - pre < 6.4
    small = b["gate"] // 2                      # 7.3 MB: covers the next QKV (6.3 MB) but not the gate matrix
    assert model.prelaunched(b, w.window_us, small) == {"gate_up": False, "qkv": True}
    tiny = b["qkv"] // 2
    assert model.prelaunched(b, w.window_us, tiny) == {"gate_up": False, "qkv": False}
    assert model.layer_time(b, w.window_us, m, tiny, prelaunch=True) == model.layer_time(b, w.window_us, m, tiny)
    assert model.prelaunched(b, (0.0, 15.0), budget)["gate_up"] is False        # no window, nothing to launch into
    # a gate/up pair far beyond the register budget still streams most of its bytes after the window
    big = model.op_bytes(8192, 16, 2, 7168, 1, 4096)
    t_pre = model.layer_time(big, (20.0, 20.0), m, 256e6, prelaunch=True)
    assert t_pre > 40.0 + (big["gate"] + big["up"] - m.reg_bytes) / m.bw_hbm


def test_default_policy_is_the_bench_configuration():
    """bench.py, the full-size parity tests and smoke() share one default policy: C = min(192 MiB, window x 4.5 MiB/us),
    256 prefetch workgroups, operators that exceed the rest of the budget prefetched in part, consumers launched into their
    windows."""
    from paper_2501_08192_amd.harness import default_policy
    c2, c4, c5 = synth.WORKLOADS["c2"], synth.WORKLOADS["c4"], synth.WORKLOADS["c5"]
    p = default_policy(c2)
    assert (p.mode, p.cu_budget, p.partial, p.prelaunch, p.join) == (1, 256, 1, 1, 0)
    assert p.budget_bytes == int(67.5 * (1 << 20))
    assert default_policy(c4).partial == 1 and default_policy(c4).budget_bytes == int(112.5 * (1 << 20))
    assert default_policy(c5).budget_bytes == 90 << 20
    assert default_policy(c2, prelaunch=0, budget_bytes=123).budget_bytes == 123
    assert default_policy(c2.scaled(window_us=(100.0, 1.0))).budget_bytes == 192 << 20      # capped at the cache


def test_sweep_driver_parses_its_command_line():
    from paper_2501_08192_amd import sweeps
    assert set(sweeps.SHAPES) == {"tp4", "tp8"}
    with pytest.raises(SystemExit):
        sweeps.main(["map", "tp16"])                      # unknown shape
    with pytest.raises(SystemExit):
        sweeps.main(["sweep", "c9"])                      # unknown workload
