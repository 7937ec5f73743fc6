"""GPU tests of the pre-launched gate/up projection on the matrix-core path (policy.prelaunch at batch 3..32):
the split-K GEMM is launched into the window after the attention block, keeps its first weight slabs on chip, walks the
window's prefetch job and waits for the tagged sums of squares of the residual kernel that follows the window on the other
stream.  Through the C ABI against the CPU oracle (|gpu - ref| <= 2e-2 + 1e-2*|ref|), bit-identical to prefetch off under
every policy, with the count of launches that really took that route checked, plus the bounded wait's error path."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_parity as bf
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session, default_policy

pytestmark = pytest.mark.gpu


def W(name, L, H, nq, nkv, F, B, T, paged=False, win=(8.0, 8.0), layout="row", fmts=("bf16", "bf16")):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, win, 1e-5, 500000.0, fmts[0], fmts[1], "head", layout)


def need_overlap(s):
    """Launching into a window needs two streams that really run side by side (the harness probes for a pair)."""
    if not s.overlap:
        pytest.skip("no pair of streams that overlap on this box: nothing is launched into a window")


def oracle_out(s, w):
    m = oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, 128, w.ffn, 16, w.rms_eps, w.rope_theta)
    fn = oracle.decode_layer if (w.weight_format, w.kv_format) == ("bf16", "bf16") else oracle.decode_layer_x
    lens = s.seq_lens_host.numpy()
    pt = s.page_table_host.numpy() if w.paged else None
    x = s.x_in.cpu().numpy().astype(np.float64)
    for l in s.layers:
        kp, vp = s.host_pools(l)
        x = fn(m, s.host_layer(l), kp, vp, pt, w.blocks_per_seq, lens, x)
    return x


# name, layers, H, nq, nkv, F, batch, context, paged, layout, windows, pre-launched gate/up projections per step
CASES = [
    ("wide_b8", 2, 8192, 8, 1, 3584, 8, 300, False, "tiled", (8.0, 8.0), 2),        # the 70B-shaped TP=8 shard
    ("wide_b8_row", 2, 8192, 8, 1, 3584, 8, 300, False, "row", (8.0, 8.0), 2),
    ("wide_b16_paged", 3, 8192, 8, 1, 3584, 16, 150, True, "tiled", (8.0, 8.0), 2),   # odd count: the last one stays behind
    ("wide_b3", 4, 4096, 4, 1, 7168, 3, 90, False, "row", (8.0, 0.0), 4),             # no window after the MLP block
    ("short_range", 2, 1024, 8, 2, 8192, 8, 70, False, "row", (8.0, 8.0), 2),         # 4 slabs per workgroup: all in the ring
    ("short_range5", 2, 1536, 12, 4, 6144, 4, 40, True, "tiled", (8.0, 8.0), 2),       # 5 slabs: one more than the ring holds
    ("no_window", 2, 8192, 8, 1, 3584, 8, 64, False, "tiled", (0.0, 8.0), 0),         # nothing to launch into
    ("b32", 2, 8192, 8, 1, 3584, 32, 64, False, "tiled", (8.0, 8.0), 2),              # two batch tiles: 8 slabs kept
    ("b17_paged_row", 2, 8192, 8, 1, 3584, 17, 100, True, "row", (8.0, 8.0), 2),
    ("b24_short", 2, 2048, 16, 2, 5632, 24, 40, False, "tiled", (8.0, 8.0), 2),       # two batch tiles, ranges of 6 slabs
    ("b48", 2, 8192, 8, 1, 3584, 48, 40, False, "tiled", (8.0, 8.0), 0),              # above the batch limit of that route
    ("b32_tp4", 2, 8192, 16, 2, 7168, 32, 40, False, "tiled", (8.0, 8.0), 0),         # less than a third of a range would stay
    ("small", 2, 1024, 8, 2, 768, 5, 129, False, "row", (8.0, 8.0), 0),               # too few workgroups to carry the job
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_prelaunched_gate_up_gemm_matches_oracle_and_prefetch_off(case):
    name, L, H, nq, nkv, F, B, T, paged, layout, win, want_pre = case
    w = W(name, L, H, nq, nkv, F, B, T, paged=paged, win=win, layout=layout)
    with Session(w, seed=97) as s:
        need_overlap(s)
        ref = oracle_out(s, w)
        off = s.run().clone()
        bf.assert_close(off.cpu().numpy(), ref, name)
        assert psv.psv_debug_last_step_prelaunches(s.ctx) == 0
        pools = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        big = 1 << 40
        for pol, pre in ((default_policy(w, budget_bytes=big), want_pre),                       # everything planned, whole
                         (default_policy(w, budget_bytes=max(1 << 20, w.weight_bytes_per_layer // 4), partial=1), want_pre),
                         (default_policy(w, budget_bytes=big, prelaunch=0), 0)):
            s.set_policy(pol)
            for rep in range(3):
                s.step()                                   # back to back: no host synchronisation between steps
            s.sync()
            assert torch.equal(s.x_out, off), "%s: a policy changes the result" % name
            assert psv.psv_debug_last_step_prelaunches(s.ctx) == pre, name
            for a, b in zip(pools, [s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers]):
                assert torch.equal(a, b)


# int8 weights: the operand is a pair of digit planes with block scales; the waiting int8 GEMM keeps 8 or 12 slabs on chip
I8_CASES = [
    ("w8_wide_b8", 2, 8192, 8, 1, 3584, 8, 200, False, "tiled", ("int8", "bf16"), 2),
    ("w8_wide_b16_row", 2, 8192, 8, 1, 3584, 16, 90, True, "row", ("int8", "bf16"), 2),
    ("w8_b3_odd", 3, 4096, 4, 1, 7168, 3, 60, False, "row", ("int8", "bf16"), 2),
    ("w8_short_range", 2, 1024, 8, 2, 8192, 8, 70, False, "tiled", ("int8", "int8"), 2),
]


@pytest.mark.parametrize("case", I8_CASES, ids=[c[0] for c in I8_CASES])
def test_prelaunched_int8_gate_up_gemm_matches_oracle_and_prefetch_off(case):
    name, L, H, nq, nkv, F, B, T, paged, layout, fmts, want_pre = case
    w = W(name, L, H, nq, nkv, F, B, T, paged=paged, layout=layout, fmts=fmts)
    with Session(w, seed=101) as s:
        need_overlap(s)
        ref = oracle_out(s, w)
        off = s.run().clone()
        bf.assert_close(off.cpu().numpy(), ref, name)
        for pol, pre in ((default_policy(w, budget_bytes=1 << 40), want_pre),
                         (default_policy(w, budget_bytes=max(1 << 20, w.weight_bytes_per_layer // 4)), want_pre),
                         (default_policy(w, budget_bytes=1 << 40, prelaunch=0), 0)):
            s.set_policy(pol)
            for rep in range(3):
                s.step()
            s.sync()
            assert torch.equal(s.x_out, off), "%s: a policy changes the result" % name
            assert psv.psv_debug_last_step_prelaunches(s.ctx) == pre, name


def test_gemm_that_gives_up_waiting_is_reported_and_the_context_survives():
    w = W("mmfail", 2, 8192, 8, 1, 3584, 8, 64, win=(300.0, 300.0), layout="tiled")     # long windows: the GEMM surely starts inside
    with Session(w, seed=99) as s:
        need_overlap(s)
        base = s.run().clone()
        s.set_policy(default_policy(w, budget_bytes=1 << 40))
        psv.psv_debug_force_wait_timeout(s.ctx, True)
        s.step()
        assert psv.psv_debug_last_step_prelaunches(s.ctx) == 2
        with pytest.raises(psv.PsvError) as e:
            s.sync()
        assert e.value.status == psv.PSV_ERR_HIP          # it read activations that were not there yet: results invalid
        psv.psv_debug_force_wait_timeout(s.ctx, False)
        assert torch.equal(s.run(), base)                 # reported once; the next step is clean
        assert psv.psv_debug_last_step_prelaunches(s.ctx) == 2


def test_waiting_gemm_outwaits_earlier_work_on_the_main_stream():
    """50 ms of unrelated work queued on the main stream ahead of the step: the gate and the projection launched ahead on
    the other stream sit it out (their waits are bounded by a second)."""
    w = W("mmbusy", 2, 8192, 8, 1, 3584, 8, 64, layout="tiled")
    with Session(w, seed=100) as s:
        need_overlap(s)
        base = s.run().clone()
        s.set_policy(default_policy(w, budget_bytes=1 << 40))
        psv.psv_spin(50000.0, s.main)
        s.step()
        s.sync()
        assert torch.equal(s.x_out, base)
        assert psv.psv_debug_last_step_prelaunches(s.ctx) == 2


def test_windows_of_any_length_layer_ranges_and_policy_changes_between_steps():
    """The waiting GEMM under windows much shorter than its own loads (it starts its wait after the window has ended) and
    much longer, over layer sub-ranges, with the policy and the windows changed between back-to-back steps."""
    w = W("mmwin", 4, 8192, 8, 1, 3584, 8, 80, layout="tiled")
    with Session(w, seed=102) as s:
        need_overlap(s)
        off = s.run().clone()
        sub = {(lb, le): s.run(layer_begin=lb, layer_end=le).clone() for lb, le in ((1, 3), (0, 1), (2, 4))}
        on = default_policy(w, budget_bytes=1 << 40)
        for win in ((0.5, 0.5), (150.0, 3.0), (2.0, 60.0)):
            s.set_windows(*win)
            s.set_policy(on)
            assert torch.equal(s.run(), off), win
            assert psv.psv_debug_last_step_prelaunches(s.ctx) == 4
            for (lb, le), ref in sub.items():
                assert torch.equal(s.run(layer_begin=lb, layer_end=le), ref), (win, lb, le)
            assert psv.psv_debug_last_step_prelaunches(s.ctx) == 2             # layers 2..3
        # policies alternate between steps without a host synchronisation in between
        s.set_windows(5.0, 5.0)
        for rep in range(3):
            s.set_policy(on)
            s.step()
            s.set_policy(default_policy(w, budget_bytes=16 << 20, prelaunch=0))
            s.step()
            s.set_policy(psv.prefetch_policy(mode=0))
            s.step()
        s.sync()
        assert torch.equal(s.x_out, off)
