"""GPU parity of the fused kernels of the batch-1 path (psv_set_fused_kernels; 1: QKV + attention + O in one launch,
gate/up + down in one launch; 2: the whole step in one launch with the windows timed inside the kernel; phases
handing over through tagged values) against the CPU oracle, through the C ABI:
same tolerance |gpu - ref| <= 2e-2 + 1e-2*|ref| and the same checks of the appended cache rows as the default
path, every policy bit-identical to prefetch off, and agreement with the one-kernel-per-operator path to rounding."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_int8 as q8
import test_gpu_parity as bf
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session, default_policy

pytestmark = pytest.mark.gpu

# name, layers, hidden, q heads, kv heads, ffn, context, paged
SHAPES = [
    ("c1_like", 2, 1024, 8, 8, 2816, 256, False),
    ("c2_like", 3, 4096, 4, 1, 1792, 700, False),         # ragged last chunk; 3 layers: odd number of stream hops
    ("tp8_70b", 2, 8192, 8, 1, 3584, 300, True),          # two loads per row in QKV and gate/up, paged cache
    ("tp4_70b", 1, 8192, 16, 2, 7168, 4096, False),       # two kv heads x 16 chunks; two loads per row in down
    ("odd", 2, 1536, 6, 3, 1280, 17, False),              # one tile, G = 2, rows that do not divide by the grid
    ("one_token", 1, 512, 4, 2, 256, 1, False),           # the step's own token is the whole span
]


# shapes the whole-step kernel takes (every thread group owns rows of every projection)
WHOLE_STEP = {"c1_like", "c2_like", "tp8_70b", "tp4_70b", "odd"}


def run_fused(w, seed, policies, mode=1):
    m = oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, 16, w.rms_eps, w.rope_theta)
    with Session(w, seed=seed, fused=mode) as s:
        x = s.x_in.cpu().numpy().astype(np.float64)
        lens = s.seq_lens_host.numpy()
        pt = s.page_table_host.numpy() if w.paged else None
        ref_pools = {}
        fn = oracle.decode_layer if w.weight_format == "bf16" else oracle.decode_layer_x
        for l in s.layers:
            kp, vp = s.host_pools(l)
            x = fn(m, s.host_layer(l), kp, vp, pt, w.blocks_per_seq, lens, x)
            ref_pools[l] = (kp, vp)
        off = s.run().clone()
        pools = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        bf.assert_close(off.cpu().numpy(), x, w.name + " fused")
        assert psv.psv_debug_last_step_path(s.ctx) == (2 if mode == 2 and w.name in WHOLE_STEP else 1)
        for l in s.layers:       # appended rows: the only cache bytes that may differ from the oracle's, and only to rounding
            for got, ref in ((synth.bits(s.k_pools[l]), ref_pools[l][0]), (synth.bits(s.v_pools[l]), ref_pools[l][1])):
                diff = got != ref
                assert diff.sum() <= w.n_kv_heads * 128
                if diff.any():
                    bf.assert_close(bf.from_bits(got[diff]), bf.from_bits(ref[diff]), "append of layer %d" % l)
        for pol in policies:
            s.set_policy(pol)
            for _ in range(2):
                assert torch.equal(s.run(), off), "%s: a policy changes the fused result" % w.name
            for a, b in zip(pools, [s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers]):
                assert torch.equal(a, b)
        # the default path on the same inputs agrees to rounding
        psv.psv_set_fused_kernels(s.ctx, 0)
        s.set_policy(psv.prefetch_policy(mode=0))
        plain = s.run().clone()
        assert torch.allclose(plain, off, rtol=1e-4, atol=1e-4)
        return off


@pytest.mark.parametrize("mode", [1, 2], ids=["per_block", "whole_step"])
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_fused_bf16_matches_oracle_and_policies_agree(shape, mode):
    name, L, H, nq, nkv, F, T, paged = shape
    w = bf.W(name, L, H, nq, nkv, F, 1, T, paged=paged, win=(6.0, 6.0))
    big = 1 << 40
    run_fused(w, 61, [default_policy(w, budget_bytes=big), default_policy(w, budget_bytes=big, prelaunch=0),
                      # a budget that hands only part of each window's operators to it: the consumer launched into the
                      # window must hold back the requests of what was not planned
                      default_policy(w, budget_bytes=max(1 << 16, w.weight_bytes_per_layer // 4)),
                      psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_WEIGHTS, budget_bytes=big, prelaunch=1, cu_budget=32)],
              mode=mode)


@pytest.mark.parametrize("mode", [1, 2], ids=["per_block", "whole_step"])
@pytest.mark.parametrize("shape", SHAPES[:3], ids=[s[0] for s in SHAPES[:3]])
def test_fused_int8_weights_match_oracle(shape, mode):
    name, L, H, nq, nkv, F, T, paged = shape
    w = q8.W(name, L, H, nq, nkv, F, 1, T, ("int8", "bf16"), paged=paged, win=(6.0, 6.0))
    run_fused(w, 62, [default_policy(w, budget_bytes=1 << 40)], mode=mode)


def test_fused_falls_back_where_the_shape_does_not_fit():
    """int8 cache, sequences beyond 4096 tokens and batch 2 run the one-kernel-per-operator path even when fused kernels
    are switched on: same bits as with the switch off."""
    for w in (q8.W("kv8", 2, 1024, 8, 2, 768, 1, 200, ("bf16", "int8")), bf.W("long", 1, 512, 4, 1, 256, 1, 5000),
              bf.W("b2", 2, 1024, 8, 2, 768, 2, 100)):
        with Session(w, seed=63, fused=True) as a, Session(w, seed=63) as b:
            xa, xb = a.run().clone(), b.run().clone()
            if w.kv_format == "int8" or w.batch > 1:      # the MLP block may still fuse: rows sums are the same bits either way
                assert torch.equal(xa, xb)
            else:
                assert torch.allclose(xa, xb, rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("mode", [1, 2], ids=["per_block", "whole_step"])
@pytest.mark.parametrize("win", [(0.0, 6.0), (12.0, 0.0), (0.0, 0.0)], ids=["only_after_mlp", "only_after_attention", "none"])
def test_fused_with_a_missing_window(win, mode):
    """A window of 0 us does not exist: nothing is launched (or timed) for it and whatever follows it requests its weights
    at once; results and policy-independence as with both windows."""
    w = bf.W("c2_like", 3, 4096, 4, 1, 1792, 1, 300, win=win)
    run_fused(w, 64, [default_policy(w, budget_bytes=1 << 40), default_policy(w, budget_bytes=1 << 40, prelaunch=0)], mode=mode)


@pytest.mark.parametrize("mode", [1, 2], ids=["per_block", "whole_step"])
def test_fused_layer_ranges_compose(mode):
    """Running layers [0, 2) and then [2, 3) on the first run's output equals one run over [0, 3), bit for bit: every
    kernel of the fused paths takes its layer's weights and cache by the layer's own index."""
    w = bf.W("c2_like", 3, 4096, 4, 1, 1792, 1, 300, win=(5.0, 5.0))
    with Session(w, seed=65, fused=mode) as s:
        s.set_policy(default_policy(w, budget_bytes=1 << 40))
        pools0 = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        whole = s.run().clone()
        pools1 = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        for t, src in zip([s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers], pools0):
            t.copy_(src)                                   # the cache as it was before the step
        mid = torch.empty_like(s.x_in)
        s.step(x_out=mid, layer_begin=0, layer_end=2)
        s.sync()
        out = torch.empty_like(s.x_in)
        s.step(x_in=mid, x_out=out, layer_begin=2, layer_end=3)
        s.sync()
        assert torch.equal(out, whole)
        for a, b in zip(pools1, [s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers]):
            assert torch.equal(a, b)


@pytest.mark.parametrize("mode", [1, 2], ids=["per_block", "whole_step"])
def test_fused_hand_over_that_expires_is_reported_and_the_context_survives(mode):
    """With every hand-over poll forced to expire at once the fused kernels still run to their end (no hang, no fault), the
    next sync reports the step as failed, once, and the context computes the right result again afterwards."""
    w = bf.W("c2_like", 2, 4096, 4, 1, 1792, 1, 300, win=(5.0, 5.0))
    with Session(w, seed=66, fused=mode) as s:
        s.set_policy(default_policy(w, budget_bytes=1 << 40))
        good = s.run().clone()
        psv.psv_debug_force_wait_timeout(s.ctx, True)
        s.step()
        with pytest.raises(psv.PsvError) as e:
            s.sync()
        assert e.value.status == psv.PSV_ERR_HIP
        psv.psv_debug_force_wait_timeout(s.ctx, False)
        assert torch.equal(s.run(), good)                 # the failed step's cache rows are rewritten by this one
        s.sync()


def test_stats_count_the_launches_of_the_path_that_ran():
    w = bf.W("c2_like", 2, 4096, 4, 1, 1792, 1, 300, win=(5.0, 5.0))
    for mode, want in ((None, 4), (1, 4), (0, 7), (2, 1)):       # by shape: per-segment kernels here; windows count as launches
        with Session(w, seed=67, fused=mode) as s:
            s.run()
            assert psv.psv_get_stats(s.ctx)["kernels_per_layer"] == want, mode
    wb = bf.W("b4", 2, 1024, 8, 2, 768, 4, 100, win=(5.0, 0.0))   # matrix-core path: ten kernels and one window
    with Session(wb, seed=67) as s:
        s.run()
        assert psv.psv_get_stats(s.ctx)["kernels_per_layer"] == 11
