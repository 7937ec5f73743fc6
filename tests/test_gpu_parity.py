"""GPU parity: the HIP decode step, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bar: |gpu - ref| <= 2e-2 + 1e-2*|ref| elementwise on the residual stream (bf16 inputs, fp32
accumulation).  The bf16 K/V entries the step appends are held to the same value tolerance, and in the
first layer of the fp32-activation path (identical inputs on both sides) to one bf16 rounding step plus
1e-4; everything else in the cache is untouched; prefetch on/off and every policy give bit-identical results."""
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import from_bits
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session

pytestmark = pytest.mark.gpu

ATOL, RTOL = 2e-2, 1e-2


GRAPH_SKIP = pytest.mark.skip(reason="HIP graph mode is retired (psv_set_graph_mode(1) answers PSV_ERR_UNSUPPORTED): test runs that "
                                     "captured, replayed and destroyed step graphs ended twice in an abort inside the HIP runtime, "
                                     "cause not found; the same policies are checked bit for bit on the eager path")


def W(name, L, H, nq, nkv, F, B, T, paged=False, win=(5.0, 5.0), theta=500000.0):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, win, 1e-5, theta)


def oracle_model(w):
    return oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, block_tokens=16,
                        rms_eps=w.rms_eps, rope_theta=w.rope_theta)


def assert_close(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.isfinite(got).all(), what + ": non-finite output"
    assert (err <= bound).all(), "%s: max|err|=%.4g at %s (got %.6g ref %.6g), max|ref|=%.3g" % (
        what, err.max(), worst, got[worst], ref[worst], np.abs(ref).max())
    return err.max()


def bf16_ulp_distance(a_bits, b_bits):
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, 0x8000 - (x & 0x7fff), 0x8000 + (x & 0x7fff))
    return np.abs(key(a_bits) - key(b_bits))


def run_oracle(sess, layers, seq_lens=None):
    """Oracle on host copies of the session's inputs.  Returns (x_out, k_pools, v_pools) after the step."""
    w = sess.w
    m = oracle_model(w)
    lens = sess.seq_lens_host.numpy() if seq_lens is None else np.asarray(seq_lens, dtype=np.int32)
    pt = sess.page_table_host.numpy() if w.paged else None
    x = sess.x_in.detach().cpu().numpy().astype(np.float64)
    kps, vps = {}, {}
    for l in layers:
        kps[l], vps[l] = sess.host_pools(l)
        x = oracle.decode_layer(m, sess.host_layer(l), kps[l], vps[l], pt, w.blocks_per_seq, lens, x)
    return x, kps, vps


def check_step(w, seed=7, seq_lens=None, pool_slack=0, policy=None, graph=False):
    with Session(w, seed=seed, pool_slack_blocks=pool_slack) as s:
        if seq_lens is not None:
            s.seq_lens.copy_(torch.tensor(seq_lens, dtype=torch.int32))
        before = {l: (synth.bits(s.k_pools[l]).copy(), synth.bits(s.v_pools[l]).copy()) for l in s.layers}
        ref, kps, vps = run_oracle(s, s.layers, seq_lens)       # oracle works on host copies taken before the step
        if policy is not None:
            s.set_policy(policy)
        if graph:
            psv.psv_set_graph_mode(s.ctx, True)
        got = s.run().cpu().numpy()
        err = assert_close(got, ref, w.name)
        lens = s.seq_lens_host.numpy() if seq_lens is None else np.asarray(seq_lens)
        pt = s.page_table_host.numpy() if w.paged else None
        for l in s.layers:
            kg, vg = synth.bits(s.k_pools[l]), synth.bits(s.v_pools[l])
            kb, vb = before[l]
            km, vm = np.zeros(kg.shape, bool), np.zeros(vg.shape, bool)
            for b in range(w.batch):                      # the slot of token T-1, restated from the layout
                t = int(lens[b]) - 1
                blk = int(pt[b, t // 16]) if pt is not None else b * w.blocks_per_seq + t // 16
                km[blk, :, t % 16, :] = True
                vm[blk, :, :, t % 16] = True
            assert np.array_equal(kg[~km], kb[~km]) and np.array_equal(vg[~vm], vb[~vm]), "cache touched outside the new slot"
            assert np.array_equal(kps[l][~km], kb[~km]) and np.array_equal(vps[l][~vm], vb[~vm])
            for name, g_, r_ in (("K", kg[km], kps[l][km]), ("V", vg[vm], vps[l][vm])):
                gv, rv = from_bits(g_), from_bits(r_)
                assert_close(gv, rv, "%s append of layer %d" % (name, l))
                if l == s.layers[0] and w.batch <= 4:
                    # fp32 activations and identical inputs on both sides: the entries differ by at most one
                    # bf16 rounding step (2^-7 relative) plus the fp32-vs-fp64 accumulation error
                    assert (np.abs(gv - rv) <= 2.0 ** -7 * np.abs(rv) + 1e-4).all(), "%s append, layer %d" % (name, l)
        return err


# ----------------------------------------------------------------------------- small and ragged cases

def test_c1_whole_step_matches_oracle():
    check_step(synth.WORKLOADS["c1"], seed=2501)


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 32, 33, 77, 128, 129, 300])
def test_ragged_context_lengths(T):
    check_step(W("ragged", 2, 512, 4, 2, 256, 3, T), seed=T)


def test_intermediates_of_one_layer():
    w = W("mid", 1, 1024, 8, 2, 768, 2, 100)
    with Session(w, seed=11) as s:
        m = oracle_model(w)
        lw = s.host_layer(0)
        kp, vp = s.host_pools(0)
        x = s.x_in.cpu().numpy().astype(np.float64)
        s.run()
        B, H, nq, nkv, F = w.batch, w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn
        QR = (nq + 2 * nkv) * 128
        h1 = psv.psv_debug_read(s.ctx, psv.PSV_DBG_H1, np.zeros((B, H), np.float32))
        qkv = psv.psv_debug_read(s.ctx, psv.PSV_DBG_QKV, np.zeros((B, QR), np.float32))
        att = psv.psv_debug_read(s.ctx, psv.PSV_DBG_ATTN, np.zeros((B, nq * 128), np.float32))
        y = psv.psv_debug_read(s.ctx, psv.PSV_DBG_Y, np.zeros((B, H), np.float32))
        h2 = psv.psv_debug_read(s.ctx, psv.PSV_DBG_H2, np.zeros((B, H), np.float32))
        mm = psv.psv_debug_read(s.ctx, psv.PSV_DBG_M, np.zeros((B, F), np.float32))
        lens = s.seq_lens_host.numpy()
        for b in range(B):
            rh1 = oracle.rmsnorm(x[b], lw["g_attn"], w.rms_eps)
            assert_close(h1[b], rh1, "h1")
            rqkv = oracle.linear(lw["w_qkv"], rh1)
            assert_close(qkv[b], rqkv, "qkv")
        ref_full = oracle.decode_layer(m, lw, kp, vp, None, w.blocks_per_seq, lens, x)     # also appends to kp/vp
        for b in range(B):
            rqkv = oracle.linear(lw["w_qkv"], oracle.rmsnorm(x[b], lw["g_attn"], w.rms_eps))
            for j in range(nq):
                q = oracle.rope(rqkv[j * 128:(j + 1) * 128], w.context - 1, w.rope_theta)
                ro = oracle.attention_head(m, kp, vp, None, w.blocks_per_seq, lens, b, j, q)
                assert_close(att[b, j * 128:(j + 1) * 128], ro, "attention b%d head %d" % (b, j))
            ratt = np.concatenate([oracle.attention_head(
                m, kp, vp, None, w.blocks_per_seq, lens, b, j,
                oracle.rope(rqkv[j * 128:(j + 1) * 128], w.context - 1, w.rope_theta)) for j in range(nq)])
            ry = x[b] + oracle.linear(lw["w_o"], ratt)
            assert_close(y[b], ry, "y")
            rh2 = oracle.rmsnorm(ry, lw["g_mlp"], w.rms_eps)
            assert_close(h2[b], rh2, "h2")
            g, u = oracle.linear(lw["w_gate"], rh2), oracle.linear(lw["w_up"], rh2)
            assert_close(mm[b], np.array([oracle.silu(v) for v in g]) * u, "swiglu")
        assert_close(s.x_out.cpu().numpy(), ref_full, "layer output")


def test_rope_disabled():
    check_step(W("norope", 1, 512, 4, 4, 256, 2, 40, theta=0.0), seed=3)


def test_query_head_groupings_one_and_sixteen_heads_per_kv_head():
    check_step(W("g1", 2, 1024, 8, 8, 512, 4, 90), seed=4)          # G = 1, batch 4 (matrix-core projections)
    check_step(W("g1b2", 2, 1024, 8, 8, 512, 2, 90), seed=4)        # G = 1, batch 2 (vector projections)
    check_step(W("g16", 1, 512, 16, 1, 256, 2, 65), seed=5)         # G = 16


@pytest.mark.parametrize("B", [5, 8, 16, 17, 33, 64])
def test_mfma_projection_path(B):
    check_step(W("mfma%d" % B, 2, 1024, 8, 1, 768, B, 70), seed=B)


def test_long_context_many_chunks():
    check_step(W("long", 1, 512, 4, 1, 256, 1, 5000), seed=6)
    check_step(W("long2", 1, 512, 8, 1, 256, 2, 40000 - 7), seed=8)     # several tiles per wave


def test_paged_cache_with_shuffled_over_provisioned_pool():
    check_step(W("paged", 2, 512, 4, 1, 256, 4, 200, paged=True), seed=9, pool_slack=13)
    check_step(W("paged8", 1, 512, 8, 2, 256, 9, 333, paged=True), seed=10, pool_slack=5)


def test_mixed_sequence_lengths():
    w = W("mixed", 2, 512, 4, 2, 256, 4, 160)
    check_step(w, seed=12, seq_lens=[160, 1, 47, 129])


def test_page_table_permutation_invariance_bitwise():
    """Same logical cache behind two different page tables gives the same bits (tiles follow logical order)."""
    w = W("perm", 1, 512, 4, 1, 256, 3, 150, paged=True)
    with Session(w, seed=13, pool_slack_blocks=7) as a, Session(w, seed=13, pool_slack_blocks=7) as b:
        nb, mb = a.pool_blocks, w.blocks_per_seq
        perm = torch.randperm(nb, generator=torch.Generator().manual_seed(1))
        new_pt = perm[a.page_table_host.long()].to(torch.int32)
        # move a's blocks to their new places in b's pools
        for l in a.layers:
            b.k_pools[l].zero_(); b.v_pools[l].zero_()
            src = a.page_table_host.long().reshape(-1).to(a.device)
            dst = new_pt.long().reshape(-1).to(a.device)
            b.k_pools[l][dst] = a.k_pools[l][src]
            b.v_pools[l][dst] = a.v_pools[l][src]
        b.page_table.copy_(new_pt)
        xa = a.run().clone()
        xb = b.run().clone()
        assert torch.equal(xa, xb)


# ----------------------------------------------------------------------------- state and policy invariance

def _policies(w):
    big = 1 << 40
    return [
        psv.prefetch_policy(mode=1, budget_bytes=big),
        psv.prefetch_policy(mode=1, budget_bytes=big, join=1),
        psv.prefetch_policy(mode=1, budget_bytes=big, chunk_bytes=1 << 20, cu_budget=8),
        psv.prefetch_policy(mode=1, budget_bytes=3 * w.ffn * w.hidden * 2, partial=1, cu_budget=300),
        psv.prefetch_policy(mode=1, budget_bytes=1 << 20, partial=1, chunk_bytes=4096),
        psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_KV, budget_bytes=big, chunk_bytes=64 << 10),
        psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_WEIGHTS, budget_bytes=big),
        psv.prefetch_policy(mode=1, budget_bytes=big, prelaunch=1),
        psv.prefetch_policy(mode=1, budget_bytes=big, prelaunch=1, chunk_bytes=1 << 20, cu_budget=8, join=1),
        psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_KV, budget_bytes=big, prelaunch=1),
    ]


@pytest.mark.parametrize("wl", [W("pol1", 3, 1024, 8, 2, 768, 2, 300),
                                W("pol2", 2, 512, 4, 1, 512, 24, 130, paged=True)])
def test_prefetch_policies_are_bit_identical(wl):
    _policies_bit_identical(wl, (False,))


@GRAPH_SKIP
@pytest.mark.parametrize("wl", [W("pol1", 3, 1024, 8, 2, 768, 2, 300),
                                W("pol2", 2, 512, 4, 1, 512, 24, 130, paged=True)])
def test_graph_mode_is_bit_identical_for_every_policy(wl):
    _policies_bit_identical(wl, (True,))


def _policies_bit_identical(wl, graph_modes):
    with Session(wl, seed=21) as s:
        def snapshot():
            x = s.run().clone()
            return x, [s.k_pools[l].clone() for l in s.layers], [s.v_pools[l].clone() for l in s.layers]
        base = snapshot()
        again = snapshot()                                   # idempotence
        assert torch.equal(base[0], again[0])
        ref, _, _ = run_oracle(s, s.layers)     # the cache already holds this step's entries; the oracle rewrites them
        assert_close(base[0].cpu().numpy(), ref, wl.name)
        for pol in _policies(wl):
            for graph in graph_modes:
                for win in ((5.0, 5.0), (0.0, 0.0), (20.0, 1.0)):
                    s.set_policy(pol)
                    s.set_windows(*win)
                    psv.psv_set_graph_mode(s.ctx, graph)
                    for rep in range(2):                     # a graph is replayed at least once
                        got = snapshot()
                        assert torch.equal(got[0], base[0]), (pol.mode, pol.join, graph, win)
                        for a, b in zip(got[1] + got[2], base[1] + base[2]):
                            assert torch.equal(a, b)
        s.set_policy(_policies(wl)[6])
        plan = psv.psv_plan(s.ctx)
        assert all(e["target_op"] != psv.PSV_OP_ATTN for e in plan)       # that policy: weights only
        assert psv.psv_get_stats(s.ctx)["steps"] > 10


@pytest.mark.parametrize("wl", [W("tune1", 2, 1024, 8, 2, 768, 2, 3000), W("tune2", 2, 512, 4, 1, 512, 24, 700, paged=True)])
def test_tuned_attention_split_matches_oracle_and_policies_stay_bit_identical(wl):
    _tuned_split(wl, (False,))


@GRAPH_SKIP
@pytest.mark.parametrize("wl", [W("tune1", 2, 1024, 8, 2, 768, 2, 3000), W("tune2", 2, 512, 4, 1, 512, 24, 700, paged=True)])
def test_graph_mode_with_a_tuned_attention_split(wl):
    _tuned_split(wl, (True,))


def _tuned_split(wl, graph_modes):
    with Session(wl, seed=31) as s:
        before = s.run().clone()
        chunk = s.tune_attention()
        assert chunk >= 128 and chunk % 128 == 0
        ref, _, _ = run_oracle(s, s.layers)
        base = s.run().clone()
        assert_close(base.cpu().numpy(), ref, wl.name)
        assert_close(before.cpu().numpy(), ref, wl.name + " (default split)")
        for pol in _policies(wl)[:3]:
            for graph in graph_modes:
                s.set_policy(pol)
                psv.psv_set_graph_mode(s.ctx, graph)
                for rep in range(2):
                    assert torch.equal(s.run(), base)
        assert s.tune_attention() % 128 == 0        # callable again; the context keeps working
        assert_close(s.run().cpu().numpy(), ref, wl.name + " (second tuning)")


def test_prelaunched_consumers_whole_steps_odd_layer_counts_and_windows():
    """Pre-launch hops streams at every window: odd hop counts, a zero window in between and back-to-back steps."""
    for L, win in ((1, (5.0, 5.0)), (2, (5.0, 0.0)), (3, (0.0, 8.0)), (3, (6.0, 6.0))):
        w = W("pre%d" % L, L, 1024, 8, 2, 768, 1, 200, win=win)
        with Session(w, seed=41) as s:
            base = s.run().clone()
            ref, _, _ = run_oracle(s, s.layers)
            assert_close(base.cpu().numpy(), ref, w.name)
            s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 40, prelaunch=1))
            for rep in range(3):
                s.step()                                  # no host synchronisation between steps
            s.sync()
            assert torch.equal(s.x_out, base), (L, win)
            assert torch.equal(s.run(layer_begin=0, layer_end=1), s.run(layer_begin=0, layer_end=1))


def test_prelaunched_consumer_that_gives_up_waiting_is_reported_and_the_context_survives():
    w = W("prefail", 2, 1024, 8, 2, 768, 1, 120, win=(300.0, 300.0))     # long windows: the consumers surely start inside them
    with Session(w, seed=42) as s:
        base = s.run().clone()
        s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 40, prelaunch=1))
        psv.psv_debug_force_wait_timeout(s.ctx, True)
        s.step()
        with pytest.raises(psv.PsvError) as e:
            s.sync()
        assert e.value.status == psv.PSV_ERR_TIMEOUT
        psv.psv_debug_force_wait_timeout(s.ctx, False)
        assert torch.equal(s.run(), base)                 # reported once; the next step is clean
        s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 40, prelaunch=0))
        psv.psv_debug_force_wait_timeout(s.ctx, True)     # nothing is pre-launched: nothing to time out
        assert torch.equal(s.run(), base)


def test_prelaunched_consumers_outwait_earlier_work_on_the_main_stream():
    """60 ms of unrelated work queued on the main stream ahead of the step: the gates and the consumers launched ahead on
    the other stream have to sit it out (their waits are bounded by a second), not give up and compute on stale data."""
    w = W("prebusy", 2, 1024, 8, 2, 768, 1, 120, win=(8.0, 8.0))
    with Session(w, seed=43) as s:
        base = s.run().clone()
        s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 40, prelaunch=1))
        psv.psv_spin(60000.0, s.main)
        s.step()
        s.sync()                                          # would raise if a consumer had given up
        assert torch.equal(s.x_out, base)


def test_length_beyond_the_descriptors_max_seq_is_an_empty_sequence():
    """The cache has room for 208 tokens per sequence, the context was created for at most 64: a length in between
    is outside what the attention grid covers and must be treated like any other invalid length (nothing appended,
    empty attention span), not half-processed."""
    w = W("gap", 1, 512, 4, 2, 256, 2, 200)
    with Session(w, seed=23, max_seq=64) as s:
        s.set_policy(psv.prefetch_policy(mode=0))
        k0, v0 = s.k_pools[0].clone(), s.v_pools[0].clone()
        s.seq_lens.copy_(torch.tensor([100, 0], dtype=torch.int32))
        a = s.run().clone()
        assert torch.isfinite(a).all()
        assert torch.equal(s.k_pools[0], k0) and torch.equal(s.v_pools[0], v0)
        s.seq_lens.copy_(torch.tensor([0, 0], dtype=torch.int32))
        assert torch.equal(s.run(), a)
        # lengths inside the range still work on the same context
        s.seq_lens.copy_(torch.tensor([64, 33], dtype=torch.int32))
        s.run()
        assert not torch.equal(s.k_pools[0], k0)


def test_layer_ranges_chain_like_the_whole_step():
    w = W("range", 3, 512, 4, 2, 256, 2, 90)
    with Session(w, seed=22) as s:
        whole = s.run().clone()
        tmp = torch.empty_like(s.x_in)
        s.step(x_out=tmp, layer_begin=0, layer_end=1)
        s.step(x_in=tmp, x_out=tmp, layer_begin=1, layer_end=3)       # in place
        s.sync()
        assert torch.equal(tmp, whole)


def test_runtime_argument_errors():
    w = W("err", 2, 512, 4, 2, 256, 2, 64)
    with Session(w, seed=23) as s:
        L = psv.lib()
        x, y = s.x_in.data_ptr(), s.x_out.data_ptr()
        assert L.psv_decode_step(s.ctx, x, y, 3, 0, 2) == psv.PSV_ERR_INVALID_ARG        # batch > max_batch
        assert L.psv_decode_step(s.ctx, x, y, 2, 1, 1) == psv.PSV_ERR_INVALID_ARG        # empty range
        assert L.psv_decode_step(s.ctx, x, y, 2, 0, 3) == psv.PSV_ERR_INVALID_ARG
        assert L.psv_decode_step(s.ctx, x + 4, y, 2, 0, 2) == psv.PSV_ERR_INVALID_ARG    # misaligned
        assert L.psv_decode_step(s.ctx, None, y, 2, 0, 2) == psv.PSV_ERR_INVALID_ARG
        assert L.psv_set_comm_windows(s.ctx, -1.0, 0.0) == psv.PSV_ERR_INVALID_ARG
        s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 30))
        assert L.psv_decode_step(s.ctx, x, y, 1, 0, 2) == psv.PSV_ERR_BAD_STATE          # plan sized for batch 2
        assert L.psv_set_graph_mode(s.ctx, 1) == psv.PSV_ERR_UNSUPPORTED                 # graph mode is retired
        assert L.psv_set_graph_mode(s.ctx, 0) == psv.PSV_OK
        assert L.psv_set_graph_mode(s.ctx, 2) == psv.PSV_ERR_INVALID_ARG
        s.run()                                                                           # still usable
    with torch.cuda.device(0):
        d = psv.model_desc(2, 512, 4, 2, 256, 2, 64)
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        ctx = psv.psv_create(d, a, b)
        xin = torch.zeros(2, 512, device="cuda")
        assert psv.lib().psv_decode_step(ctx, xin.data_ptr(), xin.data_ptr(), 2, 0, 2) == psv.PSV_ERR_BAD_STATE
        psv.psv_destroy(ctx)


# ----------------------------------------------------------------------------- stand-alone kernels

def test_spin_window_duration():
    s = torch.cuda.Stream()
    for us in (5.0, 15.0, 50.0, 200.0):
        psv.psv_spin(us, s)
        s.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(s):
            e0.record(s)
            for _ in range(20):
                psv.psv_spin(us, s)
            e1.record(s)
        s.synchronize()
        per = e0.elapsed_time(e1) * 1000.0 / 20
        assert us <= per <= us + 25.0, (us, per)


def test_prefetch_and_copy_kernels_leave_memory_unchanged_and_copy_exactly():
    s = torch.cuda.Stream()
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device="cuda")
    ref = src.clone()
    dst = torch.zeros_like(src)
    torch.cuda.synchronize()
    for nbytes in (16, 4096, 4 * (1 << 20) - 16, 4 * (1 << 20)):
        for wg in (1, 7, 64, 1000):
            psv.psv_prefetch_region(src, nbytes, wg, s)
    psv.psv_copy_bytes(dst, src, 4 * (1 << 20), s)
    s.synchronize()
    assert torch.equal(src, ref) and torch.equal(dst, ref)
