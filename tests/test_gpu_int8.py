"""GPU parity of the int8 formats (int8 weights with per-row scales, int8 KV-cache with per-token scales) against
the int8 variant of the CPU oracle, through the C ABI, on the same seeded inputs.

Bar: |gpu - ref| <= 2e-2 + 1e-2*|ref| on the residual stream.  The rows the step appends to an int8 cache are
quantised from single-precision values on both sides (the oracle rounds its double-precision rows to single first),
so a code may differ by one step where the two pipelines' inputs straddle a rounding boundary: the appended rows are
compared as dequantised values with one code step of slack, their scales to 1e-3 relative, and every other byte of
the cache must be untouched.  Prefetch on/off and graph mode must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session

pytestmark = pytest.mark.gpu

ATOL, RTOL = 2e-2, 1e-2
FORMATS = [("int8", "int8"), ("int8", "bf16"), ("bf16", "int8")]


def W(name, L, H, nq, nkv, F, B, T, fmt, paged=False, win=(5.0, 5.0), theta=500000.0):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, win, 1e-5, theta, fmt[0], fmt[1])


def oracle_model(w):
    return oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, block_tokens=16,
                        rms_eps=w.rms_eps, rope_theta=w.rope_theta)


def assert_close(got, ref, what, extra=0.0):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref) + extra
    assert np.isfinite(got).all(), what + ": non-finite output"
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert (err <= bound).all(), "%s: max|err|=%.4g at %s (got %.6g ref %.6g), max|ref|=%.3g" % (
        what, err.max(), worst, got[worst], ref[worst], np.abs(ref).max())
    return err.max()


def new_slot_mask_int8(shape, w, lens, pt):
    """Byte masks of the appended rows in an int8 pool [blocks, kv heads, 2112], restated from the layout:
    K codes of token row r at [r*128, (r+1)*128), V codes at c*16 + r, the row's scale at 2048 + 4r."""
    km, vm = np.zeros(shape, bool), np.zeros(shape, bool)
    for b in range(w.batch):
        t = int(lens[b]) - 1
        blk = int(pt[b, t // 16]) if pt is not None else b * w.blocks_per_seq + t // 16
        r = t % 16
        km[blk, :, r * 128:(r + 1) * 128] = True
        vm[blk, :, r:2048:16] = True
        km[blk, :, 2048 + 4 * r:2048 + 4 * r + 4] = True
        vm[blk, :, 2048 + 4 * r:2048 + 4 * r + 4] = True
    return km, vm


def appended_rows_int8(pool, w, lens, pt, is_v):
    """Dequantised appended rows [batch, kv heads, 128] and their scales [batch, kv heads]."""
    rows = np.zeros((w.batch, w.n_kv_heads, 128))
    scales = np.zeros((w.batch, w.n_kv_heads), dtype=np.float32)
    for b in range(w.batch):
        t = int(lens[b]) - 1
        blk = int(pt[b, t // 16]) if pt is not None else b * w.blocks_per_seq + t // 16
        r = t % 16
        for h in range(w.n_kv_heads):
            unit = pool[blk, h]
            codes = unit[r:2048:16] if is_v else unit[r * 128:(r + 1) * 128]
            sc = np.frombuffer(unit[2048 + 4 * r:2048 + 4 * r + 4].tobytes(), dtype=np.float32)[0]
            rows[b, h] = codes.view(np.int8).astype(np.float64) * float(sc)
            scales[b, h] = sc
    return rows, scales


def check_step(w, seed=7, seq_lens=None, pool_slack=0, policy=None, layers=None, lb=None, le=None):
    m = oracle_model(w)
    with Session(w, seed=seed, pool_slack_blocks=pool_slack, layers=layers) as s:
        if seq_lens is not None:
            s.seq_lens.copy_(torch.tensor(seq_lens, dtype=torch.int32))
        lens = s.seq_lens_host.numpy() if seq_lens is None else np.asarray(seq_lens, dtype=np.int32)
        pt = s.page_table_host.numpy() if w.paged else None
        before = {l: (synth.bits(s.k_pools[l]).copy(), synth.bits(s.v_pools[l]).copy()) for l in s.layers}
        x = s.x_in.detach().cpu().numpy().astype(np.float64)
        ref_pools = {}
        for l in s.layers:
            kp, vp = s.host_pools(l)
            x = oracle.decode_layer_x(m, s.host_layer(l), kp, vp, pt, w.blocks_per_seq, lens, x)
            ref_pools[l] = (kp, vp)
        kw = {} if lb is None else dict(layer_begin=lb, layer_end=le)
        off = s.run(**kw).clone()
        if policy is not None:
            s.set_policy(policy)
            on = s.run(**kw).clone()
            assert torch.equal(on, off), "prefetch on/off differ"
        err = assert_close(off.cpu().numpy(), x, w.name)
        for l in s.layers:
            kg, vg = synth.bits(s.k_pools[l]), synth.bits(s.v_pools[l])
            kb, vb = before[l]
            if w.kv_format == "int8":
                km, vm = new_slot_mask_int8(kg.shape, w, lens, pt)
                assert np.array_equal(kg[~km], kb[~km]) and np.array_equal(vg[~vm], vb[~vm]), "cache touched outside the new rows"
                for is_v, g_, r_ in ((False, kg, ref_pools[l][0]), (True, vg, ref_pools[l][1])):
                    got_rows, got_sc = appended_rows_int8(g_, w, lens, pt, is_v)
                    ref_rows, ref_sc = appended_rows_int8(r_, w, lens, pt, is_v)
                    np.testing.assert_allclose(got_sc, ref_sc, rtol=1e-3 if l == s.layers[0] else 5e-2)
                    assert_close(got_rows, ref_rows, "%s append of layer %d" % ("V" if is_v else "K", l),
                                 extra=1.01 * ref_sc[..., None].astype(np.float64))
                    if l == s.layers[0]:      # same inputs on both sides: every row reaches full scale
                        assert (np.abs(got_rows).max(axis=-1) >= 126.9 * got_sc).all()
            else:
                diff = (kg != ref_pools[l][0])
                assert diff.sum() <= w.batch * w.n_kv_heads * 128
        return err


# ----------------------------------------------------------------------------- small and ragged cases

@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("T", [1, 16, 17, 33, 129, 300])
def test_ragged_context_lengths(fmt, T):
    check_step(W("ragged", 2, 512, 4, 2, 256, 2, T, fmt), seed=T)


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("B", [1, 2, 5, 17, 64])
def test_vector_and_matrix_core_paths(fmt, B):
    check_step(W("b%d" % B, 2, 1024, 8, 1, 768, B, 70, fmt), seed=B)


@pytest.mark.parametrize("fmt", FORMATS)
def test_head_groupings(fmt):
    check_step(W("g1", 1, 1024, 8, 8, 512, 2, 90, fmt), seed=4)          # G = 1, 8 kv heads
    check_step(W("g16", 1, 512, 16, 1, 256, 3, 65, fmt), seed=5)         # G = 16


@pytest.mark.parametrize("fmt", FORMATS)
def test_paged_mixed_lengths_and_policies(fmt):
    w = W("paged", 2, 512, 4, 2, 256, 4, 200, fmt, paged=True)
    pol = psv.prefetch_policy(mode=1, budget_bytes=1 << 40, cu_budget=64)
    check_step(w, seed=9, pool_slack=13, seq_lens=[200, 1, 47, 129], policy=pol)
    w = W("paged24", 1, 512, 8, 1, 512, 24, 333, fmt, paged=True)
    pol = psv.prefetch_policy(mode=1, budget_bytes=3 << 20, partial=1, chunk_bytes=64 << 10, cu_budget=300)
    check_step(w, seed=10, pool_slack=5, policy=pol)


def test_long_context_many_chunks_int8():
    check_step(W("long", 1, 512, 4, 1, 256, 1, 5000, ("int8", "int8")), seed=6)
    check_step(W("long2", 1, 512, 8, 1, 256, 2, 40000 - 7, ("int8", "int8")), seed=8)


def test_rope_disabled_int8():
    check_step(W("norope", 1, 512, 4, 4, 256, 2, 40, ("int8", "int8"), theta=0.0), seed=3)


def test_policies_are_bit_identical_int8():
    _policies_int8((False,))


@pytest.mark.skip(reason="HIP graph mode is retired (psv_set_graph_mode(1) answers PSV_ERR_UNSUPPORTED): test runs that captured, "
                         "replayed and destroyed step graphs ended twice in an abort inside the HIP runtime, cause not found")
def test_graph_mode_is_bit_identical_int8():
    _policies_int8((True,))


def _policies_int8(graph_modes):
    w = W("pol", 3, 1024, 8, 2, 768, 2, 300, ("int8", "int8"))
    with Session(w, seed=21) as s:
        base = s.run().clone()
        pools = [s.k_pools[l].clone() for l in s.layers]
        big = 1 << 40
        for pol in (psv.prefetch_policy(mode=1, budget_bytes=big),
                    psv.prefetch_policy(mode=1, budget_bytes=big, join=1, chunk_bytes=1 << 20, cu_budget=8),
                    psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_KV, budget_bytes=1 << 20, partial=1)):
            for graph in graph_modes:
                s.set_policy(pol)
                psv.psv_set_graph_mode(s.ctx, graph)
                for rep in range(2):
                    assert torch.equal(s.run(), base)
                    for a, b in zip(pools, [s.k_pools[l] for l in s.layers]):
                        assert torch.equal(a, b)


def test_plan_and_stats_count_int8_bytes():
    w = W("bytes", 2, 1024, 8, 2, 768, 2, 300, ("int8", "int8"))
    with Session(w, seed=22) as s:
        s.set_policy(psv.prefetch_policy(mode=1, budget_bytes=1 << 40))
        plan = {(e["layer"], e["window"], e["target_op"]): e for e in psv.psv_plan(s.ctx)}
        assert plan[(0, 0, psv.PSV_OP_GATE)]["bytes"] == 768 * 1024
        assert plan[(0, 1, psv.PSV_OP_QKV)]["bytes"] == (8 + 4) * 128 * 1024
        assert plan[(0, 1, psv.PSV_OP_ATTN)]["bytes"] == 2 * 299 * 2 * (128 + 4) * 2
        st = psv.psv_get_stats(s.ctx)
        assert st["weight_bytes_per_layer"] == w.weight_bytes_per_layer
        assert st["kv_bytes_per_layer"] == w.kv_bytes_per_layer
        s.run()


def test_int8_weights_need_their_scales():
    w = W("err", 1, 512, 4, 2, 256, 2, 64, ("int8", "bf16"))
    with Session(w, seed=23) as s:
        lw = dict(s.weights[0])
        lw.pop("s_down")
        with pytest.raises(psv.PsvError):
            psv.psv_set_layer_weights(s.ctx, 0, lw)


# ----------------------------------------------------------------------------- full-size shapes

BENCH_POLICY = dict(mode=1, budget_bytes=64 << 20, cu_budget=256)


def test_c2_int8_whole_step_32_layers():
    w = synth.WORKLOADS["c2"].scaled(weight_format="int8", kv_format="int8")
    check_step(w, seed=2501, policy=psv.prefetch_policy(**BENCH_POLICY))


@pytest.mark.parametrize("name", ["c3", "c4", "c5"])
def test_large_shapes_single_layers_int8(name):
    w = synth.WORKLOADS[name].scaled(weight_format="int8", kv_format="int8")
    pol = psv.prefetch_policy(partial=1 if w.paged else 0, **BENCH_POLICY)
    check_step(w, seed=2501, policy=pol, layers=[0], lb=0, le=1)
