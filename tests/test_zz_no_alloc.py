"""The entry point that allocates nothing (psv_decode_step_static: workspace in a fixed device array inside the
library) against psv_decode_step on a created context, through the C ABI: same inputs, policy off and no windows
on the context, results and appended cache rows must agree bit for bit.  Two calls in a row share the one array,
the second with a smaller input, so stale contents of the first would show."""
import pytest
import torch

from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session

pytestmark = pytest.mark.gpu


def W(name, L, H, nq, nkv, F, B, T, paged=False, fmt=("bf16", "bf16")):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, (0.0, 0.0), 1e-5, 500000.0, fmt[0], fmt[1])


def run_both(w, seed):
    with Session(w, seed=seed, fused=0) as s:      # the static entry point always runs one kernel per operator
        s.set_policy(psv.prefetch_policy(mode=0))
        s.set_windows(0.0, 0.0)
        k0 = {l: s.k_pools[l].clone() for l in s.layers}
        v0 = {l: s.v_pools[l].clone() for l in s.layers}
        ref = s.run().clone()
        k_ref = {l: s.k_pools[l].clone() for l in s.layers}
        v_ref = {l: s.v_pools[l].clone() for l in s.layers}
        for l in s.layers:                      # back to the state before the step
            s.k_pools[l].copy_(k0[l])
            s.v_pools[l].copy_(v0[l])
        out = torch.full_like(s.x_in, float("nan"))
        torch.cuda.synchronize()
        stream = torch.cuda.Stream()
        L = w.n_layers
        psv.psv_decode_step_static(s.desc, [s.weights[l] for l in range(L)], [s.k_pools[l] for l in range(L)],
                                   [s.v_pools[l] for l in range(L)], s.page_table, w.blocks_per_seq, s.pool_blocks,
                                   s.seq_lens, s.x_in, out, w.batch, 0, L, stream)
        stream.synchronize()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), "%s: static workspace and created context differ" % w.name
        for l in s.layers:
            assert torch.equal(s.k_pools[l], k_ref[l]) and torch.equal(s.v_pools[l], v_ref[l])
            assert not torch.equal(s.k_pools[l], k0[l])


def test_static_workspace_matches_created_context_two_calls_second_smaller():
    # batch 5 on the matrix-core path with a paged cache and many attention chunks, then batch 1 on the vector path
    run_both(W("static_big", 2, 2048, 16, 2, 1792, 5, 1500, paged=True), seed=91)
    run_both(W("static_small", 2, 512, 4, 1, 256, 1, 70), seed=92)
    # int8 formats share the array as well
    run_both(W("static_q8", 1, 1024, 8, 2, 768, 3, 200, fmt=("int8", "int8")), seed=93)


def test_static_workspace_rejects_what_does_not_fit_and_bad_arguments():
    L = psv.lib()
    w = synth.WORKLOADS["c5"]
    d = psv.model_desc(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn, w.batch, w.context)
    assert psv.psv_workspace_bytes(d) > psv.PSV_STATIC_SCRATCH_BYTES
    import ctypes as C
    arr = (psv.psv_layer_weights * w.n_layers)()
    kv = psv.psv_kv_desc()
    x = torch.zeros(w.batch, w.hidden, device="cuda")
    assert L.psv_decode_step_static(C.byref(d), arr, C.byref(kv), x.data_ptr(), x.data_ptr(), w.batch, 0, 1, None) == psv.PSV_ERR_UNSUPPORTED
    assert L.psv_decode_step_static(None, arr, C.byref(kv), x.data_ptr(), x.data_ptr(), 1, 0, 1, None) == psv.PSV_ERR_INVALID_ARG
    w1 = synth.WORKLOADS["c1"]
    d1 = psv.model_desc(w1.n_layers, w1.hidden, w1.n_q_heads, w1.n_kv_heads, w1.ffn, w1.batch, w1.context)
    arr1 = (psv.psv_layer_weights * w1.n_layers)()
    assert L.psv_decode_step_static(C.byref(d1), arr1, C.byref(kv), x.data_ptr(), x.data_ptr(), 1, 0, 1, None) == psv.PSV_ERR_INVALID_ARG   # null weights
    assert L.psv_decode_step_static(C.byref(d1), arr1, C.byref(kv), x.data_ptr(), x.data_ptr(), 2, 0, 1, None) == psv.PSV_ERR_INVALID_ARG   # batch > max
