"""GPU parity of the token-major KV-cache layout (both pools [block, token, kv head, channel]; bf16 cache) against the
CPU oracle's token-major switch, through the C ABI: residual stream within |gpu - ref| <= 2e-2 + 1e-2*|ref|, the
appended rows at their token-major addresses (restated here from the layout) and nothing else touched, every policy
bit-identical to prefetch off, and -- same logical cache in both layouts -- bit-identical to the head-major run
(the kernels walk the tokens in the same order)."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_parity as bf
from helpers import from_bits
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session, default_policy

pytestmark = pytest.mark.gpu


def W(name, L, H, nq, nkv, F, B, T, paged=False, win=(5.0, 5.0), layout="token", wfmt="bf16"):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, win, 1e-5, 500000.0, wfmt, "bf16", layout)


CASES = [
    W("tm_b1", 2, 1024, 8, 2, 768, 1, 300),                 # vector projections, two local kv heads
    W("tm_b2", 2, 1024, 8, 8, 512, 2, 77),                  # G = 1, eight kv heads
    W("tm_b5", 2, 1024, 8, 2, 768, 5, 129, paged=True),     # matrix-core projections, paged
    W("tm_b17", 1, 512, 16, 1, 256, 17, 40, paged=True),    # G = 16, one kv head (K layouts coincide, V differs)
    W("tm_long", 1, 512, 6, 3, 256, 2, 5000),               # many chunks, several tiles per wave
    W("tm_w8", 2, 1024, 8, 2, 768, 3, 90, wfmt="int8"),     # int8 weights with a token-major bf16 cache
]


@pytest.mark.parametrize("w", CASES, ids=[w.name for w in CASES])
def test_token_major_matches_oracle_and_policies_agree(w):
    m = oracle.model(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, 16, w.rms_eps, w.rope_theta, kv_token_major=True)
    with Session(w, seed=71, pool_slack_blocks=3 if w.paged else 0) as s:
        lens = s.seq_lens_host.numpy()
        if w.batch >= 5:                                      # mixed lengths on the larger batches
            lens = np.array([max(1, w.context - 13 * b) for b in range(w.batch)], dtype=np.int32)
            s.seq_lens.copy_(torch.from_numpy(lens))
        pt = s.page_table_host.numpy() if w.paged else None
        x = s.x_in.cpu().numpy().astype(np.float64)
        before = {l: (synth.bits(s.k_pools[l]).copy(), synth.bits(s.v_pools[l]).copy()) for l in s.layers}
        ref = {}
        for l in s.layers:
            kp, vp = s.host_pools(l)
            x = oracle.decode_layer_x(m, s.host_layer(l), kp, vp, pt, w.blocks_per_seq, lens, x)
            ref[l] = (kp, vp)
        off = s.run().clone()
        bf.assert_close(off.cpu().numpy(), x, w.name)
        for l in s.layers:
            kg, vg = synth.bits(s.k_pools[l]), synth.bits(s.v_pools[l])
            mask = np.zeros(kg.shape, bool)                   # [block, token, kv head, channel]
            for b in range(w.batch):
                t = int(lens[b]) - 1
                blk = int(pt[b, t // 16]) if pt is not None else b * w.blocks_per_seq + t // 16
                mask[blk, t % 16, :, :] = True
            for got, (kb_, ref_) in ((kg, (before[l][0], ref[l][0])), (vg, (before[l][1], ref[l][1]))):
                assert np.array_equal(got[~mask], kb_[~mask]), "cache touched outside the new rows"
                bf.assert_close(from_bits(got[mask]), from_bits(ref_[mask]), "append of layer %d" % l)
                if l == s.layers[0] and w.batch <= 4:
                    assert (np.abs(from_bits(got[mask]) - from_bits(ref_[mask])) <= 2.0 ** -7 * np.abs(from_bits(ref_[mask])) + 1e-4).all()
        snap = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        big = 1 << 40
        for pol in (default_policy(w, budget_bytes=big), default_policy(w, budget_bytes=big, prelaunch=0),
                    psv.prefetch_policy(mode=1, targets=psv.PSV_TARGET_KV, budget_bytes=1 << 20, partial=1, chunk_bytes=1 << 16)):
            s.set_policy(pol)
            assert torch.equal(s.run(), off)
            for a, b in zip(snap, [s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers]):
                assert torch.equal(a, b)


def test_token_major_equals_head_major_on_the_same_logical_cache():
    wt = W("tm_same", 2, 1024, 8, 2, 768, 3, 200, paged=True)
    wh = W("tm_same", 2, 1024, 8, 2, 768, 3, 200, paged=True, layout="head")
    with Session(wt, seed=72) as a, Session(wh, seed=72) as b:
        for l in a.layers:           # a's cache content, re-laid out head-major: K [blk, kvh, tok, ch], V [blk, kvh, ch, tok]
            b.k_pools[l].copy_(a.k_pools[l].permute(0, 2, 1, 3))
            b.v_pools[l].copy_(a.v_pools[l].permute(0, 2, 3, 1))
        xa, xb = a.run().clone(), b.run().clone()
        assert torch.equal(xa, xb)
        for l in a.layers:
            assert torch.equal(a.k_pools[l].permute(0, 2, 1, 3), b.k_pools[l])
            assert torch.equal(a.v_pools[l].permute(0, 2, 3, 1), b.v_pools[l])


def test_token_major_is_refused_for_an_int8_cache():
    d = psv.model_desc(2, 512, 4, 2, 256, 2, 64, kv_format="int8", kv_layout="token")
    assert psv.psv_validate_desc(d) == psv.PSV_ERR_INVALID_ARG
    d = psv.model_desc(2, 512, 4, 2, 256, 2, 64, kv_layout="token")
    assert psv.psv_validate_desc(d) == psv.PSV_OK
    d.kv_layout = 2
    assert psv.psv_validate_desc(d) == psv.PSV_ERR_INVALID_ARG
