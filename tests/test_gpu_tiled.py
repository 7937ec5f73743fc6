"""GPU tests of the tiled weight layout (weight_layout = PSV_W_TILED): the conversion kernel against the layout written
out here from its definition (bit for bit), and decode steps on tiled weights through the C ABI against the CPU oracle
(which always reads the row-major matrices): residual stream within |gpu - ref| <= 2e-2 + 1e-2*|ref|, every policy
bit-identical to prefetch off, and -- where both layouts run the matrix-core projections -- bit-identical to the
row-major run of the same weights (same kernels, same order of arithmetic; only the addresses differ)."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_parity as bf
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session, default_policy

pytestmark = pytest.mark.gpu


def tiled_index(rows, cols, elem_bytes):
    """For every element of the tiled copy, the flat index of the row-major element stored there."""
    per16 = 16 // elem_bytes                       # elements per 16-byte piece
    n_slabs = cols // 64
    out = np.empty(rows * cols, dtype=np.int64)
    pos = 0
    for tile in range(rows // 128):
        for slab in range(n_slabs):
            for wave in range(4):
                for group in range(2):
                    for half in range(2 if elem_bytes == 2 else 1):
                        for lane in range(64):
                            row = tile * 128 + wave * 32 + group * 16 + lane % 16
                            col = slab * 64 + (half * 32 + (lane // 16) * 8 if elem_bytes == 2 else (lane // 16) * 16)
                            out[pos:pos + per16] = row * cols + col + np.arange(per16)
                            pos += per16
    assert pos == rows * cols
    return out


@pytest.mark.parametrize("fmt", ["bf16", "int8"])
@pytest.mark.parametrize("shape", [(128, 64), (256, 192), (384, 1024)])
def test_tile_weights_is_the_documented_permutation(shape, fmt):
    rows, cols = shape
    n = rows * cols
    if fmt == "bf16":
        src = (torch.arange(n, dtype=torch.int32) % 65521).to(torch.int16).view(torch.bfloat16).reshape(rows, cols).cuda()
    else:
        src = ((torch.arange(n, dtype=torch.int64) * 37) % 251 - 125).to(torch.int8).reshape(rows, cols).cuda()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()                                      # src is complete before another stream reads it
    stream = torch.cuda.Stream()
    psv.psv_tile_weights(dst, src, rows, cols, fmt, stream)
    stream.synchronize()
    idx = tiled_index(rows, cols, 2 if fmt == "bf16" else 1)
    assert len(np.unique(idx)) == n                               # a permutation
    want = synth.bits(src).reshape(-1)[idx]
    assert np.array_equal(synth.bits(dst).reshape(-1), want)


def W(name, L, H, nq, nkv, F, B, T, paged=False, win=(5.0, 5.0), layout="tiled", fmts=("bf16", "bf16")):
    return synth.Workload(name, L, H, nq, nkv, 128, F, B, T, paged, win, 1e-5, 500000.0, fmts[0], fmts[1], "head", layout)


CASES = [
    ("b3", 2, 1024, 8, 2, 768, 3, 90, False, ("bf16", "bf16")),
    ("b8_wide", 1, 8192, 8, 1, 3584, 8, 200, True, ("bf16", "bf16")),       # the 70B-shaped TP=8 shard
    ("b17", 2, 1536, 6, 3, 1280, 17, 40, True, ("bf16", "bf16")),           # two batch tiles, odd row-tile counts
    ("b64", 1, 2048, 4, 1, 1792, 64, 33, False, ("bf16", "bf16")),
    ("b5_int8", 2, 1024, 8, 2, 768, 5, 129, True, ("int8", "int8")),
    ("b32_w8", 1, 4096, 4, 1, 1792, 32, 50, False, ("int8", "bf16")),
    ("b1", 2, 1024, 8, 8, 2816, 1, 256, False, ("bf16", "bf16")),           # batch 1 on tiled weights: matrix-core projections
    ("b2_int8", 1, 512, 4, 2, 256, 2, 17, False, ("int8", "bf16")),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tiled_weights_match_oracle_policies_and_the_row_major_run(case):
    name, L, H, nq, nkv, F, B, T, paged, fmts = case
    w = W(name, L, H, nq, nkv, F, B, T, paged=paged, fmts=fmts)
    m = oracle.model(H, nq, nkv, 128, F, 16, w.rms_eps, w.rope_theta)
    fn = oracle.decode_layer if fmts == ("bf16", "bf16") else oracle.decode_layer_x
    with Session(w, seed=83) as s:
        lens = s.seq_lens_host.numpy()
        pt = s.page_table_host.numpy() if paged else None
        x = s.x_in.cpu().numpy().astype(np.float64)
        for l in s.layers:
            kp, vp = s.host_pools(l)
            x = fn(m, s.host_layer(l), kp, vp, pt, w.blocks_per_seq, lens, x)
        off = s.run().clone()
        bf.assert_close(off.cpu().numpy(), x, name + " tiled")
        assert psv.psv_debug_last_step_path(s.ctx) == 0
        pools = [s.k_pools[l].clone() for l in s.layers] + [s.v_pools[l].clone() for l in s.layers]
        big = 1 << 40
        for pol in (default_policy(w, budget_bytes=big), default_policy(w, budget_bytes=big, prelaunch=0),
                    default_policy(w, budget_bytes=max(1 << 16, w.weight_bytes_per_layer // 3), partial=1)):
            s.set_policy(pol)
            assert torch.equal(s.run(), off), "%s: a policy changes the result" % name
            for a, b in zip(pools, [s.k_pools[l] for l in s.layers] + [s.v_pools[l] for l in s.layers]):
                assert torch.equal(a, b)
    wr = W(name, L, H, nq, nkv, F, B, T, paged=paged, fmts=fmts, layout="row")
    with Session(wr, seed=83) as r:
        row = r.run().clone()
        if B >= 3 or (B == 2 and H > 4096):
            assert torch.equal(row, off), "%s: tiled and row-major runs of the matrix-core path differ" % name
        else:                                                      # row-major runs the vector-ALU projections here
            assert torch.allclose(row, off, rtol=1e-4, atol=1e-4)
