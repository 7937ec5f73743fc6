"""GPU tests of the matrix-core path stage by stage: each projection's result, read back through the debug interface,
against the oracle's fp64 projection of the *GPU's own* input to that stage, so that one stage's error is seen alone and
held to what its arithmetic allows -- far below the end-to-end bar of 2e-2 + 1e-2*|ref|, which a wrong scale or a
dropped low-order plane could still pass.

bf16 weights: the operand is carried as two bf16 planes (hi + lo, 16 significant bits per element), sums in fp32: relative
rms error of a projection <= 2e-5 (measured 2e-7 .. 4e-6).
int8 weights: the operand is two int8 digits per element with one scale per 128 elements, x ~ s*(d1 + d2/254) with
s = max|block|/127, i.e. a uniform step of max|block|/32258: an error of rms step/sqrt(12) = 8.9e-6*max|block| per element.
For blocks of 128 roughly Gaussian values (max about 2.8 sigma) that is 2.5e-5 of the operand's rms, and the projection's
relative error equals the operand's; heavier-tailed operands (silu(gate)*up) come to 5e-5.  The test restates the digit rule
in numpy, requires the GPU's QKV error to agree with that model within a factor 1.5 either way (a missing second digit
would be 250 times larger, a third one not needed), and bounds every stage by 1.5e-4."""
import numpy as np
import pytest

import oracle
from paper_2501_08192_amd import binding as psv
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session

pytestmark = pytest.mark.gpu

SCALE_OF = {"w_qkv": "s_qkv", "w_o": "s_o", "w_gate": "s_gate", "w_up": "s_up", "w_down": "s_down"}


def rel_rms(got, ref):
    return float(np.sqrt(((got - ref) ** 2).mean()) / np.sqrt((ref ** 2).mean()))


def digit_planes(h):
    """[B, K] fp64 -> the value the two-digit operand stands for (blocks of 128 along K)."""
    B = h.shape[0]
    blk = h.reshape(B, -1, 128)
    sc = np.abs(blk).max(-1, keepdims=True) / 127.0
    sc[sc == 0.0] = 1.0
    d1 = np.rint(blk / sc)
    d2 = np.clip(np.rint((blk / sc - d1) * 254.0), -127, 127)
    return (sc * (d1 + d2 / 254.0)).reshape(B, -1)


# name, H, nq, nkv, F, batch, context, paged, layout, weight format
CASES = [
    ("tp4_b8", 8192, 16, 2, 7168, 8, 17, True, "row", "bf16"),
    ("tp4_b32_tiled", 8192, 16, 2, 7168, 32, 40, False, "tiled", "bf16"),
    ("tp8_b3", 8192, 8, 1, 3584, 3, 70, False, "tiled", "bf16"),
    ("w8_tp4_b8", 8192, 16, 2, 7168, 8, 17, True, "row", "int8"),
    ("w8_tp4_b32_tiled", 8192, 16, 2, 7168, 32, 40, False, "tiled", "int8"),
    ("w8_tp8_b16", 8192, 8, 1, 3584, 16, 70, True, "tiled", "int8"),
    ("w8_ragged_b5", 1536, 12, 4, 6144, 5, 33, False, "row", "int8"),
    ("b40_three_tiles", 4096, 8, 2, 3584, 40, 33, True, "tiled", "bf16"),
    ("w8_b40_three_tiles", 4096, 8, 2, 3584, 40, 33, True, "tiled", "int8"),
    ("w8_b64_row", 2048, 16, 4, 5632, 64, 20, False, "row", "int8"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_each_projection_alone_against_fp64_from_its_own_input(case):
    name, H, nq, nkv, F, B, T, paged, layout, wfmt = case
    w = synth.Workload(name, 1, H, nq, nkv, 128, F, B, T, paged, (6.0, 6.0), 1e-5, 500000.0, wfmt, "bf16", "head", layout)
    with Session(w, seed=259) as s:
        lw = s.host_layer(0)
        x = s.x_in.cpu().numpy().astype(np.float64)
        out = s.run().cpu().numpy().astype(np.float64)
        QR = (nq + 2 * nkv) * 128
        rd = lambda which, cols: psv.psv_debug_read(s.ctx, which, np.zeros((B, cols), np.float32)).astype(np.float64)
        qkv, att, y, m = rd(psv.PSV_DBG_QKV, QR), rd(psv.PSV_DBG_ATTN, nq * 128), rd(psv.PSV_DBG_Y, H), rd(psv.PSV_DBG_M, F)

    def lin(n, v):
        if wfmt == "int8":
            return oracle.linear_q8(lw[n], lw[SCALE_OF[n]], v)
        return oracle.linear(lw[n], v)

    def rows(n, mat):
        return np.stack([lin(n, mat[b]) for b in range(B)])

    h1 = np.stack([oracle.rmsnorm(x[b], lw["g_attn"], w.rms_eps) for b in range(B)])
    h2 = np.stack([oracle.rmsnorm(y[b], lw["g_mlp"], w.rms_eps) for b in range(B)])
    r_qkv = rows("w_qkv", h1)
    g = rows("w_gate", h2)
    r_m = g / (1.0 + np.exp(-g)) * rows("w_up", h2)
    errs = {
        "qkv": rel_rms(qkv, r_qkv),
        "o": rel_rms(y - x, rows("w_o", att)),
        "gate_up": rel_rms(m, r_m),
        "down": rel_rms(out - y, rows("w_down", m)),
    }
    bound = 1.5e-4 if wfmt == "int8" else 2e-5
    for stage, e in errs.items():
        assert np.isfinite(e) and e <= bound, "%s %s: relative rms error %.3g above %.3g" % (name, stage, e, bound)
    if wfmt == "int8":
        model = rel_rms(rows("w_qkv", digit_planes(h1)), r_qkv)
        assert model / 1.5 <= errs["qkv"] <= model * 1.5, "%s: QKV error %.3g, two-digit operand model %.3g" % (
            name, errs["qkv"], model)
