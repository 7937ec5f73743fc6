"""Pins of the int8 variant of the CPU oracle: integer brute force, the bf16 routines (already pinned) on
inputs where both formats hold the same numbers exactly, and the nearest-code property of the append rule.
CPU only."""
import numpy as np
import pytest

import oracle
from helpers import fill_pools, random_layer, to_bits

BT = 4


def q8_pools_from_dense(k_codes, k_scales, v_codes, v_scales, bt, page_table=None, n_blocks=None):
    """int8 pools in the block layout, restated from the format: per (block, kv head) bt*d code bytes
    (K: [token][channel], V: [channel][token]) followed by bt fp32 scales."""
    B, nkv, T, d = k_codes.shape
    mb = (T + bt - 1) // bt
    if n_blocks is None:
        n_blocks = B * mb
    unit = bt * d + 4 * bt
    k = np.zeros((n_blocks, nkv, unit), dtype=np.uint8)
    v = np.zeros((n_blocks, nkv, unit), dtype=np.uint8)
    for b in range(B):
        for t in range(T):
            blk = b * mb + t // bt if page_table is None else int(page_table[b, t // bt])
            r = t % bt
            for h in range(nkv):
                k[blk, h, r * d:(r + 1) * d] = k_codes[b, h, t].astype(np.int8).view(np.uint8)
                v[blk, h, r:bt * d:bt] = v_codes[b, h, t].astype(np.int8).view(np.uint8)
                k[blk, h, bt * d + 4 * r: bt * d + 4 * r + 4] = np.frombuffer(np.float32(k_scales[b, h, t]).tobytes(), dtype=np.uint8)
                v[blk, h, bt * d + 4 * r: bt * d + 4 * r + 4] = np.frombuffer(np.float32(v_scales[b, h, t]).tobytes(), dtype=np.uint8)
    return k, v


# ----------------------------------------------------------------------------- linear

def test_linear_q8_integer_brute_force():
    rng = np.random.default_rng(11)
    rows, cols = 5, 9
    w = rng.integers(-127, 128, size=(rows, cols)).astype(np.int8)
    x = rng.integers(-3, 4, size=cols)
    s = np.array([1, 2, 4, 1, 8], dtype=np.float32)
    want = np.zeros(rows, dtype=np.int64)
    for r in range(rows):
        for c in range(cols):
            want[r] += int(w[r, c]) * int(x[c])
        want[r] *= int(s[r])
    got = oracle.linear_q8(w, s, x.astype(np.float64))
    assert np.array_equal(got, want.astype(np.float64))


def test_linear_q8_equals_bf16_linear_when_both_hold_the_same_numbers():
    # |code| <= 127 has 7 significant bits: code * 2^-k is exact in bf16
    rng = np.random.default_rng(12)
    rows, cols = 6, 40
    w = rng.integers(-127, 128, size=(rows, cols)).astype(np.int8)
    s = (2.0 ** -rng.integers(3, 9, size=rows)).astype(np.float32)
    x = rng.normal(0, 1, size=cols)
    dense = w.astype(np.float64) * s[:, None].astype(np.float64)
    assert np.array_equal(np.asarray(dense, dtype=np.float32), dense)
    want = oracle.linear(to_bits(dense), x)
    got = oracle.linear_q8(w, s, x)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    assert np.abs(want).max() > 0.1


def test_linear_q8_uses_the_row_scale_not_the_column():
    w = np.ones((2, 3), dtype=np.int8)
    got = oracle.linear_q8(w, np.array([1.0, 10.0], dtype=np.float32), np.array([1.0, 2.0, 3.0]))
    assert np.array_equal(got, [6.0, 60.0])


# ----------------------------------------------------------------------------- append rule

def test_quantize_row_is_the_nearest_code_and_fills_the_range():
    rng = np.random.default_rng(13)
    for trial in range(20):
        v = rng.normal(0, 10 ** rng.uniform(-3, 2), size=32)
        codes, s = oracle.quantize_row(v)
        vf = v.astype(np.float32)
        assert s == np.float32(np.abs(vf).max() / np.float32(127.0))
        assert np.abs(codes.astype(np.int32)).max() == 127
        grid = np.arange(-127, 128, dtype=np.float64) * float(s)
        for i in range(v.size):
            best = np.abs(grid - float(vf[i]))
            assert best[int(codes[i]) + 127] <= best.min() * (1 + 1e-6) + 1e-12
        assert np.abs(codes * float(s) - vf).max() <= 0.5 * float(s) * (1 + 1e-6)


def test_quantize_row_degenerate_and_ties():
    codes, s = oracle.quantize_row(np.zeros(8))
    assert s == np.float32(1.0) and not codes.any()
    # scale = 127/127 = 1: halves are exact ties and go to the even code
    codes, s = oracle.quantize_row(np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -126.5]))
    assert s == np.float32(1.0)
    assert codes.tolist() == [127, 0, 2, 2, 0, -2, -126]
    # the largest element always maps to +-127 and nothing is clamped away from it
    codes, s = oracle.quantize_row(np.array([-3.0, 1.0, 3.0]))
    assert codes.tolist() == [-127, 42, 127]


# ----------------------------------------------------------------------------- attention

def _exact_cache(rng, B, nkv, T, d):
    kc = rng.integers(-127, 128, size=(B, nkv, T, d))
    vc = rng.integers(-127, 128, size=(B, nkv, T, d))
    ks = 2.0 ** -rng.integers(5, 8, size=(B, nkv, T))
    vs = 2.0 ** -rng.integers(5, 8, size=(B, nkv, T))
    return kc, ks, vc, vs


@pytest.mark.parametrize("paged", [False, True])
def test_attention_q8_equals_bf16_attention_when_both_hold_the_same_numbers(paged):
    rng = np.random.default_rng(14)
    B, nq, nkv, d, T = 2, 4, 2, 8, 11
    m = oracle.model(16, nq, nkv, d, 16, block_tokens=BT, rope_theta=0.0)
    mb = (T + BT - 1) // BT
    pt = None
    n_blocks = B * mb
    if paged:
        n_blocks = B * mb + 3
        pt = rng.permutation(n_blocks)[:B * mb].reshape(B, mb).astype(np.int32)
    kc, ks, vc, vs = _exact_cache(rng, B, nkv, T, d)
    k8, v8 = q8_pools_from_dense(kc, ks, vc, vs, BT, pt, n_blocks)
    k16, v16 = fill_pools(kc * ks[..., None], vc * vs[..., None], BT, pt, n_blocks)
    lens = np.array([T, T - 3], dtype=np.int32)
    for b in range(B):
        for j in range(nq):
            q = rng.normal(0, 1, size=d)
            want = oracle.attention_head(m, k16, v16, pt, mb, lens, b, j, q)
            got = oracle.attention_head_q8(m, k8, v8, pt, mb, lens, b, j, q)
            np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_attention_q8_applies_each_tokens_own_scale():
    # two tokens, same codes, key scales far apart: the softmax must follow the scaled scores, and the
    # output the scaled values
    d = 4
    m = oracle.model(8, 1, 1, d, 8, block_tokens=BT, rope_theta=0.0)
    kc = np.ones((1, 1, 2, d), dtype=np.int64)
    vc = np.ones((1, 1, 2, d), dtype=np.int64)
    ks = np.array([[[0.0, 2.0]]])
    vs = np.array([[[1.0, 3.0]]])
    k8, v8 = q8_pools_from_dense(kc, ks, vc, vs, BT)
    out = oracle.attention_head_q8(m, k8, v8, None, 1, np.array([2], dtype=np.int32), 0, 0, np.ones(d))
    s1 = 4 * 2.0 / 2.0                      # q.k1 * k_scale / sqrt(d); token 0 scores 0
    p1 = np.exp(s1) / (1 + np.exp(s1))
    np.testing.assert_allclose(out, np.full(d, (1 - p1) * 1.0 + p1 * 3.0), rtol=1e-12)


# ----------------------------------------------------------------------------- layer

def _exact_q8_layer(rng, H, nq, nkv, d, F):
    """int8 weights whose dequantised values are exact in bf16, and the same numbers as bf16 bits."""
    def draw(rows, cols):
        codes = rng.integers(-127, 128, size=(rows, cols)).astype(np.int8)
        scale = (2.0 ** -rng.integers(8, 11, size=rows)).astype(np.float32)
        return codes, scale
    shapes = {"w_qkv": ((nq + 2 * nkv) * d, H), "w_o": (H, nq * d), "w_gate": (F, H), "w_up": (F, H), "w_down": (H, F)}
    q8, bf = {}, {}
    for n, (r, c) in shapes.items():
        codes, scale = draw(r, c)
        q8[n] = codes
        q8["s_" + n[2:]] = scale
        bf[n] = to_bits(codes.astype(np.float64) * scale[:, None])
    for n in ("g_attn", "g_mlp"):
        g = to_bits(1.0 + rng.normal(0, 0.1, size=H))
        q8[n] = g
        bf[n] = g
    return q8, bf


def test_layer_x_with_bf16_formats_is_the_bf16_layer():
    rng = np.random.default_rng(15)
    H, nq, nkv, d, F, B, T = 16, 4, 2, 8, 24, 2, 6
    m = oracle.model(H, nq, nkv, d, F, block_tokens=BT)
    w = random_layer(rng, H, nq, nkv, d, F)
    kd, vd = rng.normal(0, 1, (B, nkv, T, d)), rng.normal(0, 1, (B, nkv, T, d))
    k0, v0 = fill_pools(kd, vd, BT)
    x = rng.normal(0, 1, (B, H))
    lens = np.array([T, T - 1], dtype=np.int32)
    ka, va, kb, vb = k0.copy(), v0.copy(), k0.copy(), v0.copy()
    want = oracle.decode_layer(m, w, ka, va, None, (T + BT - 1) // BT, lens, x)
    got = oracle.decode_layer_x(m, w, kb, vb, None, (T + BT - 1) // BT, lens, x)
    assert np.array_equal(got, want)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)


def test_layer_x_with_int8_weights_equals_the_bf16_layer_on_the_same_numbers():
    rng = np.random.default_rng(16)
    H, nq, nkv, d, F, B, T = 16, 4, 2, 8, 24, 2, 7
    m = oracle.model(H, nq, nkv, d, F, block_tokens=BT)
    q8, bf = _exact_q8_layer(rng, H, nq, nkv, d, F)
    kd, vd = rng.normal(0, 1, (B, nkv, T, d)), rng.normal(0, 1, (B, nkv, T, d))
    k0, v0 = fill_pools(kd, vd, BT)
    x = rng.normal(0, 1, (B, H))
    lens = np.array([T, T], dtype=np.int32)
    ka, va, kb, vb = k0.copy(), v0.copy(), k0.copy(), v0.copy()
    want = oracle.decode_layer(m, bf, ka, va, None, (T + BT - 1) // BT, lens, x)
    got = oracle.decode_layer_x(m, q8, kb, vb, None, (T + BT - 1) // BT, lens, x)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-11)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    assert np.abs(want - x).max() > 1e-3          # the layer did something


def test_layer_x_int8_cache_appends_the_quantised_row_and_stays_close_to_the_bf16_cache_layer():
    rng = np.random.default_rng(17)
    H, nq, nkv, d, F, B, T = 16, 4, 2, 8, 24, 2, 9
    m = oracle.model(H, nq, nkv, d, F, block_tokens=BT)
    w = random_layer(rng, H, nq, nkv, d, F)
    mb = (T + BT - 1) // BT
    kc, ks, vc, vs = _exact_cache(rng, B, nkv, T, d)
    k8, v8 = q8_pools_from_dense(kc, ks, vc, vs, BT)
    k16, v16 = fill_pools(kc * ks[..., None], vc * vs[..., None], BT)
    x = rng.normal(0, 1, (B, H))
    lens = np.array([T, T - 2], dtype=np.int32)
    k8_before = k8.copy()
    want = oracle.decode_layer(m, w, k16, v16, None, mb, lens, x)
    got = oracle.decode_layer_x(m, w, k8, v8, None, mb, lens, x)
    # only the appended slots (codes of one row + its scale) changed
    changed = np.argwhere(k8 != k8_before)
    for blk, h, byte in changed:
        b = blk // mb
        r = (int(lens[b]) - 1) % BT
        assert blk == b * mb + (int(lens[b]) - 1) // BT
        assert r * d <= byte < (r + 1) * d or BT * d + 4 * r <= byte < BT * d + 4 * r + 4
    # appended key = quantisation of what the bf16 layer appended (up to its own bf16 rounding)
    unit_k = k8[0 * mb + (T - 1) // BT, 0]
    r = (T - 1) % BT
    codes = unit_k[r * d:(r + 1) * d].view(np.int8).astype(np.float64)
    scale = np.frombuffer(unit_k[BT * d + 4 * r: BT * d + 4 * r + 4].tobytes(), dtype=np.float32)[0]
    from helpers import from_bits
    k_bf16 = from_bits(k16[0 * mb + (T - 1) // BT, 0, r, :])
    assert np.abs(codes).max() == 127
    assert np.abs(codes * scale - k_bf16).max() <= 0.5 * scale + 2.0 ** -8 * np.abs(k_bf16).max()
    # one of T tokens differs by at most half a code step: the layer output moves only slightly
    assert np.abs(got - want).max() < 0.05
    assert np.abs(got - want).max() > 0.0
