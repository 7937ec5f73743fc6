"""Pins of the CPU oracle against things other than itself: closed forms, textbook identities,
exact integer brute force and PyTorch's own float64 library routines.  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from helpers import (dense_from_pools, empty_pools, fill_pools, from_bits, random_layer, to_bits)

BT = 4   # tokens per block in the tiny cases (the oracle takes any block size)


# ----------------------------------------------------------------------------- bf16

def test_bf16_widening_and_rounding_match_torch():
    rng = np.random.default_rng(1)
    vals = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 1e-3, 1000), rng.normal(0, 300, 1000),
                           [0.0, -0.0, 1.0, -1.0, 65504.0, 1e-40]]).astype(np.float32)
    # exact ties between two bf16 values: mantissa tail 0x8000 on odd and even neighbours
    ties = np.array([0x3F808000, 0x3F818000, 0xBF808000, 0x40FF8000, 0x3F7F8000], dtype=np.uint32).view(np.float32)
    vals = np.concatenate([vals, ties])
    want = to_bits(vals)
    got = np.array([oracle.f64_to_bf16(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([oracle.bf16_to_f64(int(b)) for b in want])
    assert np.array_equal(back, from_bits(want))


def test_bf16_tie_goes_to_even():
    # 1 + 2^-8 lies exactly between bf16(1.0)=0x3F80 and 0x3F81 -> even mantissa 0x3F80
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    # 1 + 3*2^-8 lies between 0x3F81 and 0x3F82 -> 0x3F82
    assert oracle.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82


# ----------------------------------------------------------------------------- linear

def test_linear_integer_brute_force():
    rng = np.random.default_rng(2)
    rows, cols = 7, 13                      # non-square: a transposed operand cannot pass
    w = rng.integers(-4, 5, size=(rows, cols))
    x = rng.integers(-4, 5, size=cols)
    want = np.zeros(rows, dtype=np.int64)
    for r in range(rows):
        for c in range(cols):
            want[r] += int(w[r, c]) * int(x[c])
    got = oracle.linear(to_bits(w), x.astype(np.float64))
    assert np.array_equal(got, want.astype(np.float64))


# ----------------------------------------------------------------------------- RMSNorm

def test_rmsnorm_closed_form_constant_magnitude():
    n, c, eps = 8, 3.0, 1e-5
    signs = np.array([1, -1, 1, 1, -1, -1, 1, -1], dtype=np.float64)
    gain = np.array([1.0, 0.5, 2.0, 1.0, 1.5, 1.0, 0.25, 1.0])
    got = oracle.rmsnorm(c * signs, to_bits(gain), eps)
    want = signs * gain * c / math.sqrt(c * c + eps)
    assert np.allclose(got, want, rtol=0, atol=1e-15)


def test_rmsnorm_matches_torch_library():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 2.0, 64)
    g = to_bits(1 + rng.normal(0, 0.1, 64))
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(from_bits(g)), eps=1e-5).numpy()
    assert np.allclose(oracle.rmsnorm(x, g, 1e-5), want, rtol=1e-13, atol=1e-14)


def test_rmsnorm_scale_invariant_without_eps():
    rng = np.random.default_rng(4)
    x = rng.normal(0, 1, 32)
    g = to_bits(np.ones(32))
    assert np.allclose(oracle.rmsnorm(x, g, 0.0), oracle.rmsnorm(7.5 * x, g, 0.0), rtol=1e-13)


# ----------------------------------------------------------------------------- RoPE

def test_rope_position_zero_is_identity():
    v = np.arange(1.0, 9.0)
    assert np.array_equal(oracle.rope(v, 0, 500000.0), v)


def test_rope_theta_zero_disables():
    v = np.arange(1.0, 9.0)
    assert np.array_equal(oracle.rope(v, 17, 0.0), v)


def test_rope_closed_form_d2():
    # single pair, frequency theta^0 = 1: (1,0) at position 1 -> (cos 1, sin 1)
    got = oracle.rope(np.array([1.0, 0.0]), 1, 10000.0)
    assert np.allclose(got, [0.5403023058681398, 0.8414709848078965], atol=1e-15)
    got = oracle.rope(np.array([0.0, 1.0]), 1, 10000.0)
    assert np.allclose(got, [-0.8414709848078965, 0.5403023058681398], atol=1e-15)


def test_rope_closed_form_d4_second_frequency_and_pairing():
    # d=4, theta=1e4: pair (1,3) turns at theta^(-2/4) = 0.01 rad/position; at position 100 -> 1 rad.
    got = oracle.rope(np.array([0.0, 1.0, 0.0, 0.0]), 100, 10000.0)
    assert np.allclose(got, [0.0, math.cos(1.0), 0.0, math.sin(1.0)], atol=1e-12)
    # pair (0,2) turns at 1 rad/position
    got = oracle.rope(np.array([1.0, 0.0, 0.0, 0.0]), 2, 10000.0)
    assert np.allclose(got, [math.cos(2.0), 0.0, math.sin(2.0), 0.0], atol=1e-12)


def test_rope_preserves_norm_and_relative_inner_product():
    rng = np.random.default_rng(5)
    q, k = rng.normal(0, 1, 16), rng.normal(0, 1, 16)
    th = 500000.0
    assert math.isclose(np.linalg.norm(oracle.rope(q, 1234, th)), np.linalg.norm(q), rel_tol=1e-12)
    a = oracle.rope(q, 40, th) @ oracle.rope(k, 33, th)
    b = oracle.rope(q, 1007, th) @ oracle.rope(k, 1000, th)
    assert math.isclose(a, b, rel_tol=1e-9, abs_tol=1e-9)
    # same position on both sides leaves the inner product unchanged
    assert math.isclose(oracle.rope(q, 77, th) @ oracle.rope(k, 77, th), q @ k, rel_tol=1e-10, abs_tol=1e-10)


def test_rope_matches_complex_rotation():
    rng = np.random.default_rng(6)
    d, pos, th = 32, 4095, 500000.0
    v = rng.normal(0, 1, d)
    z = v[: d // 2] + 1j * v[d // 2:]
    ang = pos * th ** (-np.arange(d // 2) * 2.0 / d)
    z = z * np.exp(1j * ang)
    assert np.allclose(oracle.rope(v, pos, th), np.concatenate([z.real, z.imag]), atol=1e-9)


# ----------------------------------------------------------------------------- softmax / SiLU

def test_softmax_rows_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(7)
    s = rng.normal(0, 3, 257)
    p = oracle.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-12 and (p > 0).all()
    assert np.allclose(oracle.softmax(s + 123.25), p, rtol=1e-12, atol=0)
    assert np.allclose(oracle.softmax(np.array([1000.0, 1000.0])), [0.5, 0.5])


def test_softmax_two_element_closed_form():
    p = oracle.softmax(np.array([1.0, 0.0]))
    assert np.allclose(p, [1 / (1 + math.exp(-1.0)), 1 / (1 + math.e)], atol=1e-15)


def test_silu_identities():
    assert oracle.silu(0.0) == 0.0
    for z in (-3.0, -0.5, 0.25, 2.0, 9.0):
        assert math.isclose(oracle.silu(z), z * 0.5 * (1 + math.tanh(z / 2)), rel_tol=1e-13)
        assert math.isclose(oracle.silu(z), float(F.silu(torch.tensor(z, dtype=torch.float64))), rel_tol=1e-13)
    assert math.isclose(oracle.silu(40.0), 40.0, rel_tol=1e-15)
    assert abs(oracle.silu(-40.0)) < 1e-15


# ----------------------------------------------------------------------------- attention

def _model(H=8, nq=2, nkv=1, d=4, F_=6, theta=0.0):
    return oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rms_eps=1e-5, rope_theta=theta)


def test_attention_sigmoid_closed_form_pins_the_scale():
    # d=4, q=(2,0,0,0); k0=(1,0,0,0), k1=0: scores (2*1/sqrt(4), 0) = (1, 0) -> p = (sigmoid(1), 1-sigmoid(1)).
    m = _model(nq=1, nkv=1)
    kd = np.zeros((1, 1, 2, 4)); vd = np.zeros((1, 1, 2, 4))
    kd[0, 0, 0, 0] = 1.0
    vd[0, 0, 0] = [1, 0, 0, 0]
    vd[0, 0, 1] = [0, 1, 0, 0]
    k, v = fill_pools(kd, vd, BT)
    out = oracle.attention_head(m, k, v, None, 1, [2], 0, 0, np.array([2.0, 0, 0, 0]))
    sg = 0.7310585786300049
    assert np.allclose(out, [sg, 1 - sg, 0, 0], atol=1e-15)


def test_attention_identical_keys_returns_mean_of_values():
    m = _model(nq=1, nkv=1)
    rng = np.random.default_rng(8)
    T = 16
    kd = np.tile(rng.integers(-2, 3, size=(1, 1, 1, 4)).astype(np.float64), (1, 1, T, 1))
    vd = rng.integers(-4, 5, size=(1, 1, T, 4)).astype(np.float64)
    k, v = fill_pools(kd, vd, BT)
    out = oracle.attention_head(m, k, v, None, T // BT, [T], 0, 0, rng.normal(0, 1, 4))
    assert np.allclose(out, vd[0, 0].mean(axis=0), atol=1e-14)


def test_attention_dominant_key_selects_its_value_row():
    m = _model(nq=1, nkv=1)
    T = 9                                    # ragged: last block holds one token
    kd = np.zeros((1, 1, T, 4)); vd = np.arange(T * 4, dtype=np.float64).reshape(1, 1, T, 4)
    kd[0, 0, 5] = [64, 0, 0, 0]
    k, v = fill_pools(kd, vd, BT)
    out = oracle.attention_head(m, k, v, None, 3, [T], 0, 0, np.array([8.0, 0, 0, 0]))
    assert np.allclose(out, vd[0, 0, 5], atol=1e-12)


def test_attention_single_token_returns_that_value():
    m = _model(nq=1, nkv=1)
    kd = np.array([[[[1.0, 2, 3, 4]]]]); vd = np.array([[[[0.5, -1.5, 2.0, 8.0]]]])
    k, v = fill_pools(kd, vd, BT)
    out = oracle.attention_head(m, k, v, None, 1, [1], 0, 0, np.array([1.0, 1, 1, 1]))
    assert np.array_equal(out, vd[0, 0, 0])


def test_attention_group_mapping_is_head_div_group():
    # 4 q heads on 2 kv heads: heads 0,1 read kv head 0 and heads 2,3 read kv head 1.
    m = _model(nq=4, nkv=2)
    T = 8
    kd = np.zeros((1, 2, T, 4))
    vd = np.zeros((1, 2, T, 4)); vd[0, 0] = 1.0; vd[0, 1] = 2.0
    k, v = fill_pools(kd, vd, BT)
    for head, want in ((0, 1.0), (1, 1.0), (2, 2.0), (3, 2.0)):
        out = oracle.attention_head(m, k, v, None, 2, [T], 0, head, np.ones(4))
        assert np.allclose(out, want)


def test_attention_reads_only_its_span_and_its_sequence():
    # tokens beyond seq_len and other sequences' blocks must not contribute
    m = _model(nq=1, nkv=1)
    kd = np.zeros((2, 1, 8, 4)); vd = np.zeros((2, 1, 8, 4))
    vd[0, 0, :5] = 1.0; vd[0, 0, 5:] = 100.0; vd[1, 0] = -7.0
    k, v = fill_pools(kd, vd, BT)
    out = oracle.attention_head(m, k, v, None, 2, [5, 8], 0, 0, np.ones(4))
    assert np.allclose(out, 1.0)
    out = oracle.attention_head(m, k, v, None, 2, [5, 8], 1, 0, np.ones(4))
    assert np.allclose(out, -7.0)


def test_attention_matches_torch_sdpa():
    rng = np.random.default_rng(9)
    B, nq, nkv, d, T = 2, 4, 2, 8, 13
    m = oracle.model(16, nq, nkv, d, 8, block_tokens=BT, rope_theta=0.0)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    k, v = fill_pools(kd, vd, BT)
    kq, vq = dense_from_pools(k, v, B, T)            # the bf16-rounded values the oracle sees
    q = rng.normal(0, 1, (B, nq, d))
    kk = torch.from_numpy(kq).repeat_interleave(nq // nkv, dim=1)
    vv = torch.from_numpy(vq).repeat_interleave(nq // nkv, dim=1)
    want = F.scaled_dot_product_attention(torch.from_numpy(q)[:, :, None, :], kk, vv)[:, :, 0, :].numpy()
    mb = (T + BT - 1) // BT
    for b in range(B):
        for j in range(nq):
            out = oracle.attention_head(m, k, v, None, mb, [T, T], b, j, q[b, j])
            assert np.allclose(out, want[b, j], rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- whole layer

def _torch_layer(m, w, kd, vd, T, x):
    """One decoder layer composed from PyTorch float64 library routines on dense caches
    [B, nkv, T, d] whose slot T-1 is overwritten.  Returns (x_out, k_new, v_new)."""
    H, nq, nkv, d = m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim
    t = lambda name: torch.from_numpy(from_bits(w[name]))
    x = torch.from_numpy(np.asarray(x, dtype=np.float64))
    B = x.shape[0]
    h = F.rms_norm(x, (H,), t("g_attn"), eps=m.rms_eps)
    qkv = F.linear(h, t("w_qkv")).reshape(B, nq + 2 * nkv, d)
    if m.rope_theta > 0:
        ang = (T - 1) * m.rope_theta ** (-torch.arange(d // 2, dtype=torch.float64) * 2.0 / d)
        rot = torch.polar(torch.ones_like(ang), ang)
        z = torch.complex(qkv[:, : nq + nkv, : d // 2], qkv[:, : nq + nkv, d // 2:]) * rot
        qkv = torch.cat([torch.cat([z.real, z.imag], dim=-1), qkv[:, nq + nkv:]], dim=1)
    q, kn, vn = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:]
    kn = kn.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    vn = vn.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    kd = torch.from_numpy(kd).clone(); vd = torch.from_numpy(vd).clone()
    kd[:, :, T - 1] = kn; vd[:, :, T - 1] = vn
    g = nq // nkv
    o = F.scaled_dot_product_attention(q[:, :, None, :], kd.repeat_interleave(g, 1), vd.repeat_interleave(g, 1))
    y = x + F.linear(o.reshape(B, nq * d), t("w_o"))
    h2 = F.rms_norm(y, (H,), t("g_mlp"), eps=m.rms_eps)
    mlp = F.linear(F.silu(F.linear(h2, t("w_gate"))) * F.linear(h2, t("w_up")), t("w_down"))
    return (y + mlp).numpy(), kn.numpy(), vn.numpy()


@pytest.mark.parametrize("theta", [0.0, 10000.0])
@pytest.mark.parametrize("nq,nkv", [(4, 2), (4, 1), (3, 3)])
def test_layer_matches_torch_library_composition(theta, nq, nkv):
    rng = np.random.default_rng(10 + nq + nkv)
    B, H, d, F_, T = 3, 24, 8, 20, 11
    m = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=theta)
    w = random_layer(rng, H, nq, nkv, d, F_, std=0.3)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    k, v = fill_pools(kd, vd, BT)
    kq, vq = dense_from_pools(k, v, B, T)
    x = rng.normal(0, 1, (B, H))
    want, kn, vn = _torch_layer(m, w, kq, vq, T, x)
    mb = (T + BT - 1) // BT
    got = oracle.decode_layer(m, w, k, v, None, mb, [T] * B, x)
    assert np.allclose(got, want, rtol=1e-11, atol=1e-12)
    k_after, v_after = dense_from_pools(k, v, B, T)
    # bf16 rounding of two float64 computations can differ by one unit in the last place when a
    # value sits within 1e-15 of a tie; none does for these seeds.
    assert np.array_equal(k_after[:, :, T - 1], kn) and np.array_equal(v_after[:, :, T - 1], vn)
    assert np.array_equal(k_after[:, :, : T - 1], kq[:, :, : T - 1])      # only the last slot changes
    assert np.array_equal(v_after[:, :, : T - 1], vq[:, :, : T - 1])


def test_layer_append_writes_selected_channels_exactly():
    # rope off; W_qkv rows are one-hot, so k and v of the new token are plain copies of h.
    rng = np.random.default_rng(11)
    H, nq, nkv, d, F_, T = 16, 2, 2, 4, 6, 6
    m = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=0.0)
    w = random_layer(rng, H, nq, nkv, d, F_)
    wq = np.zeros(((nq + 2 * nkv) * d, H))
    sel = rng.permutation(H)[: 2 * nkv * d]
    for i, c in enumerate(sel):
        wq[nq * d + i, c] = 1.0
    w["w_qkv"] = to_bits(wq)
    x = rng.normal(0, 1, (1, H))
    h = oracle.rmsnorm(x[0], w["g_attn"], 1e-5)
    k, v = empty_pools(2, nkv, BT, d)
    oracle.decode_layer(m, w, k, v, None, 2, [T], x)
    kd, vd = dense_from_pools(k, v, 1, T)
    want = from_bits(to_bits(h[sel]))
    assert np.array_equal(kd[0, :, T - 1].reshape(-1), want[: nkv * d])
    assert np.array_equal(vd[0, :, T - 1].reshape(-1), want[nkv * d:])
    assert not kd[0, :, : T - 1].any() and not vd[0, :, : T - 1].any()


def test_layer_zero_projections_give_identity_and_partial_residual():
    rng = np.random.default_rng(12)
    B, H, nq, nkv, d, F_, T = 2, 16, 4, 2, 4, 12, 7
    m = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=10000.0)
    w = random_layer(rng, H, nq, nkv, d, F_, std=0.3)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    x = rng.normal(0, 1, (B, H))
    w0 = dict(w); w0["w_o"] = np.zeros_like(w["w_o"]); w0["w_down"] = np.zeros_like(w["w_down"])
    k, v = fill_pools(kd, vd, BT)
    assert np.array_equal(oracle.decode_layer(m, w0, k, v, None, 2, [T] * B, x), x)
    # W_down = 0 only: the MLP adds nothing, the attention residual remains.
    w1 = dict(w); w1["w_down"] = np.zeros_like(w["w_down"])
    k, v = fill_pools(kd, vd, BT)
    got = oracle.decode_layer(m, w1, k, v, None, 2, [T] * B, x)
    kq, vq = dense_from_pools(*fill_pools(kd, vd, BT), B, T)
    want, _, _ = _torch_layer(m, w1, kq, vq, T, x)
    assert np.allclose(got, want, rtol=1e-11, atol=1e-12) and not np.allclose(got, x)


def test_layer_integer_attention_residual_exact():
    # Integer weights, W_gate = 0 (MLP contributes exactly 0), identical keys (softmax uniform over a
    # power-of-two span), rope off: y = x + W_o * mean(V) with V integer -> exact in binary floating point
    # up to the norm, which we remove by feeding the attention through zero q rows.
    rng = np.random.default_rng(13)
    B, H, nq, nkv, d, F_, T = 2, 8, 2, 1, 4, 6, 8
    m = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=0.0)
    w = random_layer(rng, H, nq, nkv, d, F_, integer=True)
    w["w_qkv"] = np.zeros_like(w["w_qkv"])            # q = k_new = v_new = 0
    w["w_gate"] = np.zeros_like(w["w_gate"])
    vd = rng.integers(-4, 5, size=(B, nkv, T, d)).astype(np.float64)
    vd[:, :, T - 1] = 0.0                              # the slot the step overwrites with v_new = 0
    kd = np.zeros((B, nkv, T, d))
    k, v = fill_pools(kd, vd, BT)
    x = rng.integers(-3, 4, size=(B, H)).astype(np.float64)
    got = oracle.decode_layer(m, w, k, v, None, 2, [T] * B, x)
    wo = from_bits(w["w_o"])
    want = np.zeros((B, H))
    for b in range(B):
        o = np.concatenate([vd[b, 0].sum(axis=0) / T] * nq)      # every head sees the same kv head
        for r in range(H):
            want[b, r] = x[b, r] + sum(wo[r, c] * o[c] for c in range(nq * d))
    assert np.allclose(got, want, rtol=0, atol=1e-13)


# ----------------------------------------------------------------------------- paging, batching, state

def _random_case(seed, B=3, H=16, nq=4, nkv=2, d=4, F_=10, T=10, theta=10000.0):
    rng = np.random.default_rng(seed)
    m = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=theta)
    w = random_layer(rng, H, nq, nkv, d, F_, std=0.3)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    x = rng.normal(0, 1, (B, H))
    return rng, m, w, kd, vd, x


def test_identity_page_table_equals_contiguous_bitwise():
    rng, m, w, kd, vd, x = _random_case(14)
    B, T = x.shape[0], kd.shape[2]
    mb = (T + BT - 1) // BT
    k0, v0 = fill_pools(kd, vd, BT)
    a = oracle.decode_layer(m, w, k0, v0, None, mb, [T] * B, x)
    ident = np.arange(B * mb, dtype=np.int32).reshape(B, mb)
    k1, v1 = fill_pools(kd, vd, BT)
    b = oracle.decode_layer(m, w, k1, v1, ident, mb, [T] * B, x)
    assert np.array_equal(a, b) and np.array_equal(k0, k1) and np.array_equal(v0, v1)


def test_page_table_permutation_invariance_bitwise():
    rng, m, w, kd, vd, x = _random_case(15)
    B, T = x.shape[0], kd.shape[2]
    mb = (T + BT - 1) // BT
    k0, v0 = fill_pools(kd, vd, BT)
    a = oracle.decode_layer(m, w, k0, v0, None, mb, [T] * B, x)
    pool = B * mb + 5                                  # over-provisioned pool
    pt = rng.permutation(pool)[: B * mb].astype(np.int32).reshape(B, mb)
    k1, v1 = fill_pools(kd, vd, BT, page_table=pt, n_blocks=pool)
    b = oracle.decode_layer(m, w, k1, v1, pt, mb, [T] * B, x)
    assert np.array_equal(a, b)
    ka, va = dense_from_pools(k0, v0, B, T)
    kb, vb = dense_from_pools(k1, v1, B, T, page_table=pt)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)


def test_batch_rows_are_independent_bitwise():
    rng, m, w, kd, vd, x = _random_case(16)
    B, T = x.shape[0], kd.shape[2]
    mb = (T + BT - 1) // BT
    k, v = fill_pools(kd, vd, BT)
    full = oracle.decode_layer(m, w, k, v, None, mb, [T] * B, x)
    for b in range(B):
        k1, v1 = fill_pools(kd[b:b + 1], vd[b:b + 1], BT)
        one = oracle.decode_layer(m, w, k1, v1, None, mb, [T], x[b:b + 1])
        assert np.array_equal(one[0], full[b])


def test_mixed_sequence_lengths_match_single_runs():
    rng, m, w, kd, vd, x = _random_case(17, B=3, T=12)
    lens = [12, 5, 9]
    k, v = fill_pools(kd, vd, BT)
    full = oracle.decode_layer(m, w, k, v, None, 3, lens, x)
    for b, T in enumerate(lens):
        k1, v1 = fill_pools(kd[b:b + 1], vd[b:b + 1], BT)
        one = oracle.decode_layer(m, w, k1, v1, None, 3, [T], x[b:b + 1])
        assert np.array_equal(one[0], full[b])


def test_step_is_idempotent():
    rng, m, w, kd, vd, x = _random_case(18)
    B, T = x.shape[0], kd.shape[2]
    k, v = fill_pools(kd, vd, BT)
    a = oracle.decode_layer(m, w, k, v, None, 3, [T] * B, x)
    ka, va = k.copy(), v.copy()
    b = oracle.decode_layer(m, w, k, v, None, 3, [T] * B, x)
    assert np.array_equal(a, b) and np.array_equal(k, ka) and np.array_equal(v, va)


def test_decode_step_chains_layers_in_order():
    rng, m, w0, kd, vd, x = _random_case(19)
    w1 = random_layer(rng, 16, 4, 2, 4, 10, std=0.3)
    B, T = x.shape[0], kd.shape[2]
    pools = [fill_pools(kd, vd, BT), fill_pools(vd, kd, BT)]
    got = oracle.decode_step(m, [w0, w1], [p[0] for p in pools], [p[1] for p in pools], None, 3, [T] * B, x)
    pools2 = [fill_pools(kd, vd, BT), fill_pools(vd, kd, BT)]
    mid = oracle.decode_layer(m, w0, pools2[0][0], pools2[0][1], None, 3, [T] * B, x)
    want = oracle.decode_layer(m, w1, pools2[1][0], pools2[1][1], None, 3, [T] * B, mid)
    assert np.array_equal(got, want)
    pools3 = [fill_pools(kd, vd, BT), fill_pools(vd, kd, BT)]
    swapped = oracle.decode_step(m, [w1, w0], [p[0] for p in pools3], [p[1] for p in pools3], None, 3, [T] * B, x)
    assert not np.allclose(swapped, got)


def test_bad_arguments_are_rejected():
    rng, m, w, kd, vd, x = _random_case(20)
    k, v = fill_pools(kd, vd, BT)
    with pytest.raises(ValueError):
        oracle.decode_layer(m, w, k, v, None, 3, [0, 5, 5], x)        # empty span
    with pytest.raises(ValueError):
        oracle.decode_layer(m, w, k, v, None, 3, [13, 5, 5], x)       # beyond the page-table row


# ---- token-major cache layout: same logical cache, other addresses ------------------------------------------

@pytest.mark.parametrize("theta", [0.0, 10000.0])
@pytest.mark.parametrize("nq,nkv", [(4, 2), (6, 3), (4, 1)])
def test_token_major_layout_matches_torch_composition_and_head_major_bitwise(theta, nq, nkv):
    """Pools [block, token, kv head, channel] (the layout in which several local kv heads make one head's reads
    strided) against the torch composition and, bit for bit, against the head-major run of the same logical cache;
    the appended rows land at the token-major addresses (read back through the helper's own restatement of the
    layout) and nothing else moves."""
    rng = np.random.default_rng(40 + nq + nkv)
    B, H, d, F_, T = 3, 24, 8, 20, 21
    m_hm = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=theta)
    m_tm = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, rope_theta=theta, kv_token_major=True)
    w = random_layer(rng, H, nq, nkv, d, F_, std=0.3)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    mb = (T + BT - 1) // BT
    pool = B * mb + 3
    pt = rng.permutation(pool)[: B * mb].astype(np.int32).reshape(B, mb)
    x = rng.normal(0, 1, (B, H))
    k0, v0 = fill_pools(kd, vd, BT, page_table=pt, n_blocks=pool)
    k1, v1 = fill_pools(kd, vd, BT, page_table=pt, n_blocks=pool, token_major=True)
    assert k1.shape == (pool, BT, nkv, d) and not np.array_equal(v0.reshape(-1), v1.reshape(-1))
    assert np.array_equal(k0.reshape(-1), k1.reshape(-1)) == (nkv == 1)      # with one kv head the K pools coincide
    kq, vq = dense_from_pools(k1, v1, B, T, page_table=pt, token_major=True)
    a = oracle.decode_layer(m_hm, w, k0, v0, pt, mb, [T] * B, x)
    b = oracle.decode_layer(m_tm, w, k1, v1, pt, mb, [T] * B, x)
    assert np.array_equal(a, b)
    want, kn, vn = _torch_layer(m_tm, w, kq, vq, T, x)
    assert np.allclose(b, want, rtol=1e-11, atol=1e-12)
    ka, va = dense_from_pools(k0, v0, B, T, page_table=pt)
    kb, vb = dense_from_pools(k1, v1, B, T, page_table=pt, token_major=True)
    assert np.array_equal(ka, kb) and np.array_equal(va, vb)
    assert np.array_equal(kb[:, :, T - 1], kn) and np.array_equal(vb[:, :, T - 1], vn)
    assert np.array_equal(kb[:, :, : T - 1], kq[:, :, : T - 1]) and np.array_equal(vb[:, :, : T - 1], vq[:, :, : T - 1])
    # reading token-major pools as head-major must NOT give the same result (the switch does something)
    if nkv > 1:
        k2, v2 = fill_pools(kd, vd, BT, page_table=pt, n_blocks=pool, token_major=True)
        c = oracle.decode_layer(m_hm, w, k2.reshape(pool, nkv, BT, d), v2.reshape(pool, nkv, d, BT), pt, mb, [T] * B, x)
        assert not np.allclose(c, a)


def test_token_major_layout_with_int8_weights_and_refusal_for_int8_cache():
    rng = np.random.default_rng(47)
    B, H, nq, nkv, d, F_, T = 2, 16, 4, 2, 8, 12, 9
    m_hm = oracle.model(H, nq, nkv, d, F_, block_tokens=BT)
    m_tm = oracle.model(H, nq, nkv, d, F_, block_tokens=BT, kv_token_major=True)
    w = random_layer(rng, H, nq, nkv, d, F_, std=0.3)
    kd = rng.normal(0, 1, (B, nkv, T, d)); vd = rng.normal(0, 1, (B, nkv, T, d))
    mb = (T + BT - 1) // BT
    x = rng.normal(0, 1, (B, H))
    k0, v0 = fill_pools(kd, vd, BT)
    k1, v1 = fill_pools(kd, vd, BT, token_major=True)
    a = oracle.decode_layer_x(m_hm, w, k0, v0, None, mb, [T] * B, x)       # the general-format entry point, bf16 everywhere
    b = oracle.decode_layer_x(m_tm, w, k1, v1, None, mb, [T] * B, x)
    assert np.array_equal(a, b)
    assert np.array_equal(dense_from_pools(k0, v0, B, T)[0], dense_from_pools(k1, v1, B, T, token_major=True)[0])
    assert np.array_equal(dense_from_pools(k0, v0, B, T)[1], dense_from_pools(k1, v1, B, T, token_major=True)[1])
