"""ctypes front-end of the C oracle (oracle/preserve_oracle.c, oracle/preserve_oracle_q8.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline leg of
bench.py; never by the GPU package.  bf16 tensors are numpy uint16 arrays holding the raw bits;
everything else is float64 / int32 / uint64 numpy.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

NODE_OTHER, NODE_COMM, NODE_MATMUL, NODE_SELFATTN = 0, 1, 2, 3

_lib = None


class _Model(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("block_tokens", C.c_int32),
                ("rms_eps", C.c_double), ("rope_theta", C.c_double), ("kv_token_major", C.c_int32)]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")]


class _KV(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("page_table", C.c_void_p),
                ("max_blocks", C.c_int32), ("seq_lens", C.c_void_p)]


class _LayerWeightsX(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "s_qkv", "s_o", "s_gate", "s_up", "s_down",
                 "g_attn", "g_mlp")]


class _KVX(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("kv_int8", C.c_int32),
                ("page_table", C.c_void_p), ("max_blocks", C.c_int32), ("seq_lens", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        L.orc_bf16_to_f64.restype = C.c_double
        L.orc_bf16_to_f64.argtypes = [C.c_uint16]
        L.orc_f64_to_bf16.restype = C.c_uint16
        L.orc_f64_to_bf16.argtypes = [C.c_double]
        L.orc_silu.restype = C.c_double
        L.orc_silu.argtypes = [C.c_double]
        L.orc_rmsnorm.restype = None
        L.orc_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_void_p]
        L.orc_linear.restype = None
        L.orc_linear.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_rope.restype = None
        L.orc_rope.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_double]
        L.orc_softmax.restype = None
        L.orc_softmax.argtypes = [C.c_void_p, C.c_int]
        L.orc_attention_head.restype = None
        L.orc_attention_head.argtypes = [C.POINTER(_Model), C.POINTER(_KV), C.c_int, C.c_int,
                                         C.c_void_p, C.c_void_p]
        L.orc_decode_layer.restype = C.c_int
        L.orc_decode_layer.argtypes = [C.POINTER(_Model), C.POINTER(_LayerWeights), C.POINTER(_KV),
                                       C.c_int, C.c_void_p]
        L.orc_linear_q8.restype = None
        L.orc_linear_q8.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_quantize_row.restype = None
        L.orc_quantize_row.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_attention_head_q8.restype = None
        L.orc_attention_head_q8.argtypes = [C.POINTER(_Model), C.POINTER(_KVX), C.c_int, C.c_int,
                                            C.c_void_p, C.c_void_p]
        L.orc_decode_layer_x.restype = C.c_int
        L.orc_decode_layer_x.argtypes = [C.POINTER(_Model), C.POINTER(_LayerWeightsX), C.POINTER(_KVX),
                                         C.c_int, C.c_void_p]
        L.orc_plan.restype = C.c_int64
        L.orc_plan.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                               C.c_void_p, C.c_void_p, C.c_int64]
        L.orc_num_threads.restype = C.c_int
        L.orc_num_threads.argtypes = []
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns, got %s" % a.dtype)
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def model(hidden, n_q_heads, n_kv_heads, head_dim, ffn, block_tokens=16, rms_eps=1e-5,
          rope_theta=500000.0, kv_token_major=False):
    return _Model(int(hidden), int(n_q_heads), int(n_kv_heads), int(head_dim), int(ffn),
                  int(block_tokens), float(rms_eps), float(rope_theta), 1 if kv_token_major else 0)


# ---- elementary pieces -------------------------------------------------------------------

def bf16_to_f64(bits) -> float:
    return float(lib().orc_bf16_to_f64(int(bits)))


def f64_to_bf16(v) -> int:
    return int(lib().orc_f64_to_bf16(float(v)))


def silu(z) -> float:
    return float(lib().orc_silu(float(z)))


def rmsnorm(x, gain_bf16, eps):
    x = _f64(x)
    g = _u16(gain_bf16)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_ptr(x), _ptr(g), x.size, float(eps), _ptr(out))
    return out


def linear(w_bf16, vec):
    w = _u16(w_bf16)
    v = _f64(vec)
    rows, cols = w.shape
    assert v.shape == (cols,)
    out = np.empty(rows, dtype=np.float64)
    lib().orc_linear(_ptr(w), _ptr(v), rows, cols, _ptr(out))
    return out


def rope(vec, pos, theta):
    v = _f64(vec).copy()
    lib().orc_rope(_ptr(v), v.size, int(pos), float(theta))
    return v


def softmax(scores):
    s = _f64(scores).copy()
    lib().orc_softmax(_ptr(s), s.size)
    return s


def _kv_struct(k_pool, v_pool, page_table, max_blocks, seq_lens):
    keep = [_u16(k_pool), _u16(v_pool), np.ascontiguousarray(seq_lens, dtype=np.int32)]
    if not (keep[0] is k_pool or np.shares_memory(keep[0], k_pool)):
        raise ValueError("k_pool must be a contiguous uint16 array (it is written in place)")
    if not (keep[1] is v_pool or np.shares_memory(keep[1], v_pool)):
        raise ValueError("v_pool must be a contiguous uint16 array (it is written in place)")
    pt = None
    if page_table is not None:
        pt = np.ascontiguousarray(page_table, dtype=np.int32)
        keep.append(pt)
    kv = _KV(_ptr(keep[0]), _ptr(keep[1]), _ptr(pt) if pt is not None else None,
             int(max_blocks), _ptr(keep[2]))
    return kv, keep


def attention_head(m, k_pool, v_pool, page_table, max_blocks, seq_lens, b, q_head, q):
    kv, keep = _kv_struct(k_pool, v_pool, page_table, max_blocks, seq_lens)
    qv = _f64(q)
    out = np.empty(m.head_dim, dtype=np.float64)
    lib().orc_attention_head(C.byref(m), C.byref(kv), int(b), int(q_head), _ptr(qv), _ptr(out))
    del keep
    return out


_WEIGHT_NAMES = ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "g_attn", "g_mlp")


def decode_layer(m, weights, k_pool, v_pool, page_table, max_blocks, seq_lens, x):
    """One decoder layer.  `weights`: dict of uint16 arrays.  k_pool / v_pool are updated in
    place (one slot per sequence).  Returns the new residual stream, float64 [batch, hidden]."""
    arrs = {n: _u16(weights[n]) for n in _WEIGHT_NAMES}
    qkv_rows = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
    assert arrs["w_qkv"].shape == (qkv_rows, m.hidden)
    assert arrs["w_o"].shape == (m.hidden, m.n_q_heads * m.head_dim)
    assert arrs["w_gate"].shape == (m.ffn, m.hidden) and arrs["w_up"].shape == (m.ffn, m.hidden)
    assert arrs["w_down"].shape == (m.hidden, m.ffn)
    assert arrs["g_attn"].shape == (m.hidden,) and arrs["g_mlp"].shape == (m.hidden,)
    lw = _LayerWeights(*[_ptr(arrs[n]) for n in _WEIGHT_NAMES])
    kv, keep = _kv_struct(k_pool, v_pool, page_table, max_blocks, seq_lens)
    xx = _f64(x).copy()
    batch = xx.shape[0]
    assert xx.shape == (batch, m.hidden)
    rc = lib().orc_decode_layer(C.byref(m), C.byref(lw), C.byref(kv), batch, _ptr(xx))
    del keep
    if rc != 0:
        raise ValueError("orc_decode_layer rejected its arguments (rc=%d)" % rc)
    return xx


def decode_step(m, layers, k_pools, v_pools, page_table, max_blocks, seq_lens, x):
    """All layers in order; `layers`, `k_pools`, `v_pools` are per-layer lists."""
    xx = _f64(x).copy()
    for lw, kp, vp in zip(layers, k_pools, v_pools):
        xx = decode_layer(m, lw, kp, vp, page_table, max_blocks, seq_lens, xx)
    return xx


# ---- int8 variant ------------------------------------------------------------------------

def kv_unit_bytes(m) -> int:
    """Bytes of one (block, kv head) unit of an int8 pool: codes, then one fp32 scale per token."""
    return m.block_tokens * m.head_dim + 4 * m.block_tokens


def linear_q8(codes, scale, vec):
    w = np.ascontiguousarray(codes)
    if w.dtype != np.int8:
        raise TypeError("int8 weights expected, got %s" % w.dtype)
    sc = np.ascontiguousarray(scale, dtype=np.float32)
    v = _f64(vec)
    rows, cols = w.shape
    assert v.shape == (cols,) and sc.shape == (rows,)
    out = np.empty(rows, dtype=np.float64)
    lib().orc_linear_q8(_ptr(w), _ptr(sc), _ptr(v), rows, cols, _ptr(out))
    return out


def quantize_row(vec):
    """Returns (int8 codes, fp32 scale) of the append rule."""
    v = _f64(vec)
    codes = np.zeros(v.size, dtype=np.int8)
    scale = np.zeros(1, dtype=np.float32)
    lib().orc_quantize_row(_ptr(v), v.size, 1, _ptr(codes), _ptr(scale))
    return codes, np.float32(scale[0])


def _pool_bytes(a, what):
    if a.dtype == np.uint16 or a.dtype == np.uint8:
        if not a.flags["C_CONTIGUOUS"]:
            raise ValueError("%s must be contiguous (it is written in place)" % what)
        return a
    raise TypeError("%s: uint16 (bf16 bits) or uint8 (int8 layout) expected, got %s" % (what, a.dtype))


def _kvx_struct(k_pool, v_pool, page_table, max_blocks, seq_lens):
    kp, vp = _pool_bytes(k_pool, "k_pool"), _pool_bytes(v_pool, "v_pool")
    if kp.dtype != vp.dtype:
        raise TypeError("k_pool and v_pool must have the same format")
    keep = [kp, vp, np.ascontiguousarray(seq_lens, dtype=np.int32)]
    pt = None
    if page_table is not None:
        pt = np.ascontiguousarray(page_table, dtype=np.int32)
        keep.append(pt)
    kv = _KVX(_ptr(kp), _ptr(vp), 1 if kp.dtype == np.uint8 else 0, _ptr(pt) if pt is not None else None,
              int(max_blocks), _ptr(keep[2]))
    return kv, keep


def attention_head_q8(m, k_pool, v_pool, page_table, max_blocks, seq_lens, b, q_head, q):
    if k_pool.dtype != np.uint8:
        raise TypeError("int8 pools are passed as uint8 byte arrays")
    kv, keep = _kvx_struct(k_pool, v_pool, page_table, max_blocks, seq_lens)
    qv = _f64(q)
    out = np.empty(m.head_dim, dtype=np.float64)
    lib().orc_attention_head_q8(C.byref(m), C.byref(kv), int(b), int(q_head), _ptr(qv), _ptr(out))
    del keep
    return out


_SCALE_OF = {"w_qkv": "s_qkv", "w_o": "s_o", "w_gate": "s_gate", "w_up": "s_up", "w_down": "s_down"}


def decode_layer_x(m, weights, k_pool, v_pool, page_table, max_blocks, seq_lens, x):
    """One decoder layer with bf16 weights (uint16 arrays) or int8 weights (int8 arrays plus fp32 per-row
    scales under s_qkv, s_o, s_gate, s_up, s_down), over a bf16 cache (uint16 pools) or an int8 cache (uint8
    pools with embedded scales).  Pools are updated in place."""
    int8_w = weights["w_qkv"].dtype == np.int8
    keep = []
    ptrs = {}
    for n in ("w_qkv", "w_o", "w_gate", "w_up", "w_down"):
        a = np.ascontiguousarray(weights[n])
        if a.dtype != (np.int8 if int8_w else np.uint16):
            raise TypeError("%s: mixed weight formats" % n)
        keep.append(a)
        ptrs[n] = _ptr(a)
        if int8_w:
            sc = np.ascontiguousarray(weights[_SCALE_OF[n]], dtype=np.float32)
            assert sc.shape == (a.shape[0],)
            keep.append(sc)
            ptrs[_SCALE_OF[n]] = _ptr(sc)
        else:
            ptrs[_SCALE_OF[n]] = None
    for n in ("g_attn", "g_mlp"):
        a = _u16(weights[n])
        keep.append(a)
        ptrs[n] = _ptr(a)
    qkv_rows = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
    assert weights["w_qkv"].shape == (qkv_rows, m.hidden)
    assert weights["w_o"].shape == (m.hidden, m.n_q_heads * m.head_dim)
    assert weights["w_gate"].shape == (m.ffn, m.hidden) and weights["w_up"].shape == (m.ffn, m.hidden)
    assert weights["w_down"].shape == (m.hidden, m.ffn)
    lw = _LayerWeightsX(*[ptrs[n] for n, _ in _LayerWeightsX._fields_])
    kv, keep2 = _kvx_struct(k_pool, v_pool, page_table, max_blocks, seq_lens)
    xx = _f64(x).copy()
    batch = xx.shape[0]
    assert xx.shape == (batch, m.hidden)
    rc = lib().orc_decode_layer_x(C.byref(m), C.byref(lw), C.byref(kv), batch, _ptr(xx))
    del keep, keep2
    if rc != 0:
        raise ValueError("orc_decode_layer_x rejected its arguments (rc=%d)" % rc)
    return xx


def decode_step_x(m, layers, k_pools, v_pools, page_table, max_blocks, seq_lens, x):
    xx = _f64(x).copy()
    for lw, kp, vp in zip(layers, k_pools, v_pools):
        xx = decode_layer_x(m, lw, kp, vp, page_table, max_blocks, seq_lens, xx)
    return xx


# ---- Algorithm 1 -------------------------------------------------------------------------

def plan(node_type, mem_size, children, capacity):
    """Prefetch insertion on a general graph.  `children[i]` lists the child node ids of node i.
    Returns [(comm node, target node), ...] in insertion order."""
    n = len(node_type)
    types = np.ascontiguousarray(node_type, dtype=np.int32)
    mem = np.ascontiguousarray(mem_size, dtype=np.uint64)
    off = np.zeros(n + 1, dtype=np.int32)
    for i, ch in enumerate(children):
        off[i + 1] = off[i] + len(ch)
    idx = np.ascontiguousarray([c for ch in children for c in ch], dtype=np.int32)
    if idx.size == 0:
        idx = np.zeros(1, dtype=np.int32)
    cap = max(1, n * n)
    oc = np.zeros(cap, dtype=np.int32)
    ot = np.zeros(cap, dtype=np.int32)
    found = lib().orc_plan(n, _ptr(types), _ptr(mem), _ptr(off), _ptr(idx), int(capacity),
                           _ptr(oc), _ptr(ot), cap)
    if found < 0 or found > cap:
        raise ValueError("orc_plan failed (%d)" % found)
    return [(int(oc[i]), int(ot[i])) for i in range(found)]
