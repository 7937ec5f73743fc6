"""ctypes binding of libpreserve_mi355x.so: the same entry points as include/preserve.h and include/preserve_aux.h.

Argument marshalling only -- every step of the decode path runs inside the library's HIP kernels.
There is no fallback: if the built library is missing, loading raises.  Device buffers are torch
tensors (or raw integer device addresses); streams are torch.cuda.Stream objects or raw handles.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpreserve_mi355x.so")

PSV_OK, PSV_ERR_INVALID_ARG, PSV_ERR_BAD_STATE, PSV_ERR_UNSUPPORTED, PSV_ERR_HIP, PSV_ERR_NOMEM = 0, -1, -2, -3, -4, -5
PSV_ERR_TIMEOUT = -6
PSV_TARGET_WEIGHTS, PSV_TARGET_KV = 1, 2
PSV_OP_QKV, PSV_OP_ATTN, PSV_OP_O, PSV_OP_GATE, PSV_OP_UP, PSV_OP_DOWN = range(6)
OP_NAMES = ["qkv", "attn", "o", "gate", "up", "down"]
PSV_FMT_BF16, PSV_FMT_INT8 = 0, 1
FORMATS = {"bf16": PSV_FMT_BF16, "int8": PSV_FMT_INT8}
PSV_KV_HEAD_MAJOR, PSV_KV_TOKEN_MAJOR = 0, 1
KV_LAYOUTS = {"head": PSV_KV_HEAD_MAJOR, "token": PSV_KV_TOKEN_MAJOR}
PSV_W_ROW_MAJOR, PSV_W_TILED = 0, 1
WEIGHT_LAYOUTS = {"row": PSV_W_ROW_MAJOR, "tiled": PSV_W_TILED}
PSV_KV_UNIT_BYTES_BF16, PSV_KV_UNIT_BYTES_INT8 = 4096, 2112
PSV_STATIC_SCRATCH_BYTES = 16 << 20
PSV_DBG_H1, PSV_DBG_QKV, PSV_DBG_ATTN, PSV_DBG_Y, PSV_DBG_H2, PSV_DBG_M = range(6)

EXPORTS = [
    "psv_strerror", "psv_validate_desc", "psv_workspace_bytes", "psv_plan_chain", "psv_create", "psv_destroy",
    "psv_set_layer_weights", "psv_set_kv", "psv_set_comm_windows", "psv_set_policy", "psv_plan",
    "psv_set_graph_mode", "psv_decode_step", "psv_sync", "psv_get_stats", "psv_tune_attention", "psv_check_overlap",
    "psv_set_profile_op",
    "psv_get_profile", "psv_prefetch_region", "psv_spin", "psv_copy_bytes", "psv_debug_read",
    "psv_debug_force_wait_timeout", "psv_decode_step_static", "psv_set_fused_kernels", "psv_debug_last_step_path", "psv_debug_last_step_prelaunches", "psv_tile_weights",
]


class psv_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("hidden", C.c_uint32), ("n_q_heads", C.c_uint32),
                ("n_kv_heads", C.c_uint32), ("head_dim", C.c_uint32), ("ffn", C.c_uint32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("max_batch", C.c_uint32),
                ("max_seq", C.c_uint32), ("weight_format", C.c_uint32), ("kv_format", C.c_uint32),
                ("kv_layout", C.c_uint32), ("weight_layout", C.c_uint32)]


class psv_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_o", "w_gate", "w_up", "w_down", "g_attn", "g_mlp",
                                          "s_qkv", "s_o", "s_gate", "s_up", "s_down")]


class psv_kv_desc(C.Structure):
    _fields_ = [("k_pools", C.POINTER(C.c_void_p)), ("v_pools", C.POINTER(C.c_void_p)),
                ("page_table", C.c_void_p), ("max_blocks", C.c_uint32), ("num_pool_blocks", C.c_uint32),
                ("seq_lens", C.c_void_p)]


class psv_prefetch_policy(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("targets", C.c_uint32), ("budget_bytes", C.c_uint64),
                ("chunk_bytes", C.c_uint64), ("cu_budget", C.c_uint32), ("partial", C.c_uint32),
                ("join", C.c_uint32), ("prelaunch", C.c_uint32)]


class psv_plan_entry(C.Structure):
    _fields_ = [("layer", C.c_uint32), ("window", C.c_uint32), ("target_layer", C.c_uint32),
                ("target_op", C.c_uint32), ("mem_size", C.c_uint64), ("bytes", C.c_uint64)]


class psv_stats(C.Structure):
    _fields_ = [("weight_bytes_per_layer", C.c_uint64), ("kv_bytes_per_layer", C.c_uint64),
                ("planned_prefetch_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64),
                ("kernels_per_layer", C.c_uint32), ("prefetch_launches", C.c_uint32),
                ("steps", C.c_uint32), ("reserved", C.c_uint32)]


class PsvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


_lib = None


def lib():
    """Loads the built library; raises if it has not been built (there is no other code path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libpreserve_mi355x.so is not built: run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` or `python paper_2501_08192_amd/build.py`")
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t
        sig = {
            "psv_strerror": (C.c_char_p, [C.c_int32]),
            "psv_validate_desc": (C.c_int32, [C.POINTER(psv_model_desc)]),
            "psv_workspace_bytes": (sz, [C.POINTER(psv_model_desc)]),
            "psv_plan_chain": (C.c_int32, [C.POINTER(psv_model_desc), u32, u32, C.POINTER(psv_prefetch_policy),
                                           C.POINTER(psv_plan_entry), sz, C.POINTER(sz)]),
            "psv_create": (C.c_int32, [C.POINTER(psv_model_desc), vp, vp, C.POINTER(vp)]),
            "psv_destroy": (C.c_int32, [vp]),
            "psv_set_layer_weights": (C.c_int32, [vp, u32, C.POINTER(psv_layer_weights)]),
            "psv_set_kv": (C.c_int32, [vp, C.POINTER(psv_kv_desc)]),
            "psv_set_comm_windows": (C.c_int32, [vp, C.c_float, C.c_float]),
            "psv_set_policy": (C.c_int32, [vp, C.POINTER(psv_prefetch_policy), u32, u32]),
            "psv_plan": (C.c_int32, [vp, C.POINTER(psv_plan_entry), sz, C.POINTER(sz)]),
            "psv_set_graph_mode": (C.c_int32, [vp, u32]),
            "psv_decode_step": (C.c_int32, [vp, vp, vp, u32, u32, u32]),
            "psv_sync": (C.c_int32, [vp]),
            "psv_get_stats": (C.c_int32, [vp, C.POINTER(psv_stats)]),
            "psv_tune_attention": (C.c_int32, [vp, vp, vp, u32, C.POINTER(u32)]),
            "psv_check_overlap": (C.c_int32, [vp, C.POINTER(C.c_int32)]),
            "psv_set_profile_op": (C.c_int32, [vp, C.c_int32]),
            "psv_get_profile": (C.c_int32, [vp, C.POINTER(C.c_double), C.POINTER(u64)]),
            "psv_prefetch_region": (C.c_int32, [vp, u64, u32, vp]),
            "psv_spin": (C.c_int32, [C.c_float, vp]),
            "psv_copy_bytes": (C.c_int32, [vp, vp, u64, vp]),
            "psv_debug_read": (C.c_int32, [vp, u32, vp, sz]),
            "psv_debug_force_wait_timeout": (C.c_int32, [vp, u32]),
            "psv_debug_last_step_path": (C.c_int32, [vp, C.POINTER(u32)]),
            "psv_debug_last_step_prelaunches": (C.c_int32, [vp, C.POINTER(u32)]),
            "psv_tile_weights": (C.c_int32, [vp, vp, u32, u32, u32, vp]),
            "psv_set_fused_kernels": (C.c_int32, [vp, u32]),
            "psv_decode_step_static": (C.c_int32, [C.POINTER(psv_model_desc), C.POINTER(psv_layer_weights),
                                                   C.POINTER(psv_kv_desc), vp, vp, u32, u32, u32, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(status, where):
    if status != PSV_OK:
        raise PsvError(status, where)


def _dev_ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s):
    if s is None or isinstance(s, int):
        return s
    return s.cuda_stream


def strerror(status):
    return lib().psv_strerror(int(status)).decode()


def model_desc(n_layers, hidden, n_q_heads, n_kv_heads, ffn, max_batch, max_seq, head_dim=128, rms_eps=1e-5,
               rope_theta=500000.0, weight_format="bf16", kv_format="bf16", kv_layout="head", weight_layout="row"):
    return psv_model_desc(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, rms_eps, rope_theta, max_batch,
                          max_seq, FORMATS[weight_format], FORMATS[kv_format], KV_LAYOUTS[kv_layout], WEIGHT_LAYOUTS[weight_layout])


def prefetch_policy(mode=0, targets=PSV_TARGET_WEIGHTS | PSV_TARGET_KV, budget_bytes=0, chunk_bytes=0, cu_budget=0,
                    partial=0, join=0, prelaunch=0):
    return psv_prefetch_policy(mode, targets, budget_bytes, chunk_bytes, cu_budget, partial, join, prelaunch)


def psv_validate_desc(desc):
    return int(lib().psv_validate_desc(C.byref(desc)))


def psv_workspace_bytes(desc):
    return int(lib().psv_workspace_bytes(C.byref(desc)))


def _entries(arr, n):
    return [dict(layer=e.layer, window=e.window, target_layer=e.target_layer, target_op=e.target_op,
                 mem_size=e.mem_size, bytes=e.bytes) for e in arr[:n]]


def psv_plan_chain(desc, batch, context, policy):
    n = C.c_size_t(0)
    _check(lib().psv_plan_chain(C.byref(desc), batch, context, C.byref(policy), None, 0, C.byref(n)), "psv_plan_chain")
    arr = (psv_plan_entry * max(1, n.value))()
    _check(lib().psv_plan_chain(C.byref(desc), batch, context, C.byref(policy), arr, n.value, C.byref(n)), "psv_plan_chain")
    return _entries(arr, n.value)


def psv_create(desc, stream_main, stream_side):
    out = C.c_void_p()
    _check(lib().psv_create(C.byref(desc), _stream(stream_main), _stream(stream_side), C.byref(out)), "psv_create")
    return out


def psv_destroy(ctx):
    _check(lib().psv_destroy(ctx), "psv_destroy")


def psv_set_layer_weights(ctx, layer, weights):
    """weights: dict name -> device tensor: w_qkv, w_o, w_gate, w_up, w_down (bf16, or int8 codes), g_attn, g_mlp
    (bf16) and, for int8 weights, the fp32 per-row scales s_qkv, s_o, s_gate, s_up, s_down."""
    w = psv_layer_weights(*[_dev_ptr(weights.get(n)) for n, _ in psv_layer_weights._fields_])
    _check(lib().psv_set_layer_weights(ctx, layer, C.byref(w)), "psv_set_layer_weights")


def psv_set_kv(ctx, k_pools, v_pools, page_table, max_blocks, num_pool_blocks, seq_lens):
    n = len(k_pools)
    ka = (C.c_void_p * n)(*[_dev_ptr(t) for t in k_pools])
    va = (C.c_void_p * n)(*[_dev_ptr(t) for t in v_pools])
    kv = psv_kv_desc(ka, va, _dev_ptr(page_table), max_blocks, num_pool_blocks, _dev_ptr(seq_lens))
    _check(lib().psv_set_kv(ctx, C.byref(kv)), "psv_set_kv")


def psv_set_comm_windows(ctx, us_after_attn, us_after_mlp):
    _check(lib().psv_set_comm_windows(ctx, us_after_attn, us_after_mlp), "psv_set_comm_windows")


def psv_set_policy(ctx, policy, batch, context):
    _check(lib().psv_set_policy(ctx, C.byref(policy), batch, context), "psv_set_policy")


def psv_plan(ctx):
    n = C.c_size_t(0)
    _check(lib().psv_plan(ctx, None, 0, C.byref(n)), "psv_plan")
    arr = (psv_plan_entry * max(1, n.value))()
    _check(lib().psv_plan(ctx, arr, n.value, C.byref(n)), "psv_plan")
    return _entries(arr, n.value)


def psv_set_graph_mode(ctx, use_graph):
    _check(lib().psv_set_graph_mode(ctx, 1 if use_graph else 0), "psv_set_graph_mode")


def psv_decode_step(ctx, x_in, x_out, batch, layer_begin, layer_end):
    _check(lib().psv_decode_step(ctx, _dev_ptr(x_in), _dev_ptr(x_out), batch, layer_begin, layer_end), "psv_decode_step")


def psv_decode_step_static(desc, layers, k_pools, v_pools, page_table, max_blocks, num_pool_blocks, seq_lens, x_in, x_out,
                           batch, layer_begin, layer_end, stream):
    """layers: list (one entry per layer of desc; None where a layer is outside the range) of weight dicts as for
    psv_set_layer_weights; k_pools / v_pools: lists of device tensors, one per layer."""
    n = len(layers)
    arr = (psv_layer_weights * n)()
    for i, w in enumerate(layers):
        if w is not None:
            arr[i] = psv_layer_weights(*[_dev_ptr(w.get(f)) for f, _ in psv_layer_weights._fields_])
    ka = (C.c_void_p * n)(*[_dev_ptr(t) for t in k_pools])
    va = (C.c_void_p * n)(*[_dev_ptr(t) for t in v_pools])
    kv = psv_kv_desc(ka, va, _dev_ptr(page_table), max_blocks, num_pool_blocks, _dev_ptr(seq_lens))
    _check(lib().psv_decode_step_static(C.byref(desc), arr, C.byref(kv), _dev_ptr(x_in), _dev_ptr(x_out), batch,
                                        layer_begin, layer_end, _stream(stream)), "psv_decode_step_static")


def psv_sync(ctx):
    _check(lib().psv_sync(ctx), "psv_sync")


def psv_get_stats(ctx):
    s = psv_stats()
    _check(lib().psv_get_stats(ctx, C.byref(s)), "psv_get_stats")
    return {n: getattr(s, n) for n, _ in psv_stats._fields_ if n != "reserved"}


def psv_tune_attention(ctx, x_in, x_out, batch):
    out = C.c_uint32(0)
    _check(lib().psv_tune_attention(ctx, _dev_ptr(x_in), _dev_ptr(x_out), batch, C.byref(out)), "psv_tune_attention")
    return int(out.value)


def psv_check_overlap(ctx):
    out = C.c_int32(0)
    _check(lib().psv_check_overlap(ctx, C.byref(out)), "psv_check_overlap")
    return bool(out.value)


def psv_set_profile_op(ctx, op):
    _check(lib().psv_set_profile_op(ctx, op), "psv_set_profile_op")


def psv_get_profile(ctx):
    ms, n = C.c_double(0), C.c_uint64(0)
    _check(lib().psv_get_profile(ctx, C.byref(ms), C.byref(n)), "psv_get_profile")
    return ms.value, n.value


def psv_prefetch_region(ptr, nbytes, workgroups, stream):
    _check(lib().psv_prefetch_region(_dev_ptr(ptr), nbytes, workgroups, _stream(stream)), "psv_prefetch_region")


def psv_spin(us, stream):
    _check(lib().psv_spin(us, _stream(stream)), "psv_spin")


def psv_copy_bytes(dst, src, nbytes, stream):
    _check(lib().psv_copy_bytes(_dev_ptr(dst), _dev_ptr(src), nbytes, _stream(stream)), "psv_copy_bytes")


def psv_debug_read(ctx, which, host_array):
    """host_array: a contiguous numpy array that receives the buffer."""
    _check(lib().psv_debug_read(ctx, which, host_array.ctypes.data_as(C.c_void_p), host_array.nbytes), "psv_debug_read")
    return host_array


def psv_set_fused_kernels(ctx, on):
    """on: 0 / False = one kernel per operator, 1 / True = one per block, 2 = the whole step as one kernel."""
    _check(lib().psv_set_fused_kernels(ctx, int(on)), "psv_set_fused_kernels")


def psv_tile_weights(dst, src, rows, cols, weight_format, stream):
    """dst, src: device tensors of rows * cols elements; weight_format "bf16" or "int8"."""
    _check(lib().psv_tile_weights(_dev_ptr(dst), _dev_ptr(src), int(rows), int(cols), FORMATS[weight_format], _stream(stream)),
           "psv_tile_weights")


def psv_debug_last_step_path(ctx):
    out = C.c_uint32(0)
    _check(lib().psv_debug_last_step_path(ctx, C.byref(out)), "psv_debug_last_step_path")
    return int(out.value)


def psv_debug_last_step_prelaunches(ctx):
    out = C.c_uint32(0)
    _check(lib().psv_debug_last_step_prelaunches(ctx, C.byref(out)), "psv_debug_last_step_prelaunches")
    return int(out.value)


def psv_debug_force_wait_timeout(ctx, on):
    _check(lib().psv_debug_force_wait_timeout(ctx, 1 if on else 0), "psv_debug_force_wait_timeout")
