"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module only draws random numbers and lays them out; it holds none of the decode step's
arithmetic.  Both the GPU tests/benchmark and the CPU oracle are fed from here.

The paper measures trained Llama3 / Qwen2 / Phi3 checkpoints (Section 4, "Experimental setup").
Timing depends only on shapes, so each workload below takes the shape of one tensor-parallel
shard of such a model and fills it with seeded Gaussians.

KV-cache layout (bt = 16 tokens per block):
    K pool [n_blocks, n_kv_heads, bt, head_dim]   (token-major inside a block)
    V pool [n_blocks, n_kv_heads, head_dim, bt]   (channel-major inside a block)
A "contiguous" cache is the same pool with the implicit page table block(b, j) = b*max_blocks + j.

int8 formats (the precision of the paper's measurements): weights are int8 codes plus one fp32 scale per
output row; a KV pool is a byte tensor [n_blocks, n_kv_heads, 2112]: 2048 codes (K token-major, V
channel-major) followed by the 16 fp32 scales of the block's tokens.
"""
from dataclasses import dataclass, replace

import torch

BLOCK_TOKENS = 16


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    batch: int
    context: int            # attention span T, including the token decoded by the step
    paged: bool
    window_us: tuple        # (after attention block, after MLP block)
    rms_eps: float = 1e-5
    rope_theta: float = 500000.0
    weight_format: str = "bf16"   # or "int8"
    kv_format: str = "bf16"       # or "int8"
    kv_layout: str = "head"       # "head": K [block, kv head, token, channel], V [block, kv head, channel, token];
                                  # "token" (bf16 only): both [block, token, kv head, channel]
    weight_layout: str = "row"    # "row": projection matrices row-major [out, in]; "tiled": the order the matrix-core
                                  # projections read them in (the harness converts; the oracle always reads row-major)

    @property
    def qkv_rows(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def blocks_per_seq(self):
        return (self.context + BLOCK_TOKENS - 1) // BLOCK_TOKENS

    @property
    def pool_blocks(self):
        return self.batch * self.blocks_per_seq

    @property
    def weight_bytes_per_layer(self):
        h, f = self.hidden, self.ffn
        per = 1 if self.weight_format == "int8" else 2
        return per * (self.qkv_rows * h + h * self.n_q_heads * self.head_dim + 3 * f * h)

    @property
    def kv_bytes_per_layer(self):
        per_token = 2 * (self.head_dim + 4) if self.kv_format == "int8" else 2 * 2 * self.head_dim   # K and V
        return per_token * self.batch * self.context * self.n_kv_heads

    @property
    def layer_bytes(self):
        return self.weight_bytes_per_layer + self.kv_bytes_per_layer

    def scaled(self, **kw):
        return replace(self, **kw)


# The five workloads of the benchmark definition.  c1 is the small case; c2 (one TP=8 shard of
# a Llama-3-8B-shaped model) is the one the headline metric is quoted on.  The batched workloads, whose projections run on
# the matrix cores, keep their weights in the tiled order those kernels read them in (scaled(weight_layout="row") for
# row-major).
WORKLOADS = {
    "c1": Workload("c1", 2, 1024, 8, 8, 128, 2816, 1, 256, False, (10.0, 10.0)),
    "c2": Workload("c2", 32, 4096, 4, 1, 128, 1792, 1, 2048, False, (15.0, 15.0)),
    "c3": Workload("c3", 80, 8192, 8, 1, 128, 3584, 8, 4096, False, (20.0, 20.0), weight_layout="tiled"),
    "c4": Workload("c4", 32, 4096, 4, 1, 128, 1792, 64, 8192, True, (25.0, 25.0), weight_layout="tiled"),
    "c5": Workload("c5", 80, 8192, 8, 1, 128, 3584, 32, 32768, True, (20.0, 20.0), weight_layout="tiled"),
}

_TENSOR_IDS = {"w_qkv": 1, "w_o": 2, "w_gate": 3, "w_up": 4, "w_down": 5, "g_attn": 6, "g_mlp": 7,
               "k_pool": 8, "v_pool": 9, "x": 10, "page_table": 11}


def _gen(seed, name, layer, device):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + _TENSOR_IDS[name] * 10007 + int(layer)) & 0x7FFFFFFFFFFFFFFF)
    return g


def _normal(shape, std, mean, seed, name, layer, device):
    g = _gen(seed, name, layer, device)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(torch.bfloat16)


CODE_STD = 42.0   # int8 codes are drawn as round(N(0, 42^2)) clamped to +-127 (3 sigma)
KV_UNIT_INT8 = BLOCK_TOKENS * 128 + 4 * BLOCK_TOKENS

_SCALE_IDS = {"w_qkv": 21, "w_o": 22, "w_gate": 23, "w_up": 24, "w_down": 25, "k_pool": 28, "v_pool": 29}


def _codes(shape, seed, name, layer, device):
    g = _gen(seed, name, layer, device)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return t.mul_(CODE_STD).round_().clamp_(-127, 127).to(torch.int8)


def _scales(shape, typical, seed, name, layer, device):
    """fp32 scales spread +-25 % around typical / CODE_STD, so that code * scale ~ N(0, typical^2)."""
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + _SCALE_IDS[name] * 10007 + int(layer)) & 0x7FFFFFFFFFFFFFFF)
    u = torch.rand(shape, generator=g, device=device, dtype=torch.float32)
    return u.mul_(0.5).add_(0.75).mul_(typical / CODE_STD)


def layer_weights(w: Workload, layer: int, seed: int = 2501, device="cpu"):
    """Weights of one layer: projections N(0, 0.02^2) (bf16, or int8 codes with fp32 row scales under s_*),
    norm gains 1 + N(0, 0.02^2) in bf16."""
    h, f, nqd = w.hidden, w.ffn, w.n_q_heads * w.head_dim
    if w.weight_format == "int8":
        shapes = {"w_qkv": (w.qkv_rows, h), "w_o": (h, nqd), "w_gate": (f, h), "w_up": (f, h), "w_down": (h, f)}
        out = {}
        for n, shp in shapes.items():
            out[n] = _codes(shp, seed, n, layer, device)
            out["s_" + n[2:]] = _scales((shp[0],), 0.02, seed, n, layer, device)
        out["g_attn"] = _normal((h,), 0.02, 1.0, seed, "g_attn", layer, device)
        out["g_mlp"] = _normal((h,), 0.02, 1.0, seed, "g_mlp", layer, device)
        return out
    return {
        "w_qkv": _normal((w.qkv_rows, h), 0.02, 0.0, seed, "w_qkv", layer, device),
        "w_o": _normal((h, nqd), 0.02, 0.0, seed, "w_o", layer, device),
        "w_gate": _normal((f, h), 0.02, 0.0, seed, "w_gate", layer, device),
        "w_up": _normal((f, h), 0.02, 0.0, seed, "w_up", layer, device),
        "w_down": _normal((h, f), 0.02, 0.0, seed, "w_down", layer, device),
        "g_attn": _normal((h,), 0.02, 1.0, seed, "g_attn", layer, device),
        "g_mlp": _normal((h,), 0.02, 1.0, seed, "g_mlp", layer, device),
    }


def kv_pools(w: Workload, layer: int, seed: int = 2501, device="cpu", n_blocks=None):
    """K and V pools of one layer, every slot ~ N(0,1): bf16, or the int8 byte layout."""
    nb = w.pool_blocks if n_blocks is None else int(n_blocks)
    if w.kv_format == "int8":
        assert w.head_dim == 128 and w.kv_layout == "head"
        pools = []
        for name in ("k_pool", "v_pool"):
            pool = torch.empty((nb, w.n_kv_heads, KV_UNIT_INT8), dtype=torch.uint8, device=device)
            codes = _codes((nb, w.n_kv_heads, BLOCK_TOKENS * 128), seed, name, layer, device)
            pool[:, :, :BLOCK_TOKENS * 128] = codes.view(torch.uint8)
            sc = _scales((nb, w.n_kv_heads, BLOCK_TOKENS), 1.0, seed, name, layer, device)
            pool[:, :, BLOCK_TOKENS * 128:] = sc.view(torch.uint8)
            pools.append(pool)
        return pools[0], pools[1]
    if w.kv_layout == "token":
        k = _normal((nb, BLOCK_TOKENS, w.n_kv_heads, w.head_dim), 1.0, 0.0, seed, "k_pool", layer, device)
        v = _normal((nb, BLOCK_TOKENS, w.n_kv_heads, w.head_dim), 1.0, 0.0, seed, "v_pool", layer, device)
        return k, v
    k = _normal((nb, w.n_kv_heads, BLOCK_TOKENS, w.head_dim), 1.0, 0.0, seed, "k_pool", layer, device)
    v = _normal((nb, w.n_kv_heads, w.head_dim, BLOCK_TOKENS), 1.0, 0.0, seed, "v_pool", layer, device)
    return k, v


def page_table(w: Workload, seed: int = 2501, n_blocks=None):
    """int32 [batch, blocks_per_seq]: a seeded shuffle of the pool's block ids dealt to the
    sequences (every logical block gets a distinct physical block).  CPU tensor."""
    nb = w.pool_blocks if n_blocks is None else int(n_blocks)
    need = w.batch * w.blocks_per_seq
    assert nb >= need
    perm = torch.randperm(nb, generator=_gen(seed, "page_table", 0, "cpu"))
    return perm[:need].to(torch.int32).reshape(w.batch, w.blocks_per_seq).contiguous()


def seq_lens(w: Workload):
    """Static batching with equal lengths (Section 4, "Experimental setup")."""
    return torch.full((w.batch,), w.context, dtype=torch.int32)


def x_in(w: Workload, seed: int = 2501, device="cpu"):
    """fp32 [batch, hidden] residual-stream input; values are bf16-representable N(0,1)."""
    return _normal((w.batch, w.hidden), 1.0, 0.0, seed, "x", 0, device).to(torch.float32)


def bits(t: torch.Tensor):
    """Host copy as numpy: raw bf16 bit patterns (uint16) for bf16 tensors, the values themselves for int8 codes,
    uint8 pools and fp32 scales."""
    if t.dtype == torch.bfloat16:
        return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")
    assert t.dtype in (torch.int8, torch.uint8, torch.float32)
    return t.detach().cpu().contiguous().numpy()
