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
        return 2 * (self.qkv_rows * h + h * self.n_q_heads * self.head_dim + 3 * f * h)

    @property
    def kv_bytes_per_layer(self):
        return 2 * 2 * self.batch * self.context * self.n_kv_heads * self.head_dim

    @property
    def layer_bytes(self):
        return self.weight_bytes_per_layer + self.kv_bytes_per_layer

    def scaled(self, **kw):
        return replace(self, **kw)


# The five workloads of the benchmark definition.  c1 is the small case; c2 (one TP=8 shard of
# a Llama-3-8B-shaped model) is the one the headline metric is quoted on.
WORKLOADS = {
    "c1": Workload("c1", 2, 1024, 8, 8, 128, 2816, 1, 256, False, (10.0, 10.0)),
    "c2": Workload("c2", 32, 4096, 4, 1, 128, 1792, 1, 2048, False, (15.0, 15.0)),
    "c3": Workload("c3", 80, 8192, 8, 1, 128, 3584, 8, 4096, False, (20.0, 20.0)),
    "c4": Workload("c4", 32, 4096, 4, 1, 128, 1792, 64, 8192, True, (25.0, 25.0)),
    "c5": Workload("c5", 80, 8192, 8, 1, 128, 3584, 32, 32768, True, (20.0, 20.0)),
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


def layer_weights(w: Workload, layer: int, seed: int = 2501, device="cpu"):
    """bf16 weights of one layer: projections N(0, 0.02^2), norm gains 1 + N(0, 0.02^2)."""
    h, f, nqd = w.hidden, w.ffn, w.n_q_heads * w.head_dim
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
    """bf16 K and V pools of one layer, every slot N(0,1)."""
    nb = w.pool_blocks if n_blocks is None else int(n_blocks)
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
    """Raw bf16 bit patterns of a tensor as a numpy uint16 array (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")
