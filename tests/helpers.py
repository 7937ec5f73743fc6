"""Shared test helpers: bf16 bit handling and KV-pool addressing restated from the layout
definition (head-major: K pool [block, kv head, token, channel]; V pool [block, kv head, channel, token];
token-major: both pools [block, token, kv head, channel])."""
import numpy as np
import torch


def to_bits(a):
    """float array (bf16-representable or not) -> bf16 bit patterns, round-to-nearest-even,
    via torch's own conversion."""
    t = torch.as_tensor(np.asarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def from_bits(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def empty_pools(n_blocks, nkv, bt, d, token_major=False):
    if token_major:
        return np.zeros((n_blocks, bt, nkv, d), dtype=np.uint16), np.zeros((n_blocks, bt, nkv, d), dtype=np.uint16)
    k = np.zeros((n_blocks, nkv, bt, d), dtype=np.uint16)
    v = np.zeros((n_blocks, nkv, d, bt), dtype=np.uint16)
    return k, v


def fill_pools(k_dense, v_dense, bt, page_table=None, n_blocks=None, token_major=False):
    """Dense float caches [B, nkv, T, d] -> bf16 pools in the block layout."""
    B, nkv, T, d = k_dense.shape
    mb = (T + bt - 1) // bt
    if n_blocks is None:
        n_blocks = B * mb
    k, v = empty_pools(n_blocks, nkv, bt, d, token_major)
    kb, vb = to_bits(k_dense), to_bits(v_dense)
    for b in range(B):
        for t in range(T):
            blk = b * mb + t // bt if page_table is None else int(page_table[b, t // bt])
            if token_major:
                k[blk, t % bt, :, :] = kb[b, :, t, :]
                v[blk, t % bt, :, :] = vb[b, :, t, :]
            else:
                k[blk, :, t % bt, :] = kb[b, :, t, :]
                v[blk, :, :, t % bt] = vb[b, :, t, :]
    return k, v


def dense_from_pools(k, v, B, T, page_table=None, token_major=False):
    """Inverse of fill_pools: float64 dense caches [B, nkv, T, d]."""
    if token_major:
        n_blocks, bt, nkv, d = k.shape
    else:
        n_blocks, nkv, bt, d = k.shape
    mb = (T + bt - 1) // bt
    kd = np.zeros((B, nkv, T, d))
    vd = np.zeros((B, nkv, T, d))
    kf, vf = from_bits(k), from_bits(v)
    for b in range(B):
        for t in range(T):
            blk = b * mb + t // bt if page_table is None else int(page_table[b, t // bt])
            if token_major:
                kd[b, :, t, :] = kf[blk, t % bt, :, :]
                vd[b, :, t, :] = vf[blk, t % bt, :, :]
            else:
                kd[b, :, t, :] = kf[blk, :, t % bt, :]
                vd[b, :, t, :] = vf[blk, :, :, t % bt]
    return kd, vd


def random_layer(rng, H, nq, nkv, d, F, std=0.1, integer=False):
    """Random bf16 layer weights as uint16 bit arrays."""
    def draw(shape):
        if integer:
            return to_bits(rng.integers(-2, 3, size=shape).astype(np.float32))
        return to_bits(rng.normal(0.0, std, size=shape))
    return {
        "w_qkv": draw(((nq + 2 * nkv) * d, H)),
        "w_o": draw((H, nq * d)),
        "w_gate": draw((F, H)),
        "w_up": draw((F, H)),
        "w_down": draw((H, F)),
        "g_attn": to_bits(1.0 + rng.normal(0, 0.1, size=H)),
        "g_mlp": to_bits(1.0 + rng.normal(0, 0.1, size=H)),
    }
