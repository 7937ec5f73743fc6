"""Device-side set-up of a synthetic workload around the C-ABI library: allocation (torch), seeded
fill (synth) and pointer hand-over (binding).  No arithmetic of the decode step lives here."""
import torch

from . import binding as psv
from . import synth


def default_policy(w: synth.Workload, **overrides):
    """The prefetch-on policy that bench.py times by default: budget C = min(192 MiB, longest window x 4.5 MiB/us)
    (what the prefetch kernel can pull inside the window), 256 prefetch workgroups, an operator that does not fit the rest
    of the budget prefetched in part (a KV cache or a wide projection can exceed any budget), first consumer of a window
    launched into the window."""
    kw = dict(mode=1, budget_bytes=int(min(192.0, max(w.window_us) * 4.5) * (1 << 20)), cu_budget=256,
              partial=1, prelaunch=1)
    kw.update(overrides)
    return psv.prefetch_policy(**kw)


class Session:
    """One workload resident on one GPU: weights, KV pools, page table, streams and a library context.

    layers: which layers to materialise (default all); others cannot be run.
    """

    def __init__(self, w: synth.Workload, seed=2501, device="cuda:0", layers=None, pool_slack_blocks=0, max_seq=None,
                 fused=None):
        if not torch.cuda.is_available():
            raise RuntimeError("the PRESERVE decode path needs a GPU; there is no CPU fallback")
        self.w = w
        self.seed = seed
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.layers = list(range(w.n_layers)) if layers is None else list(layers)
        # longest sequence the context is created for; the cache itself always has room for w.context tokens
        self.max_seq = (w.context + 15) // 16 * 16 if max_seq is None else int(max_seq)
        self.desc = psv.model_desc(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.ffn, w.batch, self.max_seq,
                                   head_dim=w.head_dim, rms_eps=w.rms_eps, rope_theta=w.rope_theta,
                                   weight_format=w.weight_format, kv_format=w.kv_format, kv_layout=w.kv_layout,
                                   weight_layout=w.weight_layout)
        # HIP maps streams onto a few hardware queues; take a side stream that really runs beside the main one
        self.main = torch.cuda.Stream(device=self.device)
        self.overlap = False
        self._spare_streams = []
        for _ in range(8):
            self.side = torch.cuda.Stream(device=self.device)
            self.ctx = psv.psv_create(self.desc, self.main, self.side)
            self.overlap = psv.psv_check_overlap(self.ctx)
            if self.overlap:
                break
            psv.psv_destroy(self.ctx)
            self._spare_streams.append(self.side)
        else:
            self.ctx = psv.psv_create(self.desc, self.main, self.side)
        if fused is not None:      # None: the library chooses by shape
            psv.psv_set_fused_kernels(self.ctx, int(fused))
        self.pool_blocks = w.pool_blocks + int(pool_slack_blocks)
        self.weights, self.k_pools, self.v_pools = {}, {}, {}
        for l in self.layers:
            self.weights[l] = synth.layer_weights(w, l, seed, self.device)
            if w.weight_layout == "tiled":      # the library gets the tiled copy; the row-major original is dropped
                cur = torch.cuda.current_stream(self.device)     # the stream the generators ran on
                for n in ("w_qkv", "w_o", "w_gate", "w_up", "w_down"):
                    src = self.weights[l][n]
                    dst = torch.empty_like(src)
                    psv.psv_tile_weights(dst, src, src.shape[0], src.shape[1], w.weight_format, cur)
                    self.weights[l][n] = dst
                cur.synchronize()
            self.k_pools[l], self.v_pools[l] = synth.kv_pools(w, l, seed, self.device, n_blocks=self.pool_blocks)
            psv.psv_set_layer_weights(self.ctx, l, self.weights[l])
        self.page_table_host = synth.page_table(w, seed, n_blocks=self.pool_blocks) if w.paged else None
        self.page_table = self.page_table_host.to(self.device) if w.paged else None
        self.seq_lens_host = synth.seq_lens(w)
        self.seq_lens = self.seq_lens_host.to(self.device)
        # layers that are not materialised share the first materialised layer's pools (never run)
        first = self.layers[0]
        kp = [self.k_pools.get(l, self.k_pools[first]) for l in range(w.n_layers)]
        vp = [self.v_pools.get(l, self.v_pools[first]) for l in range(w.n_layers)]
        psv.psv_set_kv(self.ctx, kp, vp, self.page_table, w.blocks_per_seq, self.pool_blocks, self.seq_lens)
        psv.psv_set_comm_windows(self.ctx, float(w.window_us[0]), float(w.window_us[1]))
        self.x_in = synth.x_in(w, seed, self.device)
        self.x_out = torch.empty_like(self.x_in)
        self.set_policy(psv.prefetch_policy(mode=0))
        torch.cuda.synchronize(self.device)

    def set_policy(self, policy):
        self.policy = policy
        psv.psv_set_policy(self.ctx, policy, self.w.batch, min(self.w.context, self.max_seq))

    def set_windows(self, us0, us1):
        psv.psv_set_comm_windows(self.ctx, float(us0), float(us1))

    def tune_attention(self):
        """Times the candidate attention splits on layer 0 and keeps the fastest; returns tokens per workgroup."""
        assert 0 in self.layers
        return psv.psv_tune_attention(self.ctx, self.x_in, self.x_out, self.w.batch)

    def step(self, x_in=None, x_out=None, layer_begin=None, layer_end=None):
        lb = self.layers[0] if layer_begin is None else layer_begin
        le = self.layers[-1] + 1 if layer_end is None else layer_end
        psv.psv_decode_step(self.ctx, self.x_in if x_in is None else x_in, self.x_out if x_out is None else x_out,
                            self.w.batch, lb, le)

    def sync(self):
        psv.psv_sync(self.ctx)

    def run(self, **kw):
        self.step(**kw)
        self.sync()
        return self.x_out

    def close(self):
        if self.ctx is not None:
            psv.psv_sync(self.ctx)
            psv.psv_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False

    # ---- host copies for the oracle (tests / cpu baseline only) ----
    def host_layer(self, l):
        """Row-major host copy of a layer's weights (what the oracle reads), whatever layout the library was given."""
        src = synth.layer_weights(self.w, l, self.seed, self.device) if self.w.weight_layout == "tiled" else self.weights[l]
        return {n: synth.bits(t) for n, t in src.items()}

    def host_pools(self, l):
        return synth.bits(self.k_pools[l]), synth.bits(self.v_pools[l])
