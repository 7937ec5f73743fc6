"""GPU parity of the vector-ALU projections on rows longer than 4096 elements, where a thread covers a weight row
with two 16-byte loads instead of one: 70B-shaped tensor-parallel shards at batch 1 (hidden 8192: the fused
normalisation prologue of QKV and gate/up, also in the variant launched into its window; FFN shards of 3584 and
7168: the plain down projection), an 8B-shaped shard with a 7168-wide FFN at batch 2 (two activation rows per
thread), and the batch-2 / hidden-8192 case that crosses over to the matrix cores.  Each case goes through the C ABI
and is compared with the CPU oracle exactly as in test_gpu_parity / test_gpu_int8 (same tolerance
|gpu - ref| <= 2e-2 + 1e-2*|ref|, same checks of the appended cache rows); every policy must reproduce the
prefetch-off result bit for bit."""
import pytest
import torch

import test_gpu_int8 as q8
import test_gpu_parity as bf
from paper_2501_08192_amd import synth
from paper_2501_08192_amd.harness import Session, default_policy

pytestmark = pytest.mark.gpu

# name, layers, hidden, q heads, kv heads, ffn, batch, context
SHAPES = [
    ("tp8_70b_b1", 2, 8192, 8, 1, 3584, 1, 300),
    ("tp4_70b_b1", 2, 8192, 16, 2, 7168, 1, 257),
    ("tp8_70b_b2", 1, 8192, 8, 1, 3584, 2, 130),
    ("wide_ffn_b2", 2, 4096, 4, 1, 7168, 2, 200),
]
POLICIES = ["off", "cache only", "default"]
WIN = (6.0, 6.0)


def policy_of(name, w):
    return {"off": None,
            "cache only": default_policy(w, budget_bytes=1 << 40, prelaunch=0),
            "default": default_policy(w, budget_bytes=1 << 40)}[name]


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_bf16_matches_oracle(shape, policy):
    name, L, H, nq, nkv, F, B, T = shape
    w = bf.W(name, L, H, nq, nkv, F, B, T, win=WIN)
    bf.check_step(w, seed=81, policy=policy_of(policy, w))


@pytest.mark.parametrize("fmt", q8.FORMATS, ids=["w8kv8", "w8", "kv8"])
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_int8_matches_oracle_and_policies_agree(shape, fmt):
    name, L, H, nq, nkv, F, B, T = shape
    w = q8.W(name, L, H, nq, nkv, F, B, T, fmt, win=WIN)
    q8.check_step(w, seed=82, policy=policy_of("default", w))


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_bf16_policies_bit_identical(shape):
    name, L, H, nq, nkv, F, B, T = shape
    w = bf.W(name, L, H, nq, nkv, F, B, T, win=WIN)
    with Session(w, seed=83) as s:
        off = s.run().clone()
        k_off = [s.k_pools[l].clone() for l in s.layers]
        for pol in ("cache only", "default"):
            s.set_policy(policy_of(pol, w))
            for _ in range(2):
                on = s.run()
                assert torch.equal(on, off), "%s: policy '%s' changes the result" % (name, pol)
            for l, k0 in zip(s.layers, k_off):
                assert torch.equal(s.k_pools[l], k0)
