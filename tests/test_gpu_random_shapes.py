"""GPU parity on seeded random shapes: hidden and FFN widths, head groupings, batches on both projection paths,
ragged and mixed context lengths, contiguous and paged caches, every storage format, both weight layouts and a mix of
prefetch policies -- each case run through the C ABI and compared with the CPU oracle exactly as the hand-picked cases
of test_gpu_parity / test_gpu_int8 are (same tolerance, same checks of the appended cache rows)."""
import random

import pytest

import test_gpu_int8 as q8
import test_gpu_parity as bf
from paper_2501_08192_amd.harness import default_policy

pytestmark = pytest.mark.gpu


def draw(case):
    rng = random.Random(7000 + case)
    hidden = rng.choice([512, 1024, 1536, 2048, 2560, 4096])
    nkv = rng.choice([1, 1, 2, 3, 4, 8])
    group = rng.choice([1, 2, 4, 5, 8, 16])
    if nkv * group > 32:
        group = max(1, 32 // nkv)
    ffn = rng.choice([256, 768, 1280, 1792, 2816])
    batch = rng.choice([1, 1, 2, 2, 3, 4, 7, 9, 16, 17, 31, 48, 64])
    context = rng.choice([1, 2, 15, 16, 17, 33, 64, 100, 129, 257, 400, 700, 1500])
    layers = rng.choice([1, 2, 2, 3])
    paged = rng.random() < 0.5
    fmt = rng.choice([None, None, ("int8", "int8"), ("int8", "bf16"), ("bf16", "int8")])
    win = rng.choice([(5.0, 5.0), (0.0, 6.0), (12.0, 3.0)])
    lens = [rng.randint(1, context) for _ in range(batch)] if (batch > 1 and rng.random() < 0.4) else None
    policy = rng.choice(["off", "default", "default", "cache only", "small partial"])
    slack = rng.choice([0, 5]) if paged else 0
    # drawn last: the other choices of a case do not depend on it; mostly on the batches whose projections are on the
    # matrix cores anyway, so that the vector-ALU path keeps its share of the cases
    tiled = rng.random() < 0.4 and (batch >= 3 or rng.random() < 0.3)
    return hidden, nkv * group, nkv, ffn, batch, context, layers, paged, fmt, win, lens, policy, slack, tiled


@pytest.mark.parametrize("case", range(32))
def test_random_shape(case):
    hidden, nq, nkv, ffn, batch, context, layers, paged, fmt, win, lens, policy, slack, tiled = draw(case)
    name = "rnd%d" % case
    if fmt is None:
        mod, w = bf, bf.W(name, layers, hidden, nq, nkv, ffn, batch, context, paged=paged, win=win)
    else:
        mod, w = q8, q8.W(name, layers, hidden, nq, nkv, ffn, batch, context, fmt, paged=paged, win=win)
    if tiled:                            # projection matrices in the tiled order (matrix-core projections at every batch)
        w = w.scaled(weight_layout="tiled")
    pol = {"off": None,
           "default": default_policy(w, budget_bytes=1 << 40),
           "cache only": default_policy(w, budget_bytes=1 << 40, prelaunch=0),
           "small partial": default_policy(w, budget_bytes=max(4096, w.weight_bytes_per_layer // 3), partial=1,
                                           chunk_bytes=1 << 16)}[policy]
    mod.check_step(w, seed=500 + case, seq_lens=lens, policy=pol, pool_slack=slack)
