"""Randomly drawn small policies under teacher forcing: widths, head layouts (group 1, 4 or 5; head_dim 32 or 128), FFN
width, vocabulary size (mostly not a tile multiple), depth, QKV bias and RoPE base all vary, with ragged prompts, tight
pools and staleness evictions on top.  Every logits row of the HIP engine is compared with the oracle's."""
import numpy as np
import pytest

import workloads as W
from tests.test_gpu_rollout import _teacher_forced

pytestmark = pytest.mark.gpu


def draw_shape(g):
    d = int(g.choice([32, 128]))
    group = int(g.choice([1, 4, 5]))
    hkv = int(g.integers(1, 3))
    hq = hkv * group
    if (hq * d) % 64:            # the engine wants n_q_heads * head_dim in multiples of 64
        hkv *= 2
        hq = hkv * group
    D = 64 * int(g.integers(1, 9))
    F = 64 * int(g.integers(1, 13))
    V = int(g.choice([int(g.integers(2, 300)), int(g.integers(300, 3000)), 512, 1024]))
    return W.ModelShape(int(g.integers(1, 4)), D, hq, hkv, d, F, V, float(g.choice([1e-5, 1e-6])),
                        float(g.choice([1e4, 5e5, 1e6])), int(g.integers(0, 2)))


@pytest.mark.parametrize("seed", range(32))
def test_random_policy_teacher_forced(seed):
    g = W.rng(7000 + seed)
    m = draw_shape(g)
    n = int(g.integers(1, 10))
    pmax = int(g.integers(1, 70))
    cap = int(g.integers(1, 30))
    Q = int(g.integers(1, 7))
    prompts = [g.integers(0, max(1, m.vocab - 1), int(k)).astype(np.int32) for k in g.integers(1, pmax + 1, n)]
    L = g.integers(1, cap + 1, n).astype(np.uint32)
    max_pages = (pmax + cap + 15) // 16
    pool = 0 if g.random() < 0.5 else int(max_pages + g.integers(0, max(1, Q * max_pages // 3)))
    stale = int(g.choice([-1, -1, 0, 1]))
    # the bar is relative to the logit scale (tests/_util.py LOGIT_REL_TOL): the 2e-2 of the 128-wide parity gate,
    # carried to other widths by the standard deviation of the oracle's logits
    worst, rows, agree = _teacher_forced(m, W.make_weights(m, 7100 + seed), prompts, L, Q=Q, cap=cap,
                                         G=int(g.integers(1, Q + 2)), max_prompt_len=pmax, kv_pool_pages=pool,
                                         max_staleness=stale, seed_pages=seed)
    assert rows >= int(L.sum())
