"""CPU oracle for temperature sampling in the rollout loop.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's rollouts are sampled (Sec. 4.1: several responses per prompt; Sec. 4.4.1 speaks of "sampling
parameters"), but it gives no sampler.  What is defined here: the Gumbel-max form of sampling from
softmax(logits / T) -- token = argmax_j (logits_j / T + g_j), g_j = -log(-log(u_j)) -- with u_j taken from the
counter-based Philox4x32-10 generator (Salmon et al., SC'11) at counter (j, token index, seq_id low, seq_id high)
under key (seed low, seed high).  Being an argmax it does not depend on summation order, so a parallel
implementation can reproduce it exactly up to the rounding of log.  Ties go to the lowest index.

Pinned by tests/test_oracle_sampling.py: the published known-answer vectors of Philox4x32-10, empirical token
frequencies against softmax(logits / T), T -> 0 approaching greedy, and determinism per (seed, seq_id, index).
"""
from __future__ import annotations

import math

import numpy as np

_M0, _M1, _W0, _W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Vectorised over the counter words (arrays or ints); returns the four 32-bit output words as uint64 arrays."""
    c0, c1, c2, c3 = (np.asarray(x, dtype=np.uint64) & _MASK for x in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0, k1 = int(k0) & 0xFFFFFFFF, int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = np.uint64(_M0) * c0
        p1 = np.uint64(_M1) * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0, k1 = (k0 + _W0) & 0xFFFFFFFF, (k1 + _W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def uniforms(vocab: int, seed: int, seq_id: int, index: int) -> np.ndarray:
    """u_j in (0, 1), j = 0..vocab-1: the top 24 bits of the first Philox word, centred in their bin."""
    x0, _, _, _ = philox4x32_10(np.arange(vocab), index, seq_id & 0xFFFFFFFF, (seq_id >> 32) & 0xFFFFFFFF,
                                seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return ((x0 >> np.uint64(8)).astype(np.float64) + 0.5) * 2.0 ** -24


def perturbed_scores(logits: np.ndarray, temperature: float, seed: int, seq_id: int, index: int) -> np.ndarray:
    u = uniforms(len(logits), seed, seq_id, index)
    return np.asarray(logits, dtype=np.float64) / temperature - np.log(-np.log(u))


def sample_token(logits: np.ndarray, temperature: float, seed: int, seq_id: int, index: int) -> int:
    return int(np.argmax(perturbed_scores(logits, temperature, seed, seq_id, index)))


def log_prob_at(logits: np.ndarray, tok: int, temperature: float) -> float:
    """log softmax(logits / T)[tok]: the log-probability the sampler assigned to the token it drew."""
    z = np.asarray(logits, dtype=np.float64) / temperature
    mx = float(z.max())
    return float(z[tok] - mx - math.log(float(np.exp(z - mx).sum())))
