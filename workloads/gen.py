"""Seeded generators for the synthetic rollout workloads.

Every draw comes from numpy's Philox generator keyed by an explicit seed, so
the same call yields the same arrays on every machine that runs this image.
bf16 values are carried as uint16 bit patterns (the high half of an IEEE
binary32 word, rounded to nearest-even).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Tuple

import numpy as np

__all__ = [
    "ModelShape", "Workload", "CONFIGS", "rng", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "weight_layout", "weight_count", "make_weights", "split_weights", "make_prompts",
    "make_target_lengths", "make_kv_lengths", "make_page_table", "make_attention_case",
]


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float
    rope_theta: float
    qkv_bias: int = 0

    @property
    def eos_id(self) -> int:
        return self.vocab - 1

    def with_layers(self, n_layers: int) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    n_prompts: int          # prompts loaded per group (the queue the engine is oversubscribed with)
    prompt_len: int
    len_mu: float           # LogNormal location of the output length (ln of the median)
    len_sigma: float
    cap: int                # max_new_tokens
    max_slots: int          # Q, the running-queue size
    harvest: int            # update-group size handed to rollout_harvest
    page_tokens: int = 16
    kv_pool_bytes: int = 0  # 0 = sized for the worst case
    max_staleness: int = -1
    seed_weights: int = 1
    seed_prompts: int = 2
    seed_lengths: int = 3


_TINY = ModelShape(2, 128, 4, 4, 32, 512, 512, 1e-5, 1e4, 0)
_LLAMA8B = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 5e5, 0)
_QWEN32B = ModelShape(64, 5120, 40, 8, 128, 27648, 152064, 1e-6, 1e6, 1)

CONFIGS: Dict[str, Workload] = {
    # tiny fp32-sized policy the oracle finishes in seconds
    "tiny": Workload("tiny", _TINY, 8, 16, 3.0, 0.6, 64, 8, 4),
    # LLaMA-3.1-8B shape, 8k cap
    "8b": Workload("8b", _LLAMA8B, 512, 512, math.log(1024.0), 0.9, 8192, 128, 32),
    # same shape, long-trajectory regime: 16k cap, 160 GB KV pool, staleness 1
    "8b_long": Workload("8b_long", _LLAMA8B, 1024, 512, math.log(2048.0), 1.0, 16384, 256, 64,
                        kv_pool_bytes=160 * 10**9, max_staleness=1),
    # Qwen-2.5-32B shape
    "32b": Workload("32b", _QWEN32B, 256, 512, math.log(1536.0), 0.9, 8192, 64, 16),
}

# decode-attention-alone case: 256 sequences, 32 q / 8 kv heads, head_dim 128
ATTN_CASE = dict(n_seqs=256, n_q_heads=32, n_kv_heads=8, head_dim=128, median=2048, sigma=0.8,
                 cap=16384, page_tokens=16, seed_lengths=4, seed_values=5, seed_pages=6)
__all__.append("ATTN_CASE")


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if np.any(nan):
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def weight_layout(m: ModelShape) -> List[Tuple[str, int, int]]:
    """Order and [rows=out, cols=in] shape of every tensor in the weights blob.

    Matrices are row-major [out, in] (y = x @ W.T); gains and biases are [1, n].
    """
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    lay: List[Tuple[str, int, int]] = [("embed", m.vocab, m.d_model)]
    for l in range(m.n_layers):
        p = f"l{l}."
        lay += [(p + "attn_norm", 1, m.d_model), (p + "wq", qd, m.d_model),
                (p + "wk", kvd, m.d_model), (p + "wv", kvd, m.d_model)]
        if m.qkv_bias:
            lay += [(p + "bq", 1, qd), (p + "bk", 1, kvd), (p + "bv", 1, kvd)]
        lay += [(p + "wo", m.d_model, qd), (p + "ffn_norm", 1, m.d_model),
                (p + "w_gate", m.d_ffn, m.d_model), (p + "w_up", m.d_ffn, m.d_model),
                (p + "w_down", m.d_model, m.d_ffn)]
    lay += [("final_norm", 1, m.d_model), ("lm_head", m.vocab, m.d_model)]
    return lay


def weight_count(m: ModelShape) -> int:
    return sum(r * c for _, r, c in weight_layout(m))


def make_weights(m: ModelShape, seed: int, std: float = 0.02) -> np.ndarray:
    """bf16 blob (uint16) in weight_layout order: N(0, std) everywhere, norm gains 1.0."""
    g = rng(seed)
    out = np.empty(weight_count(m), dtype=np.uint16)
    off = 0
    for name, r, c in weight_layout(m):
        n = r * c
        if name.endswith("norm"):
            out[off:off + n] = 0x3F80
        else:
            done = 0
            while done < n:  # draw in slabs to bound host memory
                k = min(n - done, 1 << 26)
                out[off + done:off + done + k] = f32_to_bf16_bits(
                    g.standard_normal(k, dtype=np.float32) * np.float32(std))
                done += k
        off += n
    return out


def split_weights(blob: np.ndarray, m: ModelShape) -> Dict[str, np.ndarray]:
    """Views of the uint16 blob, one [rows, cols] array per tensor."""
    d, off = {}, 0
    for name, r, c in weight_layout(m):
        d[name] = blob[off:off + r * c].reshape(r, c)
        off += r * c
    assert off == blob.size
    return d


def make_prompts(n: int, prompt_len: int, vocab: int, seed: int) -> np.ndarray:
    """int32 [n, prompt_len], ids uniform on [0, vocab-1) (the last id is reserved for EOS)."""
    return rng(seed).integers(0, vocab - 1, size=(n, prompt_len), dtype=np.int64).astype(np.int32)


def _lognormal_lengths(n: int, mu: float, sigma: float, cap: int, seed: int) -> np.ndarray:
    z = rng(seed).standard_normal(n)  # float64
    return np.minimum(cap, np.maximum(1, np.ceil(np.exp(mu + sigma * z)))).astype(np.int32)


def make_target_lengths(n: int, mu: float, sigma: float, cap: int, seed: int) -> np.ndarray:
    """Output lengths L_i = min(cap, max(1, ceil(LogNormal(mu, sigma)))), int32 [n]."""
    return _lognormal_lengths(n, mu, sigma, cap, seed)


def make_kv_lengths(n: int, median: float, sigma: float, cap: int, seed: int) -> np.ndarray:
    return _lognormal_lengths(n, math.log(median), sigma, cap, seed)


def make_page_table(lens: np.ndarray, page_tokens: int, seed: int, pool_factor: float = 1.25
                    ) -> Tuple[np.ndarray, int]:
    """Scatter each sequence's pages over a pool by a seeded permutation.

    Returns (table int32 [n, max_pages] padded with -1, n_pool_pages).
    """
    need = (np.asarray(lens, dtype=np.int64) + page_tokens - 1) // page_tokens
    total = int(need.sum())
    n_pool = max(total, int(math.ceil(total * pool_factor)))
    perm = rng(seed).permutation(n_pool).astype(np.int32)
    table = np.full((len(lens), int(need.max()) if len(lens) else 0), -1, dtype=np.int32)
    at = 0
    for i, k in enumerate(need):
        table[i, :k] = perm[at:at + k]
        at += int(k)
    return table, n_pool


def make_attention_case(lens: np.ndarray, n_q_heads: int, n_kv_heads: int, head_dim: int, seed: int):
    """q [n, Hq, d] and per-sequence k, v [len_i, Hkv, d], all N(0,1) rounded to bf16 (uint16 bits).

    k and v are returned as flat [sum(len), Hkv, d] arrays with the row offsets of each sequence.
    """
    g = rng(seed)
    n = len(lens)
    q = f32_to_bf16_bits(g.standard_normal((n, n_q_heads, head_dim), dtype=np.float32))
    offs = np.zeros(n + 1, dtype=np.int64)
    offs[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    tot = int(offs[-1])
    k = np.empty((tot, n_kv_heads, head_dim), dtype=np.uint16)
    v = np.empty((tot, n_kv_heads, head_dim), dtype=np.uint16)
    step = 1 << 15
    for a in range(0, tot, step):
        b = min(tot, a + step)
        k[a:b] = f32_to_bf16_bits(g.standard_normal((b - a, n_kv_heads, head_dim), dtype=np.float32))
        v[a:b] = f32_to_bf16_bits(g.standard_normal((b - a, n_kv_heads, head_dim), dtype=np.float32))
    return q, k, v, offs
