"""CPU oracle for the policy forward pass of the rollout phase.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product path never does, and it shares no code with the HIP
library.

The paper (Sec. 2.2, Sec. 4.1) only names the policies (LLaMA-3.1-8B,
Qwen-2.5-32B) and says rollout is bound by streaming weights and KV caches; it
does not write the forward pass down.  What is computed here is therefore the
textbook pre-norm decoder those model families use, spelled out with no
blocking, fusion or reordering:

    h = E[tok]
    per layer:  a = rms(h, g1);  q,k,v = a Wq^T (+bq), a Wk^T (+bk), a Wv^T (+bv)
                q,k <- rope(q,k,pos);  cache k,v at position pos
                o_j = softmax(q_j . K_{j//G}^T / sqrt(d)) . V_{j//G}   over positions 0..pos
                h += concat(o) Wo^T;  m = rms(h, g2);  h += (silu(m Wg^T) * (m Wu^T)) Wd^T
    logits = rms(h, gf) Wlm^T

Weights are [out, in] row-major.  Arithmetic runs in `dtype` (float64 unless the
caller asks for float32); softmax is the two-pass max-subtracted form.

Pinned by tests/test_oracle_model.py: brute-force T x T attention in float64,
softmax rows summing to 1, single-token context returning V, equal keys
returning mean(V), RoPE identity at position 0 / norm preservation / relative
property, RMSNorm closed forms, SwiGLU and projections against a scalar triple
loop, incremental decode == full-prefix recompute, paged == contiguous cache,
and the Wo = Wd = 0 closed form for the whole network.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope_cos_sin(pos: int, head_dim: int, theta: float):
    """cos/sin of pos * theta^(-2i/d), i = 0..d/2-1, evaluated in float64."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    ang = float(pos) * np.power(float(theta), -2.0 * i / head_dim)
    return np.cos(ang), np.sin(ang)


def rope(x: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotate-half RoPE on the last axis: dim i pairs with dim i + d/2."""
    d = x.shape[-1]
    c, s = rope_cos_sin(pos, d, theta)
    c, s = c.astype(x.dtype), s.astype(x.dtype)
    x1, x2 = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def gqa_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query token.  q [Hq, d]; K, V [T, Hkv, d] -> o [Hq, d].

    Query head j reads kv head j // (Hq // Hkv).
    """
    Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    o = np.empty_like(q)
    for j in range(Hq):
        kv = j // G
        p = softmax(K[:, kv, :] @ q[j] / math.sqrt(d))
        o[j] = p @ V[:, kv, :]
    return o


class ContiguousKV:
    """Per-sequence, per-layer K/V lists in position order."""

    def __init__(self, n_layers: int):
        self.k: List[List[np.ndarray]] = [[] for _ in range(n_layers)]
        self.v: List[List[np.ndarray]] = [[] for _ in range(n_layers)]

    def put(self, layer: int, pos: int, k: np.ndarray, v: np.ndarray) -> None:
        assert pos == len(self.k[layer])
        self.k[layer].append(k)
        self.v[layer].append(v)

    def get(self, layer: int, n: int):
        return np.stack(self.k[layer][:n]), np.stack(self.v[layer][:n])


class PagedKV:
    """A pool of fixed-size pages shared by all sequences; a view binds one sequence's page list."""

    def __init__(self, n_layers: int, n_pages: int, page_tokens: int, n_kv_heads: int, head_dim: int, dtype):
        shape = (n_layers, n_pages, page_tokens, n_kv_heads, head_dim)
        self.k = np.full(shape, np.nan, dtype=dtype)
        self.v = np.full(shape, np.nan, dtype=dtype)
        self.page_tokens = page_tokens

    def view(self, pages: Sequence[int]) -> "_PagedView":
        return _PagedView(self, pages)


class _PagedView:
    def __init__(self, pool: PagedKV, pages: Sequence[int]):
        self.pool, self.pages = pool, pages

    def put(self, layer: int, pos: int, k: np.ndarray, v: np.ndarray) -> None:
        pt = self.pool.page_tokens
        page = self.pages[pos // pt]
        self.pool.k[layer, page, pos % pt] = k
        self.pool.v[layer, page, pos % pt] = v

    def get(self, layer: int, n: int):
        pt = self.pool.page_tokens
        idx = [self.pages[i // pt] for i in range(n)]
        off = [i % pt for i in range(n)]
        return self.pool.k[layer, idx, off], self.pool.v[layer, idx, off]


class OracleModel:
    """The decoder-only policy.  `weights` maps tensor names (workloads.weight_layout) to float arrays."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], dtype=np.float64):
        self.m = shape
        self.dtype = dtype
        self.w = {k: np.asarray(v, dtype=dtype) for k, v in weights.items()}

    # one token at absolute position `pos`, reading and extending `cache`
    def token_forward(self, tok: int, pos: int, cache) -> np.ndarray:
        m, w = self.m, self.w
        h = self.w["embed"][tok].copy()
        for l in range(m.n_layers):
            p = f"l{l}."
            a = rmsnorm(h, w[p + "attn_norm"][0], m.rms_eps)
            q = w[p + "wq"] @ a
            k = w[p + "wk"] @ a
            v = w[p + "wv"] @ a
            if m.qkv_bias:
                q, k, v = q + w[p + "bq"][0], k + w[p + "bk"][0], v + w[p + "bv"][0]
            q = rope(q.reshape(m.n_q_heads, m.head_dim), pos, m.rope_theta)
            k = rope(k.reshape(m.n_kv_heads, m.head_dim), pos, m.rope_theta)
            v = v.reshape(m.n_kv_heads, m.head_dim)
            cache.put(l, pos, k, v)
            K, V = cache.get(l, pos + 1)
            o = gqa_attention(q, K, V)
            h = h + w[p + "wo"] @ o.reshape(-1)
            mm = rmsnorm(h, w[p + "ffn_norm"][0], m.rms_eps)
            h = h + w[p + "w_down"] @ (silu(w[p + "w_gate"] @ mm) * (w[p + "w_up"] @ mm))
        return self.w["lm_head"] @ rmsnorm(h, w["final_norm"][0], m.rms_eps)

    def run_tokens(self, toks: Sequence[int], pos0: int, cache) -> np.ndarray:
        """Feed toks at positions pos0.. through the model; returns the logits after the last one."""
        logits = None
        for i, t in enumerate(toks):
            logits = self.token_forward(int(t), pos0 + i, cache)
        return logits

    def full_recompute(self, toks: Sequence[int]) -> np.ndarray:
        """Logits after the last token, recomputed from an empty cache."""
        return self.run_tokens(toks, 0, ContiguousKV(self.m.n_layers))


def greedy_token(logits: np.ndarray) -> int:
    """argmax with the lowest index winning ties; the logits are compared as binary32 values (the precision the
    engine's logits have), so two entries that round to the same binary32 number tie."""
    return int(np.argmax(np.asarray(logits, dtype=np.float32)))


def log_prob(logits: np.ndarray, tok: int) -> float:
    """log softmax(logits)[tok]."""
    mx = float(np.max(logits))
    return float(logits[tok] - mx - math.log(float(np.sum(np.exp(logits - mx)))))


def paged_decode_attention(q: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray,
                           page_table: np.ndarray, lens: np.ndarray) -> np.ndarray:
    """Ragged decode attention alone: one query token per sequence over its paged KV.

    q [n, Hq, d]; k_pool, v_pool [n_pages, page_tokens, Hkv, d]; page_table [n, max_pages];
    lens [n] -> o [n, Hq, d].
    """
    n = q.shape[0]
    pt = k_pool.shape[1]
    out = np.empty_like(q)
    for i in range(n):
        L = int(lens[i])
        pages = page_table[i, : (L + pt - 1) // pt]
        K = k_pool[pages].reshape(-1, *k_pool.shape[2:])[:L]
        V = v_pool[pages].reshape(-1, *v_pool.shape[2:])[:L]
        out[i] = gqa_attention(q[i], K, V)
    return out
