"""Pins for oracle/model.py: each test checks the oracle against something other than itself
(brute force, a closed form, an invariant, or a differently-structured dense computation)."""
import math

import numpy as np
import pytest

import workloads as W
from oracle import (ContiguousKV, OracleModel, PagedKV, gqa_attention, log_prob, paged_decode_attention,
                    rmsnorm, rope, silu, softmax)


def _r(seed):
    return np.random.default_rng(seed)


# ---------------- attention ----------------------------------------------------------------
@pytest.mark.parametrize("G", [1, 4, 5])
@pytest.mark.parametrize("T", [1, 15, 16, 17, 33])
def test_attention_matches_bruteforce_score_matrix(G, T):
    """Causal attention via the explicit H x T x T score matrix, in float64."""
    Hkv, d = 2, 8
    Hq = Hkv * G
    g = _r(100 + G * 40 + T)
    q = g.standard_normal((T, Hq, d))
    k = g.standard_normal((T, Hkv, d))
    v = g.standard_normal((T, Hkv, d))
    S = np.full((Hq, T, T), -np.inf)
    for h in range(Hq):
        for i in range(T):
            for j in range(i + 1):
                S[h, i, j] = sum(q[i, h, e] * k[j, h // G, e] for e in range(d)) / math.sqrt(d)
    P = np.exp(S - S.max(axis=2, keepdims=True))
    P /= P.sum(axis=2, keepdims=True)
    assert np.allclose(P.sum(axis=2), 1.0, atol=1e-12)
    for i in range(T):
        ref = np.stack([P[h, i, :] @ v[:, h // G, :] for h in range(Hq)])
        got = gqa_attention(q[i], k[: i + 1], v[: i + 1])
        assert np.allclose(got, ref, atol=1e-12)


def test_softmax_rows_sum_to_one_and_are_shift_invariant():
    x = _r(1).standard_normal((7, 50)) * 30
    p = softmax(x)
    assert np.allclose(p.sum(axis=-1), 1.0, atol=1e-12)
    assert np.allclose(p, softmax(x + 1234.5), atol=1e-12)
    assert np.all(p >= 0)


def test_attention_single_token_returns_v_exactly():
    g = _r(2)
    q, k, v = g.standard_normal((8, 16)), g.standard_normal((1, 2, 16)), g.standard_normal((1, 2, 16))
    o = gqa_attention(q, k, v)
    for j in range(8):
        assert np.array_equal(o[j], v[0, j // 4])


def test_attention_equal_keys_returns_mean_of_v():
    g = _r(3)
    T = 23
    q = g.standard_normal((4, 8))
    k = np.repeat(g.standard_normal((1, 2, 8)), T, axis=0)
    v = g.standard_normal((T, 2, 8))
    o = gqa_attention(q, k, v)
    for j in range(4):
        assert np.allclose(o[j], v[:, j // 2].mean(axis=0), atol=1e-12)


def test_attention_uses_the_right_kv_head_and_scale():
    """One dominant key per kv head: output must pick that head's value row; scale 1/sqrt(d) checked
    through a two-key case with a known probability."""
    d = 4
    q = np.array([[2.0, 0, 0, 0], [0, 2.0, 0, 0]])          # Hq = 2, Hkv = 2, G = 1
    k = np.zeros((2, 2, d))
    k[1, 0, 0] = 3.0                                         # head 0: key 1 scores 6/2 = 3, key 0 scores 0
    k[0, 1, 1] = 1.0                                         # head 1: key 0 scores 2/2 = 1
    v = np.arange(16, dtype=np.float64).reshape(2, 2, d)
    o = gqa_attention(q, k, v)
    p0 = 1.0 / (1.0 + math.exp(3.0))
    assert np.allclose(o[0], p0 * v[0, 0] + (1 - p0) * v[1, 0], atol=1e-14)
    p1 = 1.0 / (1.0 + math.exp(-1.0))
    assert np.allclose(o[1], p1 * v[0, 1] + (1 - p1) * v[1, 1], atol=1e-14)


def test_paged_decode_attention_equals_contiguous():
    g = _r(4)
    lens = np.array([1, 15, 16, 17, 40])
    table, n_pool = W.make_page_table(lens, 16, seed=9)
    Hq, Hkv, d = 8, 2, 16
    q = g.standard_normal((len(lens), Hq, d))
    kp = np.full((n_pool, 16, Hkv, d), np.nan)
    vp = np.full((n_pool, 16, Hkv, d), np.nan)
    ref = []
    for i, L in enumerate(lens):
        k, v = g.standard_normal((L, Hkv, d)), g.standard_normal((L, Hkv, d))
        for t in range(L):
            kp[table[i, t // 16], t % 16] = k[t]
            vp[table[i, t // 16], t % 16] = v[t]
        ref.append(gqa_attention(q[i], k, v))
    got = paged_decode_attention(q, kp, vp, table, lens)
    assert np.array_equal(got, np.stack(ref))


# ---------------- RoPE ----------------------------------------------------------------------
def test_rope_identity_at_position_zero_is_bit_exact():
    x = _r(5).standard_normal((3, 32))
    assert np.array_equal(rope(x, 0, 1e4), x)
    x32 = x.astype(np.float32)
    assert np.array_equal(rope(x32, 0, 5e5), x32)


def test_rope_preserves_pair_norms_and_pairs_i_with_i_plus_half():
    d = 32
    x = _r(6).standard_normal((2, d))
    y = rope(x, 1234, 1e4)
    n_in = x[:, : d // 2] ** 2 + x[:, d // 2:] ** 2
    n_out = y[:, : d // 2] ** 2 + y[:, d // 2:] ** 2
    assert np.allclose(n_in, n_out, atol=1e-12)
    # explicit angle for pair i: pos * theta^(-2i/d)
    e = np.zeros(d)
    e[3] = 1.0
    ang = 7 * 1e4 ** (-2 * 3 / d)
    r = rope(e, 7, 1e4)
    assert abs(r[3] - math.cos(ang)) < 1e-15 and abs(r[3 + d // 2] - math.sin(ang)) < 1e-15


def test_rope_scores_depend_only_on_relative_position():
    d = 32
    g = _r(7)
    q, k = g.standard_normal(d), g.standard_normal(d)
    a = rope(q, 100, 5e5) @ rope(k, 60, 5e5)
    b = rope(q, 16895, 5e5) @ rope(k, 16855, 5e5)
    assert abs(a - b) < 1e-9


# ---------------- RMSNorm / SwiGLU ---------------------------------------------------------
def test_rmsnorm_closed_forms():
    c, eps, n = 3.0, 1e-5, 64
    gain = np.linspace(0.5, 1.5, n)
    out = rmsnorm(np.full(n, c), gain, eps)
    assert np.allclose(out, c / math.sqrt(c * c + eps) * gain, atol=1e-15)
    x = _r(8).standard_normal(n)
    y = rmsnorm(x, np.ones(n), eps)
    ms = np.mean(x * x)
    assert abs(np.mean(y * y) - ms / (ms + eps)) < 1e-12
    assert np.allclose(rmsnorm(5 * x, np.ones(n), 0.0), rmsnorm(x, np.ones(n), 0.0), atol=1e-12)


def test_silu_values():
    assert silu(np.array([0.0]))[0] == 0.0
    assert abs(silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(silu(np.array([-2.0]))[0] - (-2.0 / (1.0 + math.exp(2.0)))) < 1e-15


# ---------------- whole network --------------------------------------------------------------
def _tiny(seed=1, **kw):
    base = dict(n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24, vocab=20,
                rms_eps=1e-5, rope_theta=1e4, qkv_bias=1)
    base.update(kw)
    m = W.ModelShape(**base)
    g = _r(seed)
    w = {n: g.standard_normal((r, c)) * 0.3 for n, r, c in W.weight_layout(m)}
    for n in w:
        if n.endswith("norm"):
            w[n] = 1.0 + 0.1 * g.standard_normal(w[n].shape)
    return m, w


def _dense_forward(m, w, toks):
    """All positions at once with an explicit causal mask: no cache, no per-token loop."""
    T = len(toks)
    G = m.n_q_heads // m.n_kv_heads
    d = m.head_dim
    h = w["embed"][toks]
    pos = np.arange(T)[:, None]
    i = np.arange(d // 2)[None, :]
    ang = pos * (m.rope_theta ** (-2.0 * i / d))
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]

    def rot(x):                                            # x [T, H, d]
        a, b = x[..., : d // 2], x[..., d // 2:]
        return np.concatenate([a * cos - b * sin, b * cos + a * sin], axis=-1)

    mask = np.where(np.arange(T)[None, :] <= np.arange(T)[:, None], 0.0, -np.inf)
    for l in range(m.n_layers):
        p = f"l{l}."
        a = h / np.sqrt((h * h).mean(-1, keepdims=True) + m.rms_eps) * w[p + "attn_norm"]
        q = (a @ w[p + "wq"].T + w[p + "bq"]).reshape(T, m.n_q_heads, d)
        k = (a @ w[p + "wk"].T + w[p + "bk"]).reshape(T, m.n_kv_heads, d)
        v = (a @ w[p + "wv"].T + w[p + "bv"]).reshape(T, m.n_kv_heads, d)
        q, k = rot(q), rot(k)
        kk, vv = np.repeat(k, G, axis=1), np.repeat(v, G, axis=1)
        s = np.einsum("ihd,jhd->hij", q, kk) / math.sqrt(d) + mask[None]
        pr = np.exp(s - s.max(-1, keepdims=True))
        pr /= pr.sum(-1, keepdims=True)
        o = np.einsum("hij,jhd->ihd", pr, vv).reshape(T, -1)
        h = h + o @ w[p + "wo"].T
        mm = h / np.sqrt((h * h).mean(-1, keepdims=True) + m.rms_eps) * w[p + "ffn_norm"]
        gate = mm @ w[p + "w_gate"].T
        h = h + (gate / (1 + np.exp(-gate)) * (mm @ w[p + "w_up"].T)) @ w[p + "w_down"].T
    hf = h / np.sqrt((h * h).mean(-1, keepdims=True) + m.rms_eps) * w["final_norm"]
    return hf @ w["lm_head"].T


def test_incremental_decode_equals_dense_causal_forward_at_every_step():
    m, w = _tiny()
    toks = list(_r(11).integers(0, m.vocab, 21))
    ref = _dense_forward(m, w, toks)
    model = OracleModel(m, w)
    cache = ContiguousKV(m.n_layers)
    for t, tok in enumerate(toks):
        lg = model.token_forward(int(tok), t, cache)
        assert np.allclose(lg, ref[t], atol=1e-10), t
    # full-prefix recompute of a prefix agrees too
    assert np.allclose(model.full_recompute(toks[:9]), ref[8], atol=1e-10)


def test_paged_cache_equals_contiguous_cache_bit_exact():
    m, w = _tiny(seed=2)
    toks = list(_r(12).integers(0, m.vocab, 37))
    model = OracleModel(m, w)
    a = ContiguousKV(m.n_layers)
    pool = PagedKV(m.n_layers, 9, 16, m.n_kv_heads, m.head_dim, np.float64)
    b = pool.view([7, 2, 5])
    for t, tok in enumerate(toks):
        assert np.array_equal(model.token_forward(int(tok), t, a), model.token_forward(int(tok), t, b))


def test_zero_output_projections_give_closed_form_logits():
    """Wo = Wd = 0 makes every layer the identity: logits = rms(E[tok]) Wlm^T."""
    m, w = _tiny(seed=3)
    for l in range(m.n_layers):
        w[f"l{l}.wo"][:] = 0
        w[f"l{l}.w_down"][:] = 0
    model = OracleModel(m, w)
    cache = ContiguousKV(m.n_layers)
    for t, tok in enumerate([3, 7, 7, 1]):
        e = w["embed"][tok]
        ref = w["lm_head"] @ (e / math.sqrt(float(np.mean(e * e)) + m.rms_eps) * w["final_norm"][0])
        assert np.allclose(model.token_forward(tok, t, cache), ref, atol=1e-12)


def test_single_layer_single_token_by_scalar_loops():
    """P = 1: softmax over one position is 1, so o = v; everything else by scalar loops."""
    m, w = _tiny(seed=4, n_layers=1, n_q_heads=2, n_kv_heads=1, head_dim=4, d_model=6, d_ffn=5, vocab=7)
    tok = 4
    D, F = m.d_model, m.d_ffn

    def rms(x, g):
        s = math.sqrt(sum(t * t for t in x) / len(x) + m.rms_eps)
        return [x[i] / s * g[i] for i in range(len(x))]

    h = [float(t) for t in w["embed"][tok]]
    a = rms(h, w["l0.attn_norm"][0])
    v = [sum(w["l0.wv"][o, i] * a[i] for i in range(D)) + w["l0.bv"][0, o] for o in range(m.head_dim)]
    att = v + v                                            # both query heads read the single kv head
    h = [h[o] + sum(w["l0.wo"][o, i] * att[i] for i in range(2 * m.head_dim)) for o in range(D)]
    mm = rms(h, w["l0.ffn_norm"][0])
    gate = [sum(w["l0.w_gate"][f, i] * mm[i] for i in range(D)) for f in range(F)]
    up = [sum(w["l0.w_up"][f, i] * mm[i] for i in range(D)) for f in range(F)]
    act = [gate[f] / (1 + math.exp(-gate[f])) * up[f] for f in range(F)]
    h = [h[o] + sum(w["l0.w_down"][o, f] * act[f] for f in range(F)) for o in range(D)]
    hf = rms(h, w["final_norm"][0])
    ref = [sum(w["lm_head"][o, i] * hf[i] for i in range(D)) for o in range(m.vocab)]
    got = OracleModel(m, w).full_recompute([tok])
    assert np.allclose(got, ref, atol=1e-12)


def test_log_prob_is_log_of_softmax_and_greedy_is_max_prob():
    lg = _r(13).standard_normal(50) * 5
    p = softmax(lg)
    for t in (0, 17, int(np.argmax(lg))):
        assert abs(math.exp(log_prob(lg, t)) - p[t]) < 1e-12
    assert 0 < math.exp(log_prob(lg, int(np.argmax(lg)))) <= 1


def test_greedy_token_ties_go_to_the_lowest_index():
    """Exact ties at the maximum: inside one run of positions, far apart, at both ends, everywhere; and entries that
    differ only below binary32 resolution tie as well (logits are compared as fp32)."""
    from oracle import greedy_token
    x = np.array([0.5, 2.0, -1.0, 2.0, 2.0, 1.0])
    assert greedy_token(x) == 1
    assert greedy_token(x[::-1].copy()) == 1               # reversed: maxima at 1, 2, 4
    y = np.full(5000, -3.0)
    y[[4096, 17]] = 7.25
    assert greedy_token(y) == 17
    y[0] = y[4999] = 7.25
    assert greedy_token(y) == 0
    assert greedy_token(np.zeros(33)) == 0
    assert greedy_token(np.array([1.0, 3.0, 3.0 + 1e-12, 2.0])) == 1      # equal after rounding to binary32
    assert greedy_token(np.array([1.0, 3.0, 3.0 + 1e-6, 2.0])) == 2       # distinct in binary32
    assert greedy_token(np.array([-np.inf, -5.0, -5.0])) == 1


def test_float32_oracle_tracks_float64():
    m, w = _tiny(seed=5)
    toks = list(_r(14).integers(0, m.vocab, 12))
    a = OracleModel(m, w, np.float64).full_recompute(toks)
    b = OracleModel(m, w, np.float32).full_recompute(toks)
    assert b.dtype == np.float32
    assert np.max(np.abs(a - b)) < 1e-4
