import numpy as np

import workloads as W


def test_bf16_round_trip_and_ties_to_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -0.02, 0.0], dtype=np.float32)
    y = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.015625
    assert abs(y[3] + 0.02) < 0.02 * 2 ** -8
    assert np.array_equal(W.f32_to_bf16_bits(y), W.f32_to_bf16_bits(x))


def test_lengths_follow_the_stated_rule_and_are_seeded():
    c = W.CONFIGS["8b_long"]
    a = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    b = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    assert np.array_equal(a, b) and a.min() >= 1 and a.max() == c.cap
    assert 1500 < np.median(a) < 2700
    t = W.CONFIGS["tiny"]
    l = W.make_target_lengths(t.n_prompts, t.len_mu, t.len_sigma, t.cap, t.seed_lengths)
    assert l.max() <= 64 and l.min() >= 1


def test_weights_blob_layout():
    m = W.CONFIGS["tiny"].model
    blob = W.make_weights(m, 1)
    assert blob.dtype == np.uint16 and blob.size == W.weight_count(m)
    w = W.split_weights(blob, m)
    assert w["embed"].shape == (512, 128) and w["l1.w_down"].shape == (128, 512)
    assert np.all(w["l0.attn_norm"] == 0x3F80) and np.all(w["final_norm"] == 0x3F80)
    std = W.bf16_bits_to_f32(w["lm_head"]).std()
    assert 0.019 < std < 0.021
    q = W.CONFIGS["32b"].model.with_layers(1)
    names = [n for n, _, _ in W.weight_layout(q)]
    assert "l0.bq" in names and names.index("l0.bq") == names.index("l0.wv") + 1


def test_prompts_never_contain_eos_and_page_table_is_a_partial_permutation():
    p = W.make_prompts(64, 16, 512, 2)
    assert p.min() >= 0 and p.max() <= 510
    lens = np.array([1, 16, 17, 100])
    tab, n_pool = W.make_page_table(lens, 16, 3)
    used = tab[tab >= 0]
    assert len(used) == 1 + 1 + 2 + 7 and len(set(used.tolist())) == len(used) and used.max() < n_pool
