"""Pins for oracle/sampling.py."""
import numpy as np

from oracle import (OracleModel, OracleRollout, PagedKV, log_prob_at, perturbed_scores, philox4x32_10, sample_token,
                    softmax, uniforms)
import workloads as W


def test_philox4x32_10_known_answer_vectors():
    """The three known-answer vectors distributed with the reference implementation of Philox4x32-10."""
    cases = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
             ((0xffffffff,) * 4, (0xffffffff, 0xffffffff), (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
             ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
              (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in cases:
        got = philox4x32_10(*ctr, *key)
        assert tuple(int(x) for x in got) == want
    # vectorised over the first counter word
    v = philox4x32_10(np.arange(4), 0, 0, 0, 0, 0)
    assert int(v[0][0]) == 0x6627e8d5 and len(set(int(x) for x in v[0])) == 4


def test_uniforms_are_in_the_open_interval_and_look_uniform():
    u = uniforms(200_000, seed=7, seq_id=3, index=5)
    assert u.min() > 0 and u.max() < 1
    assert abs(u.mean() - 0.5) < 3e-3 and abs(u.var() - 1 / 12) < 2e-3
    assert not np.array_equal(u[:100], uniforms(100, 7, 3, 6)) and not np.array_equal(u[:100], uniforms(100, 7, 4, 5))
    assert np.array_equal(u[:100], uniforms(100, 7, 3, 5))


def test_gumbel_max_draws_follow_softmax_of_scaled_logits():
    logits = np.array([2.0, 1.0, 0.0, -1.0, 0.5, 1.5])
    for T in (0.7, 1.0, 2.0):
        n = 20_000
        counts = np.zeros(len(logits))
        for i in range(n):
            counts[sample_token(logits, T, seed=11, seq_id=i, index=0)] += 1
        p = softmax(logits / T)
        # binomial standard error sqrt(p(1-p)/n) <= 0.0025; allow 5 sigma
        assert np.all(np.abs(counts / n - p) < 5 * np.sqrt(p * (1 - p) / n) + 1e-4), (T, counts / n, p)


def test_low_temperature_approaches_greedy_and_logprob_is_log_softmax():
    g = np.random.default_rng(2)
    logits = g.standard_normal(300) * 3
    assert all(sample_token(logits, 1e-3, 5, s, 0) == int(np.argmax(logits)) for s in range(20))
    t = sample_token(logits, 0.9, 5, 1, 2)
    assert abs(np.exp(log_prob_at(logits, t, 0.9)) - softmax(logits / 0.9)[t]) < 1e-12
    sc = perturbed_scores(logits, 0.9, 5, 1, 2)
    assert sc.shape == (300,) and int(np.argmax(sc)) == t


def test_sampled_rollout_is_deterministic_and_uses_seq_id_and_index():
    m = W.ModelShape(1, 16, 2, 2, 8, 32, 12, 1e-5, 1e4, 0)
    g = np.random.default_rng(3)
    w = {n: g.standard_normal((r, c)) * 0.5 for n, r, c in W.weight_layout(m)}

    def run(seed):
        o = OracleRollout(max_slots=2, page_tokens=4, n_pages=16, max_new_tokens=8, eos_id=11, model=OracleModel(m, w),
                          kv_pool=PagedKV(1, 16, 4, 2, 8, np.float64), temperature=1.3, sample_seed=seed)
        o.submit([np.array([1, 2, 3], np.int32)] * 4, [6, 6, 6, 6])      # the same prompt four times
        o.run_to_completion(2)
        return [s.tokens for s in o.seqs], [s.logp for s in o.seqs]

    a, la = run(1)
    b, lb = run(1)
    c, _ = run(2)
    assert a == b and la == lb and a != c
    assert len({tuple(t) for t in a}) > 1            # k responses to one prompt differ through seq_id
    assert all(t[-1] == 11 for t in a) and all(x <= 1e-12 for l in la for x in l)
