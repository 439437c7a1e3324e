"""rollout_step takes the arg-max / Gumbel-max draw, the EOS logit and the log-sum-exp in the LM head's epilogue and never
writes a logits row; rollout_step_forced keeps the fp32 logits (teacher forcing reads them).  Both must emit the same
tokens, and the same log-probs up to the order of the fp32 sums, and the fused path must agree with the oracle."""
import numpy as np
import pytest

import workloads as W
from tests._util import flat_prompts, make_engine

pytestmark = pytest.mark.gpu


def _run(R, m, blob, prompts, L, *, Q, P, cap, fused, **kw):
    """Free-running rollout to completion; returns {seq_id: (tokens, log-probs, completion_step, slot)}."""
    ctx = make_engine(m, blob, max_slots=Q, max_prompt_len=P, cap=cap, max_seqs=len(prompts), **kw)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        free = np.full(Q, -1, np.int32)
        out = {}
        while True:
            i = R.rollout_step(ctx) if fused else R.rollout_step_forced(ctx, free, None)
            if i.n_finished_unharvested:
                ng, recs, tk, lp = R.rollout_harvest(ctx, 1)
                for r in recs:
                    out[int(r.seq_id)] = (tk[r.tok_off:r.tok_off + r.gen_len].copy(), lp[r.tok_off:r.tok_off + r.gen_len].copy(),
                                          r.completion_step, r.slot)
            if i.n_active == 0 and i.n_queued == 0:
                return out
    finally:
        R.rollout_destroy(ctx)


def _dup_lm_head(blob, m, dist):
    lm = W.split_weights(blob, m)["lm_head"]
    half = (m.vocab // 2) if dist == "far" else None
    if dist == "far":
        lm[half:2 * half] = lm[:half]
    else:
        lm[1:2 * (m.vocab // 2):2] = lm[0:2 * (m.vocab // 2):2]


@pytest.mark.parametrize("Q,vocab,temp,dup,eos_mode", [
    (5, 512, 0.0, None, 0),        # one 32-row block
    (40, 1000, 0.0, None, 0),      # two row blocks, vocabulary not a multiple of the 128-column tile
    (100, 4096, 0.0, "far", 0),    # four row blocks, every maximum an exact tie 2048 columns apart (different workgroups)
    (200, 4096, 0.0, "near", 1),   # eight row blocks, ties between neighbouring columns (same lane), natural EOS
    (24, 1000, 0.9, None, 0),      # sampling
    (150, 2000, 1.3, "far", 1),    # sampling, eight row blocks, duplicated rows (equal logits, different Gumbel noise)
    (300, 640, 0.0, None, 0),      # more than 256 rows: two row blocks of workgroups
])
def test_fused_statistics_equal_the_logits_path(Q, vocab, temp, dup, eos_mode):
    import paper_2603_23414_amd as R
    m = W.ModelShape(1, 128, 4, 4, 32, 128, vocab, 1e-5, 1e4, 0)
    blob = W.make_weights(m, 71, std=0.05)
    if dup:
        _dup_lm_head(blob, m, dup)
    g = W.rng(72)
    n = Q + 7
    prompts = [g.integers(0, vocab - 1, int(k)).astype(np.int32) for k in g.integers(1, 12, n)]
    L = g.integers(1, 6, n).astype(np.uint32)
    L[::5] = 0                                               # some rollouts end at the cap (or on a natural EOS)
    kw = dict(Q=Q, P=12, cap=5, temperature=temp, sample_seed=5, eos_mode=eos_mode)
    a = _run(R, m, blob, prompts, L, fused=True, **kw)
    b = _run(R, m, blob, prompts, L, fused=False, **kw)
    assert sorted(a) == sorted(b) == list(range(n))
    for sid in a:
        assert list(a[sid][0]) == list(b[sid][0]), sid
        assert a[sid][2:] == b[sid][2:]
        assert np.max(np.abs(a[sid][1] - b[sid][1])) < 2e-5
    if dup == "far" and temp == 0.0:                         # the lower twin wins every tie
        assert all(t < vocab // 2 for sid in a for t in a[sid][0][:-1])
    if dup == "near" and temp == 0.0:
        assert all(t % 2 == 0 or t == vocab - 1 for sid in a for t in a[sid][0])


def test_fused_path_matches_the_oracle_free_running():
    """Greedy free-running rollouts of the tiny policy through rollout_step: every emitted token equals the oracle's
    choice on the same prefix unless the oracle's two best logits are a rounding apart, and log-probs agree."""
    import paper_2603_23414_amd as R
    from oracle import OracleModel, greedy_token, log_prob
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, c.seed_weights)
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    L = np.minimum(W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths), 10).astype(np.uint32)
    got = _run(R, m, blob, prompts, L, Q=c.max_slots, P=c.prompt_len, cap=c.cap, fused=True)
    model = OracleModel(m, {k: W.bf16_bits_to_f32(v) for k, v in W.split_weights(blob, m).items()}, np.float64)
    checked = 0
    for sid, (tk, lp, _, _) in got.items():
        assert len(tk) == L[sid] and tk[-1] == m.vocab - 1
        for t in range(len(tk)):
            ref = model.full_recompute(list(prompts[sid]) + [int(x) for x in tk[:t]])
            assert abs(lp[t] - log_prob(ref, int(tk[t]))) < 4e-2        # twice the logits bar
            if t < len(tk) - 1:
                top = np.sort(ref)[-2:]
                if top[1] - top[0] > 4e-2:
                    assert greedy_token(ref) == int(tk[t])
                    checked += 1
    assert checked > 20
