"""End-to-end parity of the HIP rollout engine (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import workloads as W
from tests._util import LOGIT_REL_TOL, LogitError, flat_prompts, info_tuple, make_engine, make_oracle

pytestmark = pytest.mark.gpu


def _harvest_both(R, ctx, orc, G, flush=False):
    ng, recs, toks, logp = R.rollout_harvest(ctx, G, R.ROLLOUT_FLUSH if flush else 0)
    groups = orc.harvest(G, flush=flush)
    assert ng == len(groups)
    flat = [s for g in groups for s in g]
    assert len(recs) == len(flat)
    for r, s in zip(recs, flat):
        assert (r.seq_id, r.slot, r.completion_step, r.gen_len, r.group_idx, r.n_preempt, r.policy_version) == \
               (s.seq_id, s.last_slot, s.completion_step, s.gen_len, s.group_idx, s.n_preempt, s.policy_version)
    return recs, toks, logp, flat


def _compare_stats(R, ctx, orc):
    st, so = R.rollout_stats(ctx), orc.stats()
    for k in ("steps", "busy", "idle", "steps_q", "idle_q", "gen_tokens", "discarded_tokens", "prefill_tokens",
              "n_preempt", "n_stale", "version", "max_pages_used"):
        assert getattr(st, k) == so[k], k


def _scheduler_only(L, *, Q, P, cap, G, kv_pool_pages=0, max_staleness=-1, mode=0, page_seed=0, harvest_every=True):
    """NO_MODEL run of the device scheduler against the integer oracle, step by step."""
    import paper_2603_23414_amd as R
    shape = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    page_bytes = shape.n_layers * shape.n_kv_heads * 2 * 16 * shape.head_dim * 2
    kvb = kv_pool_pages * page_bytes
    n = len(L)
    prompts = [np.full(P, 1, np.int32) for _ in range(n)]
    orc = make_oracle(shape, max_slots=Q, max_prompt_len=P, cap=cap, kv_pool_bytes=kvb, mode=mode,
                      max_staleness=max_staleness, page_seed=page_seed)
    ctx = make_engine(shape, None, max_slots=Q, max_prompt_len=P, cap=cap, max_seqs=n, kv_pool_bytes=kvb, mode=mode,
                      max_staleness=max_staleness, page_seed=page_seed, debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        toks, offs = flat_prompts(prompts)
        assert R.rollout_submit(ctx, toks, offs, L) == orc.submit(prompts, L)
        harvested = 0
        while orc.queue or any(x is not None for x in orc.slots):
            before = [s.gen_len for s in orc.seqs]
            pf_before = orc.prefill_tokens
            io = orc.step()
            ig = R.rollout_step(ctx)
            assert info_tuple(ig) == info_tuple(io), (info_tuple(ig), info_tuple(io))
            assert ig.ctx_tokens == sum(len(s.prompt) + s.gen_len for s in orc.slots if s is not None)
            # the step's own work record: decode rows and the context they attended, prefilled positions and their
            # causal query-key pairs
            adm = {sid for sid, _ in io["admitted"]}
            ran = [s for s in orc.seqs if s.gen_len > before[s.seq_id]]
            dec = [s for s in ran if s.seq_id not in adm]
            pairs = 0
            for s in ran:
                if s.seq_id in adm:
                    n_tok, p0 = len(s.prompt) + s.gen_len - 1, s.prefill_from
                    pairs += (n_tok * (n_tok + 1) - p0 * (p0 + 1)) // 2
            assert (ig.n_decode_rows, ig.decode_ctx_tokens, ig.prefill_tokens, ig.prefill_ctx_pairs) == \
                   (len(dec), sum(len(s.prompt) + s.gen_len - 1 for s in dec), orc.prefill_tokens - pf_before, pairs)
            for slot in range(0, Q, max(1, Q // 4)):                  # sampled page tables
                s = orc.slots[slot]
                pages = R.rollout_slot_pages(ctx, slot, 4096)
                assert list(pages) == (s.pages if s is not None else [])
            if harvest_every and len(orc.finished) >= G:
                recs, *_ = _harvest_both(R, ctx, orc, G)
                harvested += len(recs)
        recs, tk, lp, flat = _harvest_both(R, ctx, orc, G, flush=True)
        harvested += len(recs)
        assert harvested == n
        for r, s in zip(recs, flat):
            assert list(tk[r.tok_off:r.tok_off + r.gen_len]) == s.tokens
        _compare_stats(R, ctx, orc)
        assert abs(R.rollout_stats(ctx).idle / (Q * R.rollout_stats(ctx).steps) - orc.bubble_ratio()) < 1e-15
    finally:
        R.rollout_destroy(ctx)


def test_scheduler_bit_exact_continuous_refill():
    L = W.make_target_lengths(96, 3.2, 0.8, 120, seed=21)
    _scheduler_only(L, Q=12, P=20, cap=120, G=8)


def test_scheduler_bit_exact_with_staleness_and_late_harvests():
    L = W.make_target_lengths(80, 3.5, 0.9, 200, seed=22)
    _scheduler_only(L, Q=16, P=7, cap=200, G=5, max_staleness=1)
    _scheduler_only(L, Q=16, P=7, cap=200, G=5, max_staleness=0, page_seed=99)


def test_scheduler_bit_exact_under_pool_exhaustion_and_preemption():
    L = W.make_target_lengths(40, 4.0, 0.7, 160, seed=23)
    # pages per max sequence = ceil((33 + 160) / 16) = 13; 30 pages for 8 slots forces preemption
    _scheduler_only(L, Q=8, P=33, cap=160, G=4, kv_pool_pages=30)


def test_scheduler_bit_exact_sync_baseline_and_on_policy_modes():
    L = W.make_target_lengths(48, 3.0, 0.8, 100, seed=24)
    _scheduler_only(L, Q=8, P=5, cap=100, G=8, mode=2)
    _scheduler_only(L, Q=8, P=5, cap=100, G=4, mode=1)


def test_scheduler_hand_built_preemption_case():
    # same case as tests/test_oracle_scheduler.py: needs 4-token pages there; with 16-token pages use P = 15
    _scheduler_only(np.array([40, 40, 40], np.int32), Q=3, P=15, cap=64, G=3, kv_pool_pages=5)


def _teacher_forced(m, blob, prompts, L, *, Q, cap, G, max_prompt_len=None, kv_pool_pages=0, max_staleness=-1,
                    abs_tol=None, seed_pages=0, swap_blob=None, w_std=0.02):
    """Run oracle (with the model) and engine in lockstep; the engine is fed the oracle's token at every step and
    its fp32 logits rows are compared.  The bar is the same on every shape: worst error below LOGIT_REL_TOL times
    the standard deviation of the oracle's logits (which is 2e-2 absolute on the 128-wide parity config; abs_tol
    additionally asserts an absolute bound).  Returns (worst |logit error|, rows compared, argmax agreement)."""
    import paper_2603_23414_amd as R
    P = max_prompt_len or max(len(p) for p in prompts)
    page_bytes = m.n_layers * m.n_kv_heads * 2 * 16 * m.head_dim * 2
    kvb = kv_pool_pages * page_bytes
    orc = make_oracle(m, max_slots=Q, max_prompt_len=P, cap=cap, kv_pool_bytes=kvb, max_staleness=max_staleness,
                      page_seed=seed_pages, weights_blob=blob)
    ctx = make_engine(m, blob, max_slots=Q, max_prompt_len=P, cap=cap, max_seqs=len(prompts), kv_pool_bytes=kvb,
                      max_staleness=max_staleness, page_seed=seed_pages)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        logits = np.zeros((Q, m.vocab), np.float32)
        err = LogitError(w_std * np.sqrt(m.d_model))
        agree, harvested = 0, []
        while orc.queue or any(x is not None for x in orc.slots):
            before = [s.gen_len for s in orc.seqs]
            io = orc.step()
            forced = np.full(Q, -1, np.int32)
            ran = {}
            for s in orc.seqs:                                   # every sequence that emitted a token this step
                if s.gen_len > before[s.seq_id]:
                    forced[s.last_slot] = s.tokens[-1]
                    ran[s.last_slot] = s
            logits[:] = np.nan
            ig = R.rollout_step_forced(ctx, forced, logits)
            assert info_tuple(ig) == info_tuple(io)
            assert len(ran) == io["r"]
            for slot, s in ran.items():
                ref = orc.last_logits[slot]
                err.add(logits[slot], ref)
                agree += int(np.argmax(logits[slot]) == int(np.argmax(ref)))
            if len(orc.finished) >= G:
                recs, tk, lp, flat = _harvest_both(R, ctx, orc, G)
                harvested += [(r, tk, lp, s) for r, s in zip(recs, flat)]
                if swap_blob is not None:                        # the trainer's update arrives at this boundary
                    from oracle import OracleModel
                    w2 = {k: W.bf16_bits_to_f32(v) for k, v in W.split_weights(swap_blob, m).items()}
                    orc.update_weights(OracleModel(m, w2, np.float64))
                    R.rollout_update_weights(ctx, swap_blob)
                    swap_blob = None
        recs, tk, lp, flat = _harvest_both(R, ctx, orc, G, flush=True)
        harvested += [(r, tk, lp, s) for r, s in zip(recs, flat)]
        assert len(harvested) == len(prompts)
        err.check(f"D={m.d_model} L={m.n_layers} V={m.vocab}", abs_tol)
        for r, tk, lp, s in harvested:
            assert list(tk[r.tok_off:r.tok_off + r.gen_len]) == s.tokens
            # |d log-prob| <= |d logit of the token| + |d log-sum-exp| <= twice the logits bar
            assert np.max(np.abs(lp[r.tok_off:r.tok_off + r.gen_len] - np.array(s.logp))) < 2 * LOGIT_REL_TOL * err.sigma
            assert np.all(lp[r.tok_off:r.tok_off + r.gen_len] <= 1e-6)
        _compare_stats(R, ctx, orc)
        return err.worst, err.rows, agree
    finally:
        R.rollout_destroy(ctx)


def test_tiny_policy_teacher_forced_logits_and_scheduler():
    """The parity gate: the 2-layer fp32-sized policy of the smallest config, every (sequence, step) logits row
    within 2e-2 of the oracle under teacher forcing, scheduler output identical."""
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, c.seed_weights)
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    L = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    worst, rows, agree = _teacher_forced(m, blob, prompts, L, Q=c.max_slots, cap=c.cap, G=c.harvest, abs_tol=2e-2)
    assert rows == int(L.sum())
    assert agree >= 0.98 * rows


@pytest.mark.parametrize("shape", [
    W.ModelShape(2, 256, 8, 2, 32, 512, 1000, 1e-5, 1e4, 0),      # GQA group 4, head_dim 32, vocab not a tile multiple
    W.ModelShape(1, 512, 4, 1, 128, 512, 512, 1e-5, 5e5, 0),      # group 4, head_dim 128
    W.ModelShape(1, 640, 5, 1, 128, 768, 640, 1e-6, 1e6, 1),      # group 5, QKV bias (the 32B family's traits)
])
def test_gqa_shapes_ragged_prompts_staleness_and_preemption(shape):
    """Multi-tile prefill (ragged prompts up to 150 tokens), re-prefill of prompt + generated tokens after staleness
    evictions and pool-exhaustion preemptions, all under teacher forcing."""
    g = W.rng(31)
    n = 14
    plen = g.integers(1, 150, n)
    prompts = [g.integers(0, shape.vocab - 1, int(k)).astype(np.int32) for k in plen]
    L = W.make_target_lengths(n, 3.0, 0.7, 60, seed=32)
    # 150 + 60 tokens -> 14 pages per maximum sequence; 40 pages for 5 slots forces preemption
    worst, rows, agree = _teacher_forced(shape, W.make_weights(shape, 33), prompts, L, Q=5, cap=60, G=3,
                                         max_prompt_len=150, kv_pool_pages=40, max_staleness=1, seed_pages=7)
    assert rows >= int(L.sum())
    assert agree >= 0.95 * rows


@pytest.mark.parametrize("stale", [-1, 0])
def test_weight_update_at_a_boundary(stale):
    """A new policy is installed after the first harvest: later logits must follow the new weights on top of the caches
    that survive (stale = -1: old-policy KV is kept; stale = 0: it is rebuilt by re-prefill under the new weights)."""
    c = W.CONFIGS["tiny"]
    m = c.model
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    L = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    worst, rows, agree = _teacher_forced(m, W.make_weights(m, 1), prompts, L, Q=5, cap=c.cap, G=2, max_staleness=stale,
                                         swap_blob=W.make_weights(m, 77))
    assert rows >= int(L.sum())


def test_prompt_longer_than_one_prefill_pass():
    """A 4500-token prompt spans two prefill passes and 141 query tiles; the logits after it must still match."""
    shape = W.ModelShape(1, 128, 4, 4, 32, 128, 256, 1e-5, 1e4, 0)
    g = W.rng(41)
    prompts = [g.integers(0, shape.vocab - 1, 4500).astype(np.int32), g.integers(0, shape.vocab - 1, 33).astype(np.int32)]
    worst, rows, agree = _teacher_forced(shape, W.make_weights(shape, 42), prompts, np.array([3, 2], np.uint32), Q=2,
                                         cap=4, G=2)
    assert rows == 5


def test_tiny_policy_free_running_is_deterministic_and_matches_schedule():
    import paper_2603_23414_amd as R
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, c.seed_weights)
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    L = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    runs = []
    for _ in range(2):
        ctx = make_engine(m, blob, max_slots=c.max_slots, max_prompt_len=c.prompt_len, cap=c.cap, max_seqs=c.n_prompts)
        try:
            toks, offs = flat_prompts(prompts)
            R.rollout_submit(ctx, toks, offs, L)
            out = []
            while True:
                i = R.rollout_step(ctx)
                if i.n_finished_unharvested >= c.harvest:
                    ng, recs, tk, lp = R.rollout_harvest(ctx, c.harvest)
                    out += [(r.seq_id, r.slot, r.completion_step, r.gen_len, tuple(tk[r.tok_off:r.tok_off + r.gen_len]))
                            for r in recs]
                if i.n_active == 0 and i.n_queued == 0:
                    break
            ng, recs, tk, lp = R.rollout_harvest(ctx, c.harvest, R.ROLLOUT_FLUSH)
            out += [(r.seq_id, r.slot, r.completion_step, r.gen_len, tuple(tk[r.tok_off:r.tok_off + r.gen_len]))
                    for r in recs]
            runs.append(out)
        finally:
            R.rollout_destroy(ctx)
    assert runs[0] == runs[1]
    assert sorted(r[0] for r in runs[0]) == list(range(c.n_prompts))
    assert [r[3] for r in sorted(runs[0])] == list(L)
    orc = make_oracle(m, max_slots=c.max_slots, max_prompt_len=c.prompt_len, cap=c.cap)
    orc.submit(prompts, L)
    ref = [(s.seq_id, s.last_slot, s.completion_step, s.gen_len) for g in orc.run_to_completion(c.harvest) for s in g]
    assert [r[:4] for r in runs[0]] == ref


def test_temperature_sampling_matches_the_oracle_sampler_on_the_engine_logits():
    """Free-running sampled rollout (T = 0.8).  The schedule is length-forced, so the integer oracle tells which
    sequence sits in which slot; the oracle's Gumbel-max sampler applied to the ENGINE's logits row must pick the
    engine's token (a different pick is accepted only when the two best perturbed scores are a rounding apart), and the
    recorded log-prob must be log softmax(logits / T) of that token."""
    import paper_2603_23414_amd as R
    from oracle import log_prob_at, perturbed_scores
    c = W.CONFIGS["tiny"]
    m = c.model
    T, seed = 0.8, 0xC0FFEE1234
    blob = W.make_weights(m, c.seed_weights)
    prompts = [W.make_prompts(1, c.prompt_len, m.vocab, 5)[0]] * 6          # six responses to one prompt
    L = W.make_target_lengths(6, c.len_mu, c.len_sigma, c.cap, 8)
    orc = make_oracle(m, max_slots=4, max_prompt_len=c.prompt_len, cap=c.cap)    # integer schedule only
    ctx = make_engine(m, blob, max_slots=4, max_prompt_len=c.prompt_len, cap=c.cap, max_seqs=6, temperature=T,
                      sample_seed=seed)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        logits = np.zeros((4, m.vocab), np.float32)
        none = np.full(4, -1, np.int32)
        checked = mismatched = 0
        final = {}
        while orc.queue or any(x is not None for x in orc.slots):
            before = [s.gen_len for s in orc.seqs]
            io = orc.step()
            ig = R.rollout_step_forced(ctx, none, logits)
            assert info_tuple(ig) == info_tuple(io)
            for s in orc.seqs:
                if s.gen_len > before[s.seq_id]:
                    t = before[s.seq_id]
                    tk, lp, state, slot = R.rollout_peek(ctx, s.seq_id, c.cap)
                    assert len(tk) == t + 1
                    final[s.seq_id] = tk.copy()
                    row = logits[s.last_slot].astype(np.float64)
                    if t + 1 == s.target_len:
                        assert tk[t] == m.vocab - 1
                        continue
                    sc = perturbed_scores(row, T, seed, s.seq_id, t)
                    checked += 1
                    if int(np.argmax(sc)) != int(tk[t]):
                        top2 = np.sort(sc)[-2:]
                        assert top2[1] - top2[0] < 1e-3 and sc[tk[t]] >= top2[0] - 1e-6
                        mismatched += 1
                    assert abs(lp[t] - log_prob_at(row, int(tk[t]), T)) < 2e-4
        assert checked > 50 and mismatched <= 1
        assert len({tuple(v[:3]) for v in final.values()}) > 1       # the six responses are not all alike
    finally:
        R.rollout_destroy(ctx)


def test_error_paths():
    import paper_2603_23414_amd as R
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, 1)
    ctx = make_engine(m, blob, max_slots=4, max_prompt_len=16, cap=32, max_seqs=4)
    try:
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit(ctx, np.arange(17, dtype=np.int32), [0, 17], [5])
        assert e.value.code == -4
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit(ctx, np.array([m.vocab], np.int32), [0, 1], [5])
        assert e.value.code == -4
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit(ctx, np.zeros(5, np.int32), [0, 1, 2, 3, 4, 5], [1] * 5)
        assert e.value.code == -3
        assert R.rollout_harvest(ctx, 2)[0] == 0
        R.rollout_submit(ctx, np.zeros(3, np.int32), [0, 3], [2])
        with pytest.raises(R.RolloutError) as e:                 # a forced token outside the vocabulary: refused whole
            R.rollout_step_forced(ctx, np.array([m.vocab, -1, -1, -1], np.int32), None)
        assert e.value.code == -4 and R.rollout_stats(ctx).steps == 0
        R.rollout_step(ctx)
        tk, lp, state, slot = R.rollout_peek(ctx, 0, 32)
        assert len(tk) == 1 and state == 1 and slot == 0
        R.rollout_step(ctx)
        ng, recs, tk, lp = R.rollout_harvest(ctx, 1)
        assert ng == 1 and recs[0].gen_len == 2 and tk[-1] == m.vocab - 1
    finally:
        R.rollout_destroy(ctx)
    with pytest.raises(R.RolloutError):
        make_engine(m, blob[:-5], max_slots=4, max_prompt_len=16, cap=32, max_seqs=4)
