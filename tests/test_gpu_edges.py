"""Edge cases of the HIP engine through the C ABI: degenerate sizes, natural EOS, the reload gate, the cap, 1024 slots."""
import numpy as np
import pytest

import workloads as W
from tests._util import LOGIT_REL_TOL, flat_prompts, info_tuple, make_engine, make_oracle

pytestmark = pytest.mark.gpu


def _lockstep(R, ctx, orc, G, Q, vocab, use_model):
    """Teacher-forced lockstep until drained; returns (harvested oracle seqs, engine records, tokens, worst error)."""
    logits = np.zeros((Q, vocab), np.float32)
    worst = 0.0
    recs_all, flat_all, tok_all = [], [], []
    while orc.queue or any(x is not None for x in orc.slots):
        before = [s.gen_len for s in orc.seqs]
        io = orc.step()
        forced = np.full(Q, -1, np.int32)
        ran = {}
        for s in orc.seqs:
            if s.gen_len > before[s.seq_id]:
                forced[s.last_slot] = s.tokens[-1]
                ran[s.last_slot] = s
        ig = R.rollout_step_forced(ctx, forced, logits if use_model else None)
        assert info_tuple(ig) == info_tuple(io), (info_tuple(ig), info_tuple(io))
        if use_model:
            for slot in ran:
                worst = max(worst, float(np.max(np.abs(logits[slot] - orc.last_logits[slot]))))
        if len(orc.finished) >= G:
            ng, recs, tk, lp = R.rollout_harvest(ctx, G)
            groups = orc.harvest(G)
            assert ng == len(groups)
            for r, s in zip(recs, [s for g in groups for s in g]):
                recs_all.append(r); flat_all.append(s); tok_all.append(tk[r.tok_off:r.tok_off + r.gen_len].copy())
    ng, recs, tk, lp = R.rollout_harvest(ctx, G, R.ROLLOUT_FLUSH)
    groups = orc.harvest(G, flush=True)
    for r, s in zip(recs, [s for g in groups for s in g]):
        recs_all.append(r); flat_all.append(s); tok_all.append(tk[r.tok_off:r.tok_off + r.gen_len].copy())
    return flat_all, recs_all, tok_all, worst


def test_natural_eos_and_cap_finish_rollouts():
    """eos_mode = NATURAL_OR_FORCED with a 64-token vocabulary (EOS shows up by chance), no target lengths on half of
    the prompts (they end on natural EOS or at the cap), under teacher forcing."""
    import paper_2603_23414_amd as R
    m = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    blob = W.make_weights(m, 5, std=0.1)        # 5x the usual weight scale: EOS wins the argmax now and then
    g = W.rng(4)
    prompts = [g.integers(0, m.vocab - 1, int(k)).astype(np.int32) for k in g.integers(1, 20, 12)]
    L = np.array([0, 7, 0, 0, 12, 0, 3, 0, 0, 1, 0, 0], np.uint32)
    orc = make_oracle(m, max_slots=4, max_prompt_len=20, cap=25, eos_mode=1, weights_blob=blob)
    ctx = make_engine(m, blob, max_slots=4, max_prompt_len=20, cap=25, max_seqs=12, eos_mode=1)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        flat, recs, tok, worst = _lockstep(R, ctx, orc, 3, 4, m.vocab, True)
        # the same relative bar as everywhere (LOGIT_REL_TOL of the logit standard deviation, here 0.1 * sqrt(64))
        sigma = 0.1 * np.sqrt(m.d_model)
        print(f"natural EOS: worst |logit error| {worst:.4f} = {worst / sigma:.4f} of the logit std {sigma:.2f}")
        assert len(flat) == 12 and worst < LOGIT_REL_TOL * sigma, worst
        natural = capped = 0
        for s, r, t in zip(flat, recs, tok):
            assert (r.seq_id, r.gen_len, r.completion_step, r.slot) == (s.seq_id, s.gen_len, s.completion_step, s.last_slot)
            assert list(t) == s.tokens
            if s.target_len == 0:
                natural += int(s.tokens[-1] == m.vocab - 1 and s.gen_len < 25)
                capped += int(s.gen_len == 25)
        assert natural + capped == 8 and natural >= 1
    finally:
        R.rollout_destroy(ctx)


def test_single_slot_single_token_and_empty_submit():
    import paper_2603_23414_amd as R
    m = W.CONFIGS["tiny"].model
    blob = W.make_weights(m, 1)
    ctx = make_engine(m, blob, max_slots=1, max_prompt_len=16, cap=4, max_seqs=3)
    orc = make_oracle(m, max_slots=1, max_prompt_len=16, cap=4, weights_blob=blob)
    try:
        assert R.rollout_submit(ctx, np.zeros(0, np.int32), [0], np.zeros(0, np.uint32)) == 0     # nothing to feed
        i = R.rollout_step(ctx)                                                              # a step with nothing to do
        assert (i.n_ran, i.n_active, i.n_queued) == (0, 0, 0)
        orc.step()
        prompts = [np.array([5], np.int32), np.arange(16, dtype=np.int32), np.array([7, 8], np.int32)]
        L = np.array([1, 4, 0], np.uint32)                      # one token; full length; no target -> cap of 4
        toks, offs = flat_prompts(prompts)
        assert R.rollout_submit(ctx, toks, offs, L) == 0
        orc.submit(prompts, L)
        flat, recs, tok, worst = _lockstep(R, ctx, orc, 1, 1, m.vocab, True)
        assert [r.gen_len for r in sorted(recs, key=lambda r: r.seq_id)] == [1, 4, 4]
        assert worst < 2e-2
        st = R.rollout_stats(ctx)
        assert st.steps == orc.step_no and st.idle == orc.idle and st.gen_tokens == 9
    finally:
        R.rollout_destroy(ctx)


def test_reload_gate_refuses_new_prompts_until_the_group_is_harvested():
    """Sec. 3.1 cache-aware loading: no new prompts until every loaded prompt has been fed to the trainer."""
    import paper_2603_23414_amd as R
    m = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    cfg = R.make_cfg(m, max_slots=2, max_prompt_len=4, max_new_tokens=8, max_seqs=8, grouped_loading=1,
                     debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    ctx = R.rollout_init(np.zeros(1, np.uint16), cfg)
    try:
        p = np.ones(12, np.int32)
        R.rollout_submit(ctx, p, [0, 4, 8, 12], [2, 3, 5])
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit(ctx, p[:4], [0, 4], [2])
        assert e.value.code == -3
        done = 0
        while done < 3:
            i = R.rollout_step(ctx)
            if i.n_finished_unharvested >= 1:
                done += len(R.rollout_harvest(ctx, 1)[1])
            if done < 3:
                with pytest.raises(R.RolloutError):
                    R.rollout_submit(ctx, p[:4], [0, 4], [2])
        assert R.rollout_submit(ctx, p[:4], [0, 4], [2]) == 3      # gate open again, ids continue
    finally:
        R.rollout_destroy(ctx)


def test_scheduler_with_1024_slots():
    import paper_2603_23414_amd as R
    m = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    n, Q = 3000, 1024
    L = W.make_target_lengths(n, 3.0, 1.0, 90, seed=55)
    prompts = [np.ones(3, np.int32)] * n
    orc = make_oracle(m, max_slots=Q, max_prompt_len=3, cap=90, max_staleness=2)
    ctx = make_engine(m, None, max_slots=Q, max_prompt_len=3, cap=90, max_seqs=n, max_staleness=2,
                      debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        flat, recs, tok, _ = _lockstep(R, ctx, orc, 128, Q, m.vocab, False)
        assert len(recs) == n
        assert [(r.seq_id, r.slot, r.completion_step, r.gen_len) for r in recs] == \
               [(s.seq_id, s.last_slot, s.completion_step, s.gen_len) for s in flat]
        st, so = R.rollout_stats(ctx), orc.stats()
        assert (st.steps, st.idle, st.n_stale, st.prefill_tokens) == (so["steps"], so["idle"], so["n_stale"], so["prefill_tokens"])
    finally:
        R.rollout_destroy(ctx)


@pytest.mark.parametrize("vocab,partner", [
    (4096, lambda v: v + 2048),       # duplicates 2048 columns apart: held by different threads and wavefronts of the arg-max
    (4096, lambda v: v + 1),          # adjacent duplicates (even, odd): the same 16-byte vector of one thread
    (4099, lambda v: v + 2048),       # a vocabulary that is not a multiple of 4 (scalar walk): same thread, later visit
])
def test_argmax_ties_take_the_lowest_index(vocab, partner):
    """An LM head with duplicated rows makes every maximum an exact tie (identical rows give bit-identical logits);
    greedy decoding must emit the lower index, on the engine's own logits and in agreement with the oracle, and a
    forced EOS still overrides."""
    import paper_2603_23414_amd as R
    from oracle import OracleModel, greedy_token
    m = W.ModelShape(1, 128, 4, 4, 32, 128, vocab, 1e-5, 1e4, 0)
    blob = W.make_weights(m, 61)
    lm = W.split_weights(blob, m)["lm_head"]                      # a view: edits land in the blob
    half = 2048
    lows = np.arange(half) if partner(0) == half else np.arange(0, 2 * half, 2)
    lm[[partner(int(v)) for v in lows]] = lm[lows]
    pair_of = {int(v): partner(int(v)) for v in lows}
    n, P, L = 24, 9, 3
    g = W.rng(62)
    prompts = [g.integers(0, vocab - 1, int(k)).astype(np.int32) for k in g.integers(1, P + 1, n)]
    ctx = make_engine(m, blob, max_slots=n, max_prompt_len=P, cap=L, max_seqs=n)
    model = OracleModel(m, {k: W.bf16_bits_to_f32(v) for k, v in W.split_weights(blob, m).items()}, np.float64)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, np.full(n, L, np.uint32))
        logits = np.zeros((n, vocab), np.float32)
        free = np.full(n, -1, np.int32)
        decided = 0
        for step in range(L):
            logits[:] = np.nan
            i = R.rollout_step_forced(ctx, free, logits)           # nothing forced: the engine's own choice
            assert i.n_ran == n
            for sid in range(n):                                   # all admitted at step 0 in order: slot == seq id
                tk, _, state, slot = R.rollout_peek(ctx, sid, L)
                assert len(tk) == step + 1 and (slot == sid or step == L - 1)
                row = logits[sid]
                if step == L - 1:
                    assert tk[-1] == vocab - 1                     # forced EOS whatever the logits say
                    continue
                tok = int(tk[-1])
                assert tok == int(np.argmax(row))                  # numpy's argmax returns the first maximum
                if tok in pair_of:                                 # (a column without a twin can win when vocab is odd-sized)
                    assert row[tok] == row[pair_of[tok]]           # the tie is real, and the lower index was emitted
                    decided += 1
                else:
                    assert tok not in pair_of.values()
                ref = model.full_recompute(list(prompts[sid]) + [int(t) for t in tk[:-1]])
                top = np.sort(np.unique(ref.astype(np.float32)))[-2:]
                if top[1] - top[0] > 4e-2:                         # unless two distinct values are a rounding apart
                    assert greedy_token(ref) == tok
        assert decided >= 2 * n - 4
    finally:
        R.rollout_destroy(ctx)


def test_harvest_larger_than_the_staging_buffers_goes_out_in_batches():
    """600 rollouts of 7000 tokens each (4.2 M tokens) harvested in one call: more than the library's packed staging
    buffers hold (2^22 elements), so the gather runs in several batches; every trajectory must land at its offset."""
    import paper_2603_23414_amd as R
    shape = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    n, Lg = 600, 7000
    ctx = make_engine(shape, None, max_slots=n, max_prompt_len=4, cap=Lg, max_seqs=n, debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        prompts = [np.full(3, 1, np.int32)] * n
        toks, offs = flat_prompts(prompts)
        L = (Lg - np.arange(n) % 7).astype(np.uint32)          # lengths 6994..7000
        R.rollout_submit(ctx, toks, offs, L)
        for _ in range(Lg):
            i = R.rollout_step(ctx)
        assert i.n_active == 0 and i.n_finished_unharvested == n
        ng, recs, tk, lp = R.rollout_harvest(ctx, n, R.ROLLOUT_FLUSH)
        assert ng == 1 and len(recs) == n and len(tk) == int(L.sum()) > 1 << 22
        off = 0
        for r in recs:
            assert r.tok_off == off and r.gen_len == L[r.seq_id]
            seg = tk[off:off + r.gen_len]
            assert seg[-1] == shape.vocab - 1 and not seg[:-1].any()        # scheduler-only tokens: zeros, then the forced EOS
            off += r.gen_len
        assert [r.gen_len for r in recs] == sorted(r.gen_len for r in recs)   # length-ordered
        assert not lp.any()
    finally:
        R.rollout_destroy(ctx)
