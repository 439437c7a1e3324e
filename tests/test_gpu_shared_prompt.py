"""Several responses per prompt sharing the prompt's full KV pages (rollout_submit_n): the HIP engine against the
CPU oracle, through the C ABI -- the scheduler bit for bit (page tables included), the model under teacher forcing."""
import numpy as np
import pytest

import workloads as W
from tests._util import flat_prompts, info_tuple, make_engine, make_oracle
from tests.test_gpu_rollout import _compare_stats, _harvest_both

pytestmark = pytest.mark.gpu

SHAPE = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)


def _prompts(n, lo, hi, vocab, seed):
    g = W.rng(seed)
    return [g.integers(0, vocab - 1, int(k)).astype(np.int32) for k in g.integers(lo, hi, n)]


@pytest.mark.parametrize("mode,stale,pool_pages", [(0, -1, 0), (0, -1, 24), (0, 1, 24), (1, -1, 0), (1, -1, 24), (2, -1, 0)])
def test_scheduler_bit_exact_with_shared_prompt_pages(mode, stale, pool_pages):
    import paper_2603_23414_amd as R
    n, k, Q, P, cap, G = 14, 4, 10, 70, 90, 6
    prompts = _prompts(n, 1, P + 1, 50, 31)
    L = W.make_target_lengths(n * k, 3.0, 0.9, cap, seed=32)
    kvb = pool_pages * SHAPE.n_layers * SHAPE.n_kv_heads * 2 * 16 * SHAPE.head_dim * 2
    kw = dict(max_slots=Q, max_prompt_len=P, cap=cap, kv_pool_bytes=kvb, mode=mode, max_staleness=stale, page_seed=5)
    orc = make_oracle(SHAPE, **kw)
    ctx = make_engine(SHAPE, None, max_seqs=n * k, debug_flags=R.ROLLOUT_DEBUG_NO_MODEL, **kw)
    try:
        toks, offs = flat_prompts(prompts)
        assert R.rollout_submit_n(ctx, toks, offs, L, k) == orc.submit(prompts, L, n_responses=k)
        harvested, shared_steps = 0, 0
        while orc.queue or any(x is not None for x in orc.slots):
            io = orc.step()
            ig = R.rollout_step(ctx)
            assert info_tuple(ig) == info_tuple(io), (info_tuple(ig), info_tuple(io))
            for slot in range(Q):                                    # every page table, shared prefix included
                s = orc.slots[slot]
                assert list(R.rollout_slot_pages(ctx, slot, 4096)) == (s.pages if s is not None else [])
            shared_steps += int(any(s is not None and s.group is not None and s.group.ref > 1 for s in orc.slots))
            if len(orc.finished) >= G:
                harvested += len(_harvest_both(R, ctx, orc, G)[0])
        harvested += len(_harvest_both(R, ctx, orc, G, flush=True)[0])
        assert harvested == n * k and shared_steps > 0
        _compare_stats(R, ctx, orc)
        if pool_pages and mode == 0 and stale < 0:
            assert orc.n_preempt > 0
        # the sequence and group tables are free again: the same load can be fed once more
        assert R.rollout_submit_n(ctx, toks, offs, L, k) == n * k
    finally:
        R.rollout_destroy(ctx)


@pytest.mark.parametrize("shape,stale", [("tiny", -1), ("gqa4", 1)])
def test_sampled_responses_on_shared_pages_teacher_forced(shape, stale):
    """Temperature sampling, k = 4 responses per prompt, prompts from 1 to 3 pages: the engine's logits for every
    (rollout, step) against the oracle, which reads the same shared pages; tokens, log-probs, stats."""
    import paper_2603_23414_amd as R
    m = W.CONFIGS["tiny"].model if shape == "tiny" else W.ModelShape(2, 256, 8, 2, 32, 512, 1000, 1e-5, 1e4, 0)
    blob = W.make_weights(m, 4)
    n, k, Q, P, cap, G, T = 5, 4, 6, 40, 14, 4, 0.9
    prompts = _prompts(n, 1, P + 1, m.vocab, 41)
    L = np.minimum(W.make_target_lengths(n * k, 2.0, 0.6, cap, seed=42), cap)
    kw = dict(max_slots=Q, max_prompt_len=P, cap=cap, max_staleness=stale, temperature=T, sample_seed=99)
    orc = make_oracle(m, weights_blob=blob, **kw)
    ctx = make_engine(m, blob, max_seqs=n * k, **kw)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit_n(ctx, toks, offs, L, k)
        orc.submit(prompts, L, n_responses=k)
        logits = np.zeros((Q, m.vocab), np.float32)
        worst, attached, harvested = 0.0, 0, []
        while orc.queue or any(x is not None for x in orc.slots):
            before = [s.gen_len for s in orc.seqs]
            io = orc.step()
            attached += sum(1 for s in orc.slots if s is not None and s.prefill_from > 0 and s.gen_len == 1)
            forced = np.full(Q, -1, np.int32)
            ran = {}
            for s in orc.seqs:
                if s.gen_len > before[s.seq_id]:
                    forced[s.last_slot] = s.tokens[-1]
                    ran[s.last_slot] = s
            ig = R.rollout_step_forced(ctx, forced, logits)
            assert info_tuple(ig) == info_tuple(io)
            for slot in ran:
                worst = max(worst, float(np.max(np.abs(logits[slot].astype(np.float64) - orc.last_logits[slot]))))
            if len(orc.finished) >= G:
                recs, tk, lp, flat = _harvest_both(R, ctx, orc, G)
                harvested += [(r, tk, lp, s) for r, s in zip(recs, flat)]
        recs, tk, lp, flat = _harvest_both(R, ctx, orc, G, flush=True)
        harvested += [(r, tk, lp, s) for r, s in zip(recs, flat)]
        assert len(harvested) == n * k and attached > 0
        assert worst < 2e-2, worst
        for r, tk, lp, s in harvested:
            assert list(tk[r.tok_off:r.tok_off + r.gen_len]) == s.tokens
            assert np.max(np.abs(lp[r.tok_off:r.tok_off + r.gen_len] - np.array(s.logp))) < 3e-2
        _compare_stats(R, ctx, orc)
        multi = [i for i in range(n) if len(prompts[i]) > 16]
        assert any(len({tuple(orc.seqs[i * k + r].tokens) for r in range(k)}) > 1 for i in multi)   # siblings differ
    finally:
        R.rollout_destroy(ctx)


def test_free_running_sampled_siblings_share_prefill_and_differ():
    """No teacher forcing: the engine samples by itself.  Every rollout is harvested once, siblings of a long prompt
    get different responses, and the prefill counter shows the shared part was computed once per attachment."""
    import paper_2603_23414_amd as R
    m = W.CONFIGS["tiny"].model
    blob = W.make_weights(m, 1)
    n, k, Q, P, cap = 3, 8, 24, 48, 10
    prompts = [W.rng(50 + i).integers(0, m.vocab - 1, P).astype(np.int32) for i in range(n)]
    L = np.full(n * k, cap, np.uint32)
    ctx = make_engine(m, blob, max_slots=Q, max_prompt_len=P, cap=cap, max_seqs=n * k, temperature=1.0, sample_seed=3)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit_n(ctx, toks, offs, L, k)
        for _ in range(cap):
            R.rollout_step(ctx)
        ng, recs, tk, lp = R.rollout_harvest(ctx, k, R.ROLLOUT_FLUSH)
        assert ng == n and sorted(r.seq_id for r in recs) == list(range(n * k))
        by_prompt = {}
        for r in recs:
            by_prompt.setdefault(r.seq_id // k, set()).add(tuple(tk[r.tok_off:r.tok_off + r.gen_len - 1]))
        assert all(len(v) > 1 for v in by_prompt.values())
        st = R.rollout_stats(ctx)
        # all 24 admitted in step 0: per prompt one full prefill (48) and 7 attachments of 48 - 2*16 = 16 tokens
        assert st.prefill_tokens == n * (P + (k - 1) * (P - 32))
        assert st.max_pages_used == n * (2 + k * 2)               # 2 shared + per rollout pages 2 and 3 (48 + 10 tokens)
    finally:
        R.rollout_destroy(ctx)


def test_submit_n_error_paths():
    import paper_2603_23414_amd as R
    ctx = make_engine(SHAPE, None, max_slots=2, max_prompt_len=8, cap=4, max_seqs=6, debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        p = np.arange(4, dtype=np.int32)
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit_n(ctx, p, [0, 4], np.zeros(0, np.uint32), 0)
        assert e.value.code == -1
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit_n(ctx, p, [0, 4], np.ones(7, np.uint32), 7)          # 7 > max_seqs
        assert e.value.code == -3
        with pytest.raises(R.RolloutError) as e:
            R.rollout_submit_n(ctx, p, [0, 4], np.array([1, 9], np.uint32), 2)     # target_len > cap
        assert e.value.code == -4
        assert R.rollout_submit_n(ctx, p, [0, 4], np.array([1, 2, 3], np.uint32), 3) == 0
    finally:
        R.rollout_destroy(ctx)
