"""Stored expected values (tests/golden/*.json, written by tests/golden/make_golden.py from the oracle alone):
the oracle must keep reproducing them, they must satisfy what the method fixes independently of any implementation,
and the HIP engine must match them through the C ABI."""
import json
import os

import numpy as np
import pytest

import workloads as W
from tests._util import flat_prompts, make_engine

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
SCHEDULES = ["schedule_partial_refill", "schedule_stale_preempt", "schedule_on_policy", "schedule_sync_baseline",
             "schedule_shared_prompt"]
SHAPE = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)


def _load(name):
    with open(os.path.join(GOLDEN, name + ".json")) as f:
        return json.load(f)


@pytest.mark.parametrize("name", SCHEDULES + ["tiny_model_rollout"])
def test_oracle_still_reproduces_the_stored_values(name):
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(GOLDEN, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    stored = _load(name)
    if name == "tiny_model_rollout":
        fresh, _ = mg.model_fixture()
    else:
        c = stored["config"]
        fresh, _ = mg.schedule_fixture(name, Q=c["max_slots"], n=c["n_prompts"], P=c["prompt_len"], cap=c["cap"],
                                       G=c["harvest"], pool_pages=c["pool_pages"], stale=c["max_staleness"],
                                       mode=c["mode"], len_mu=c["len_mu"], len_sigma=c["len_sigma"], seed=c["seed"],
                                       k=c["responses_per_prompt"])
    assert json.loads(json.dumps(fresh)) == stored


@pytest.mark.parametrize("name", SCHEDULES)
def test_stored_schedules_satisfy_what_the_method_fixes(name):
    """Checked on the stored numbers alone: exactly-once harvest, groups in (completion step, length, id) order and of
    the harvest size, eq. 4 from the counters, one emitted token per busy slot-step, and for the synchronous
    baseline the closed form 1 - sum L / (Q * sum over batches of the longest length)."""
    d = _load(name)
    c, L, st = d["config"], d["target_len"], d["stats"]
    n = c["n_prompts"] * c["responses_per_prompt"]
    flat = [i for g in d["groups"] for i in g]
    assert sorted(flat) == list(range(n))
    assert all(len(g) == c["harvest"] for g in d["groups"][:-1]) and 1 <= len(d["groups"][-1]) <= c["harvest"]
    keys = [(d["completion_step"][i], L[i], i) for i in flat]
    if c["mode"] != 2 and c["max_staleness"] < 0 and c["mode"] != 1:
        assert keys == sorted(keys)                       # total order when nothing is evicted between harvests
    for g in d["groups"]:
        k = [(d["completion_step"][i], L[i], i) for i in g]
        assert k == sorted(k)
    assert st["busy"] + st["idle"] == c["max_slots"] * st["steps"]
    assert d["bubble_ratio"] == st["idle"] / (c["max_slots"] * st["steps"])
    assert st["gen_tokens"] == st["busy"] == sum(L) + st["discarded_tokens"]
    assert all(0 <= s < c["max_slots"] for s in d["last_slot"])
    if c["mode"] == 2:
        Q = c["max_slots"]
        steps = sum(max(L[b:b + Q]) for b in range(0, n, Q))
        assert st["steps"] == steps and abs(d["bubble_ratio"] - (1 - sum(L) / (Q * steps))) < 1e-15
    if c["max_staleness"] < 0 and c["mode"] == 0 and st["n_preempt"] == 0:
        assert st["prefill_tokens"] == n * c["prompt_len"]   # every prompt prefilled exactly once


@pytest.mark.gpu
@pytest.mark.parametrize("name", SCHEDULES)
def test_engine_reproduces_the_stored_schedules(name):
    import paper_2603_23414_amd as R
    d = _load(name)
    c = d["config"]
    k, n = c["responses_per_prompt"], c["n_prompts"]
    page_bytes = SHAPE.n_layers * SHAPE.n_kv_heads * 2 * 16 * SHAPE.head_dim * 2
    ctx = make_engine(SHAPE, None, max_slots=c["max_slots"], max_prompt_len=c["prompt_len"], cap=c["cap"],
                      max_seqs=n * k, kv_pool_bytes=c["pool_pages"] * page_bytes, mode=c["mode"],
                      max_staleness=c["max_staleness"], page_seed=c["seed"], debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        toks, offs = flat_prompts([np.zeros(c["prompt_len"], np.int32)] * n)
        R.rollout_submit_n(ctx, toks, offs, np.array(d["target_len"], np.uint32), k)
        recs = []
        while True:
            i = R.rollout_step(ctx)
            if i.n_finished_unharvested >= c["harvest"]:
                recs += R.rollout_harvest(ctx, c["harvest"])[1]
            if i.n_active == 0 and i.n_queued == 0:
                break
        recs += R.rollout_harvest(ctx, c["harvest"], R.ROLLOUT_FLUSH)[1]
        groups = {}
        for r in recs:
            groups.setdefault(r.group_idx, []).append(int(r.seq_id))
        assert [groups[g] for g in sorted(groups)] == d["groups"]
        by_id = {int(r.seq_id): r for r in recs}
        assert [by_id[i].completion_step for i in range(n * k)] == d["completion_step"]
        assert [by_id[i].slot for i in range(n * k)] == d["last_slot"]
        assert [by_id[i].n_preempt for i in range(n * k)] == d["n_preempt"]
        st = R.rollout_stats(ctx)
        for key, v in d["stats"].items():
            assert getattr(st, key) == v, key
    finally:
        R.rollout_destroy(ctx)


@pytest.mark.gpu
def test_engine_matches_the_stored_tiny_rollout_under_teacher_forcing():
    import paper_2603_23414_amd as R
    d = _load("tiny_model_rollout")
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, c.seed_weights)
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    ctx = make_engine(m, blob, max_slots=c.max_slots, max_prompt_len=c.prompt_len, cap=c.cap, max_seqs=c.n_prompts)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, np.full(c.n_prompts, 6, np.uint32))
        logits = np.zeros((c.max_slots, m.vocab), np.float32)
        for t in range(6):                                   # all 8 prompts fit the 8 slots: slot i = prompt i
            forced = np.array([d["tokens"][i][t] for i in range(c.n_prompts)], np.int32)
            R.rollout_step_forced(ctx, forced, logits)
            if t == 0:
                for slot, ref in d["first_step_logits_0_8"].items():
                    assert np.max(np.abs(logits[int(slot), :8] - np.array(ref))) < 2e-2
        ng, recs, tk, lp = R.rollout_harvest(ctx, c.harvest, R.ROLLOUT_FLUSH)
        assert len(recs) == c.n_prompts
        for r in recs:
            assert list(tk[r.tok_off:r.tok_off + 6]) == d["tokens"][r.seq_id]
            assert np.max(np.abs(lp[r.tok_off:r.tok_off + 6] - np.array(d["logp"][r.seq_id]))) < 3e-2
    finally:
        R.rollout_destroy(ctx)
