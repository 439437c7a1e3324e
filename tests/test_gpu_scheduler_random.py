"""Randomised sweep of the device scheduler against the integer oracle (no forward pass: ROLLOUT_DEBUG_NO_MODEL).

Every case draws its own slot count, prompt and target lengths, responses per prompt, pool size (ample or tight enough
to force preemption), operating mode, staleness bound, harvest group size and harvest timing, and feeds the prompts
in up to three batches at different steps.  Step records, every page table, harvest order, trajectories and counters
must agree bit for bit."""
import numpy as np
import pytest

import workloads as W
from tests._util import flat_prompts, info_tuple, make_engine, make_oracle
from tests.test_gpu_rollout import _compare_stats, _harvest_both

SHAPE = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
PAGE_BYTES = SHAPE.n_layers * SHAPE.n_kv_heads * 2 * 16 * SHAPE.head_dim * 2


def draw_case(seed):
    """Plain-Python description of one case (shared by the CPU self-check below and the GPU test)."""
    g = W.rng(1000 + seed)
    Q = int(g.integers(1, 25))
    P = int(g.integers(1, 81))
    cap = int(g.integers(1, 121))
    k = int(g.choice([1, 1, 2, 3, 5]))
    n = int(g.integers(1, 41 if k == 1 else 13))
    mode = int(g.choice([0, 0, 0, 1, 2]))
    stale = int(g.choice([-1, -1, 0, 1, 2])) if mode == 0 else -1
    G = int(g.integers(1, Q + 4))
    max_pages = (P + cap + 15) // 16
    pool_pages = 0 if g.random() < 0.35 else int(max_pages + g.integers(0, max(1, Q * max_pages // 5)))
    prompts = [g.integers(0, 50, int(m)).astype(np.int32) for m in g.integers(1, P + 1, n)]
    if g.random() < 0.5:
        L = np.minimum(cap, np.maximum(1, np.ceil(g.lognormal(np.log(max(2, cap // 3)), 0.9, n * k)))).astype(np.int32)
    else:
        L = g.integers(1, cap + 1, n * k).astype(np.int32)
    n_batches = int(g.integers(1, 4))
    cuts = sorted(set([0, n] + [int(c) for c in g.integers(0, n + 1, n_batches - 1)]))
    batches = [(cuts[i], cuts[i + 1]) for i in range(len(cuts) - 1) if cuts[i + 1] > cuts[i]]
    submit_at = [0] + sorted(int(s) for s in g.integers(1, 60, len(batches) - 1))
    p_harvest = float(g.choice([1.0, 1.0, 0.5, 0.1]))
    return dict(Q=Q, P=P, cap=cap, k=k, n=n, mode=mode, stale=stale, G=G, pool_pages=pool_pages, prompts=prompts, L=L,
                batches=batches, submit_at=submit_at, p_harvest=p_harvest, page_seed=seed, harvest_seed=5000 + seed)


def oracle_for(c):
    return make_oracle(SHAPE, max_slots=c["Q"], max_prompt_len=c["P"], cap=c["cap"], kv_pool_bytes=c["pool_pages"] * PAGE_BYTES,
                       mode=c["mode"], max_staleness=c["stale"], page_seed=c["page_seed"])


def drive(c, orc, eng=None):
    """Run one case on the oracle and, when an engine is given, on the engine in lockstep with every comparison."""
    R = eng[0] if eng else None
    ctx = eng[1] if eng else None
    k, L = c["k"], c["L"]
    gh = W.rng(c["harvest_seed"])
    pending = list(zip(c["submit_at"], c["batches"]))
    harvested = 0
    while pending or orc.queue or any(x is not None for x in orc.slots):
        while pending and (pending[0][0] <= orc.step_no or not (orc.queue or any(x is not None for x in orc.slots))):
            _, (a, b) = pending.pop(0)
            first = orc.submit(c["prompts"][a:b], L[a * k:b * k], n_responses=k)
            if eng:
                toks, offs = flat_prompts(c["prompts"][a:b])
                assert R.rollout_submit_n(ctx, toks, offs, L[a * k:b * k], k) == first
        io = orc.step()
        assert orc.step_no < 50000
        if eng:
            ig = R.rollout_step(ctx)
            assert info_tuple(ig) == info_tuple(io), (info_tuple(ig), info_tuple(io))
            assert ig.ctx_tokens == sum(len(s.prompt) + s.gen_len for s in orc.slots if s is not None)
            for slot in range(c["Q"]):
                s = orc.slots[slot]
                assert list(R.rollout_slot_pages(ctx, slot, 4096)) == (s.pages if s is not None else [])
        if len(orc.finished) >= c["G"] and gh.random() < c["p_harvest"]:
            if eng:
                recs, tk, _, flat = _harvest_both(R, ctx, orc, c["G"])
                for r, s in zip(recs, flat):
                    assert list(tk[r.tok_off:r.tok_off + r.gen_len]) == s.tokens
                harvested += len(recs)
            else:
                harvested += sum(len(x) for x in orc.harvest(c["G"]))
    while True:      # late harvests leave several groups; a flush takes them all, then the remainder
        if eng:
            recs, tk, _, flat = _harvest_both(R, ctx, orc, c["G"], flush=True)
            for r, s in zip(recs, flat):
                assert list(tk[r.tok_off:r.tok_off + r.gen_len]) == s.tokens
            got = len(recs)
        else:
            got = sum(len(x) for x in orc.harvest(c["G"], flush=True))
        harvested += got
        if got == 0 or harvested == c["n"] * k:
            break
        # on-policy and staleness boundaries can put rollouts back in the queue: keep stepping
        while orc.queue or any(x is not None for x in orc.slots):
            io = orc.step()
            assert orc.step_no < 50000
            if eng:
                assert info_tuple(R.rollout_step(ctx)) == info_tuple(io)
    assert harvested == c["n"] * k, (harvested, c["n"] * k)
    if eng:
        _compare_stats(R, ctx, orc)


@pytest.mark.parametrize("seed", range(48))
def test_cases_are_well_formed_and_terminate_on_the_oracle(seed):
    c = draw_case(seed)
    drive(c, oracle_for(c))


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(160))
def test_random_case_bit_exact(seed):
    import paper_2603_23414_amd as R
    c = draw_case(seed)
    orc = oracle_for(c)
    ctx = make_engine(SHAPE, None, max_slots=c["Q"], max_prompt_len=c["P"], cap=c["cap"], max_seqs=c["n"] * c["k"],
                      kv_pool_bytes=c["pool_pages"] * PAGE_BYTES, mode=c["mode"], max_staleness=c["stale"],
                      page_seed=c["page_seed"], debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        drive(c, orc, (R, ctx))
    finally:
        R.rollout_destroy(ctx)


@pytest.mark.gpu
def test_two_engines_side_by_side_do_not_disturb_each_other():
    """Two contexts with different shapes of work and operating modes, stepped alternately: each still
    agrees with its own oracle, so the library keeps no state outside its contexts."""
    import paper_2603_23414_amd as R
    ca, cb = draw_case(3), draw_case(11)
    oa, ob = oracle_for(ca), oracle_for(cb)

    def mk(c):
        return make_engine(SHAPE, None, max_slots=c["Q"], max_prompt_len=c["P"], cap=c["cap"], max_seqs=c["n"] * c["k"],
                           kv_pool_bytes=c["pool_pages"] * PAGE_BYTES, mode=c["mode"], max_staleness=c["stale"],
                           page_seed=c["page_seed"], debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)

    xa, xb = mk(ca), mk(cb)
    try:
        for c, o, x in ((ca, oa, xa), (cb, ob, xb)):
            toks, offs = flat_prompts(c["prompts"])
            assert R.rollout_submit_n(x, toks, offs, c["L"], c["k"]) == o.submit(c["prompts"], c["L"], n_responses=c["k"])
        live = [(ca, oa, xa), (cb, ob, xb)]
        while live:
            for c, o, x in list(live):
                if not (o.queue or any(s is not None for s in o.slots)):
                    live.remove((c, o, x))
                    continue
                assert info_tuple(R.rollout_step(x)) == info_tuple(o.step())
                if len(o.finished) >= c["G"]:
                    _harvest_both(R, x, o, c["G"])
        for c, o, x in ((ca, oa, xa), (cb, ob, xb)):
            while o.finished or o.queue or any(s is not None for s in o.slots):
                if o.queue or any(s is not None for s in o.slots):
                    assert info_tuple(R.rollout_step(x)) == info_tuple(o.step())
                else:
                    _harvest_both(R, x, o, c["G"], flush=True)
            _compare_stats(R, x, o)
    finally:
        R.rollout_destroy(xa)
        R.rollout_destroy(xb)
