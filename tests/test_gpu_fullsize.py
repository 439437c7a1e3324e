"""Parity at the benchmark's full sizes: sampled outputs the oracle can compute one by one, the integer scheduler in
full, and teacher-forced logits on one-layer slices of the 8B and 32B widths."""
import numpy as np
import pytest

import workloads as W
from tests._util import LogitError, flat_prompts, lockstep_teacher_forced, make_engine, make_oracle

pytestmark = pytest.mark.gpu


def test_attention_case_full_size_sampled_rows():
    """The 256-sequence long-tail decode-attention case exactly as bench.py launches it; 10 sampled sequences
    (shortest, longest, and a seeded draw) are checked against the oracle."""
    import torch
    import paper_2603_23414_amd as R
    from oracle import gqa_attention
    a = W.ATTN_CASE
    Hq, Hkv, d, n = a["n_q_heads"], a["n_kv_heads"], a["head_dim"], a["n_seqs"]
    lens = W.make_kv_lengths(n, a["median"], a["sigma"], a["cap"], a["seed_lengths"])
    table, n_pool = W.make_page_table(lens, 16, a["seed_pages"])
    dev = torch.device("cuda:0")
    g = torch.Generator(device="cuda:0")
    g.manual_seed(a["seed_values"])
    pool = torch.empty(R.rollout_attn_pool_bytes(n_pool, Hkv, d) // 2, dtype=torch.bfloat16, device=dev)
    pool.normal_(0.0, 1.0, generator=g)
    q = torch.empty((n, Hq, d), dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g)
    tab = torch.from_numpy(np.maximum(table, 0).astype(np.int32)).to(dev)
    ws_bytes = R.rollout_attn_workspace_bytes(n, int(lens.sum()), Hq, d)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    n_work, chunk = R.rollout_attn_plan(lens, Hq, Hkv, d, ws.data_ptr(), ws_bytes)
    out = torch.empty((n, Hq, d), dtype=torch.float32, device=dev)
    R.rollout_attn_decode(pool.data_ptr(), Hq, Hkv, d, q.data_ptr(), tab.data_ptr(), table.shape[1], n, n_work,
                          chunk, out.data_ptr(), 1, ws.data_ptr())
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # decode the pool layout on the host for the sampled sequences: block (page, kvh) = K [d/8][16][8] then V [2][d][8]
    blk = 2 * 16 * d
    pick = sorted({int(np.argmin(lens)), int(np.argmax(lens)), *W.rng(77).integers(0, n, 8).tolist()})
    qh = q.float().cpu().numpy().astype(np.float64)
    for i in pick:
        L = int(lens[i])
        pages = table[i, : (L + 15) // 16]
        idx = torch.from_numpy(((pages[:, None, None].astype(np.int64) * Hkv + np.arange(Hkv)[None, :, None]) * blk
                                + np.arange(blk)[None, None, :])).to(dev)
        raw = pool[idx].float().cpu().numpy().astype(np.float64)           # [pages, Hkv, blk]
        K = raw[:, :, : 16 * d].reshape(len(pages), Hkv, d // 8, 16, 8).transpose(0, 3, 1, 2, 4).reshape(-1, Hkv, d)[:L]
        V = raw[:, :, 16 * d:].reshape(len(pages), Hkv, 2, d, 8).transpose(0, 2, 4, 1, 3).reshape(-1, Hkv, d)[:L]
        ref = gqa_attention(qh[i], K, V)
        assert np.abs(got[i] - ref).max() < 2e-2, (i, L)


@pytest.mark.parametrize("name", ["8b", "8b_long", "32b"])
def test_scheduler_bit_exact_at_full_scale(name):
    """The device scheduler alone (no model) over the whole workload against the integer oracle: per-step counters on
    a sampled stride, every harvest record, and the final statistics."""
    import paper_2603_23414_amd as R
    c = W.CONFIGS[name]
    L = W.make_target_lengths(c.n_prompts, c.len_mu, c.len_sigma, c.cap, c.seed_lengths)
    shape = W.ModelShape(1, 64, 2, 2, 32, 64, 64, 1e-5, 1e4, 0)
    page_bytes = 1 * 2 * 2 * 16 * 32 * 2
    real_page_bytes = c.model.n_layers * c.model.n_kv_heads * 2 * 16 * c.model.head_dim * 2
    kvb = (c.kv_pool_bytes // real_page_bytes) * page_bytes if c.kv_pool_bytes else 0
    prompts = [np.zeros(c.prompt_len, np.int32)] * c.n_prompts
    orc = make_oracle(shape, max_slots=c.max_slots, max_prompt_len=c.prompt_len, cap=c.cap, kv_pool_bytes=kvb,
                      max_staleness=c.max_staleness)
    ctx = make_engine(shape, None, max_slots=c.max_slots, max_prompt_len=c.prompt_len, cap=c.cap, max_seqs=c.n_prompts,
                      kv_pool_bytes=kvb, max_staleness=c.max_staleness, debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        got, ref = [], []
        while orc.queue or any(x is not None for x in orc.slots):
            io = orc.step()
            ig = R.rollout_step(ctx)
            if io["step"] % 97 == 0 or io["finished"] or io["admitted"]:
                assert (ig.step, ig.n_ran, ig.n_active, ig.n_finished_unharvested, ig.n_queued, ig.free_pages,
                        ig.n_admitted, ig.n_finished_step) == \
                       (io["step"], io["r"], io["n_active"], io["n_finished_unharvested"], io["n_queued"],
                        io["free_pages"], len(io["admitted"]), len(io["finished"]))
            if len(orc.finished) >= c.harvest:
                ng, recs, tk, lp = R.rollout_harvest(ctx, c.harvest, 0, want_logp=False)
                got += [(r.seq_id, r.slot, r.completion_step, r.gen_len, r.group_idx, r.policy_version) for r in recs]
                ref += [(s.seq_id, s.last_slot, s.completion_step, s.gen_len, s.group_idx, s.policy_version)
                        for g in orc.harvest(c.harvest) for s in g]
        ng, recs, tk, lp = R.rollout_harvest(ctx, c.harvest, R.ROLLOUT_FLUSH, want_logp=False)
        got += [(r.seq_id, r.slot, r.completion_step, r.gen_len, r.group_idx, r.policy_version) for r in recs]
        ref += [(s.seq_id, s.last_slot, s.completion_step, s.gen_len, s.group_idx, s.policy_version)
                for g in orc.harvest(c.harvest, flush=True) for s in g]
        assert got == ref and len(got) == c.n_prompts
        st, so = R.rollout_stats(ctx), orc.stats()
        for k in ("steps", "busy", "idle", "steps_q", "idle_q", "gen_tokens", "prefill_tokens", "n_preempt", "n_stale",
                  "version", "max_pages_used"):
            assert getattr(st, k) == so[k], k
    finally:
        R.rollout_destroy(ctx)


@pytest.mark.parametrize("name,layers", [("8b", 1), ("32b", 1), ("8b", 2), ("32b", 2), ("8b", 4)])
def test_slices_at_full_widths_teacher_forced(name, layers):
    """One, two and four layers of the real widths (d_model, heads, FFN, full vocabulary): a few rollouts with 17-70 token
    prompts under teacher forcing.  The bar is the one of the 128-wide parity gate carried over by the logit scale
    (LOGIT_REL_TOL of the oracle logits' standard deviation); the absolute and the relative error are printed per
    depth."""
    import paper_2603_23414_amd as R
    m = W.CONFIGS[name].model.with_layers(layers)
    blob = W.make_weights(m, 5)
    g = W.rng(6)
    prompts = [g.integers(0, m.vocab - 1, int(k)).astype(np.int32) for k in ((40, 70, 17) if layers == 1 else (21, 9))]
    L = np.array([3, 2, 4] if layers == 1 else [2, 3], np.uint32)
    orc = make_oracle(m, max_slots=2, max_prompt_len=70, cap=8, weights_blob=blob, dtype=np.float32)
    ctx = make_engine(m, blob, max_slots=2, max_prompt_len=70, cap=8, max_seqs=len(prompts))
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        err = LogitError(0.02 * np.sqrt(m.d_model))
        lockstep_teacher_forced(R, ctx, orc, 2, m.vocab, 2, err)
        assert err.rows == int(L.sum())
        err.check(f"{name} widths, {layers} layer(s)")
    finally:
        R.rollout_destroy(ctx)
