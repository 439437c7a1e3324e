"""Helpers shared by the GPU parity tests: build the oracle and the HIP engine from the same seeded inputs."""
import math

import numpy as np

import workloads as W


def n_pages_for(shape, max_slots, max_prompt_len, cap, kv_pool_bytes=0, page_tokens=16):
    max_pages = (max_prompt_len + cap + page_tokens - 1) // page_tokens
    if kv_pool_bytes:
        return kv_pool_bytes // (shape.n_layers * shape.n_kv_heads * 2 * page_tokens * shape.head_dim * 2)
    return max_slots * max_pages


def make_oracle(shape, *, max_slots, max_prompt_len, cap, kv_pool_bytes=0, eos_mode=0, mode=0, max_staleness=-1,
                page_seed=0, weights_blob=None, dtype=np.float64, temperature=0.0, sample_seed=0):
    from oracle import OracleModel, OracleRollout, PagedKV
    n_pages = n_pages_for(shape, max_slots, max_prompt_len, cap, kv_pool_bytes)
    model = pool = None
    if weights_blob is not None:
        w = {k: W.bf16_bits_to_f32(v) for k, v in W.split_weights(weights_blob, shape).items()}
        model = OracleModel(shape, w, dtype)
        pool = PagedKV(shape.n_layers, n_pages, 16, shape.n_kv_heads, shape.head_dim, dtype)
    return OracleRollout(max_slots=max_slots, page_tokens=16, n_pages=n_pages, max_new_tokens=cap,
                         eos_id=shape.vocab - 1, eos_mode=eos_mode, mode=mode, max_staleness=max_staleness,
                         page_seed=page_seed, model=model, kv_pool=pool, temperature=temperature,
                         sample_seed=sample_seed)


def make_engine(shape, weights_blob, *, max_slots, max_prompt_len, cap, max_seqs, kv_pool_bytes=0, eos_mode=0,
                mode=0, max_staleness=-1, page_seed=0, debug_flags=0, temperature=0.0, sample_seed=0):
    import paper_2603_23414_amd as R
    cfg = R.make_cfg(shape, max_slots=max_slots, max_prompt_len=max_prompt_len, max_new_tokens=cap,
                     max_seqs=max_seqs, kv_pool_bytes=kv_pool_bytes, eos_mode=eos_mode, mode=mode,
                     max_staleness=max_staleness, page_seed=page_seed, debug_flags=debug_flags,
                     temperature=temperature, sample_seed=sample_seed)
    if weights_blob is None:
        weights_blob = np.zeros(1, np.uint16)
    return R.rollout_init(weights_blob, cfg)


def flat_prompts(prompts):
    offs = np.zeros(len(prompts) + 1, np.uint32)
    offs[1:] = np.cumsum([len(p) for p in prompts])
    return np.concatenate([np.asarray(p, np.int32) for p in prompts]), offs


def info_tuple(i):
    """Comparable view of a step record from either side."""
    if isinstance(i, dict):
        return (i["step"], i["r"], i["n_active"], i["n_finished_unharvested"], i["n_queued"], i["free_pages"],
                len(i["admitted"]), len(i["finished"]), len(i["preempted"]))
    return (i.step, i.n_ran, i.n_active, i.n_finished_unharvested, i.n_queued, i.free_pages, i.n_admitted,
            i.n_finished_step, i.n_preempted_step)


# the benchmark spec states the logits gate as max abs error 2e-2 on the 128-wide two-layer policy, whose logits have standard
# deviation 0.02 * sqrt(128) = 0.226 (unit-RMS final-norm output times N(0, 0.02) LM-head rows).  bf16 rounding of the
# GEMM inputs gives an error proportional to the logit scale, so the same bar on any other width or weight scale is
# this constant times the standard deviation of the oracle's logits.
LOGIT_REL_TOL = 2e-2 / (0.02 * math.sqrt(128.0))


class LogitError:
    """Accumulates max |engine - oracle| over logits rows together with the oracle logits' pooled standard deviation."""

    def __init__(self, design_sigma):
        self.design_sigma = float(design_sigma)    # weight std * sqrt(d_model): used when too few logits were seen
        self.worst = 0.0
        self.rows = 0
        self.n = 0
        self.s1 = 0.0
        self.s2 = 0.0

    def add(self, got, ref):
        ref = np.asarray(ref, np.float64)
        self.worst = max(self.worst, float(np.max(np.abs(np.asarray(got, np.float64) - ref))))
        self.rows += 1
        self.n += ref.size
        self.s1 += float(ref.sum())
        self.s2 += float((ref * ref).sum())

    @property
    def sigma(self):
        if self.n < 512:
            return self.design_sigma
        return math.sqrt(max(self.s2 / self.n - (self.s1 / self.n) ** 2, 0.0))

    @property
    def rel(self):
        return self.worst / self.sigma

    def check(self, label="", abs_tol=None):
        print(f"{label}: worst |logit error| {self.worst:.4f} = {self.rel:.4f} of the logit std {self.sigma:.3f} "
              f"over {self.rows} rows (bar {LOGIT_REL_TOL:.4f})")
        assert self.rel < LOGIT_REL_TOL, (self.worst, self.sigma, self.rel)
        if abs_tol is not None:
            assert self.worst < abs_tol, self.worst


def lockstep_teacher_forced(R, ctx, orc, Q, vocab, G, err, on_step=None):
    """Oracle and engine step together until drained; the engine is fed the oracle's token at every step and every
    logits row that ran is added to `err` (a LogitError).  Harvest records are compared whenever a group is ready.
    Returns the harvested (engine record, engine tokens, engine log-probs, oracle sequence) tuples."""
    logits = np.zeros((Q, vocab), np.float32)
    out = []

    def harvest(flush):
        ng, recs, tk, lp = R.rollout_harvest(ctx, G, R.ROLLOUT_FLUSH if flush else 0)
        groups = orc.harvest(G, flush=flush)
        flat = [s for g in groups for s in g]
        assert ng == len(groups) and len(recs) == len(flat)
        for r, s in zip(recs, flat):
            assert (r.seq_id, r.slot, r.completion_step, r.gen_len, r.group_idx, r.n_preempt, r.policy_version) == \
                   (s.seq_id, s.last_slot, s.completion_step, s.gen_len, s.group_idx, s.n_preempt, s.policy_version)
            out.append((r, tk[r.tok_off:r.tok_off + r.gen_len].copy(), lp[r.tok_off:r.tok_off + r.gen_len].copy(), s))

    while orc.queue or any(x is not None for x in orc.slots):
        before = [s.gen_len for s in orc.seqs]
        io = orc.step()
        forced = np.full(Q, -1, np.int32)
        ran = {}
        for s in orc.seqs:
            if s.gen_len > before[s.seq_id]:
                forced[s.last_slot] = s.tokens[-1]
                ran[s.last_slot] = s
        logits[:] = np.nan
        ig = R.rollout_step_forced(ctx, forced, logits)
        assert info_tuple(ig) == info_tuple(io), (info_tuple(ig), info_tuple(io))
        for slot in ran:
            err.add(logits[slot], orc.last_logits[slot])
        if on_step is not None:
            on_step(io, ig)
        if len(orc.finished) >= G:
            harvest(False)
    harvest(True)
    for r, tk, lp, s in out:
        assert list(tk) == s.tokens
    return out
