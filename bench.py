#!/usr/bin/env python3
"""Rollout benchmark on one MI355X: `python bench.py --gpus 1 --steps K --warmup W` prints ONE JSON line.

A step is one rollout_step() of the whole hot path (refill + prefill, decode of every running slot through all
layers, LM head, argmax/EOS, eviction, page growth; harvest whenever a full update group is ready) on the
8B-shaped, 16k-cap workload.

`value` is measured on a timed window of K steps that starts from a representative mid-run state: the library's
scheduler is first run alone (no model) over the whole workload, the step whose in-flight context is closest to the
run's average is taken, and that state is recreated through the public API by submitting each running rollout as
prompt + already generated tokens (what partial mode re-feeds after an interruption); their prefill is warm-up.

`whole_job` puts the whole workload -- cold start, steady state, the bulk re-prefills after staleness evictions and
the tail drain -- into the same line without running its half million kernels: a few more short windows are timed at
other points of the scheduler-only trace (cold start, late steady state, three points of the tail drain), a
per-step cost model  t = a + b rows + c cached_tokens (+ g + alpha prefill_tokens + beta prefill_query_key_pairs on
steps that refill slots)  is fitted to every timed step, and the model is summed over the exact per-step work record
of the scheduler-only trace.  `bench.py --full-run` executes the whole job for real; its last recorded figure is
quoted beside the estimate.
"""
import argparse
import json
import math
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def recorded(path, key):
    """A `key = number` line of a tracked profile summary (None when the file or the key is missing)."""
    try:
        m = re.search(rf"^{re.escape(key)}\s*=\s*([-+0-9.eE]+)", open(os.path.join(ROOT, "profiles", path)).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def device_weights(torch, m, seed):
    """bf16 N(0, 0.02) blob in weights-blob order, generated on the GPU (norm gains 1)."""
    import workloads as W
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    n = W.weight_count(m)
    blob = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
    off = 0
    for name, r, c in W.weight_layout(m):
        v = blob[off:off + r * c]
        if name.endswith("norm"):
            v.fill_(1.0)
        else:
            step = 1 << 28
            for a in range(0, r * c, step):
                v[a:a + step].normal_(0.0, 0.02, generator=g)
        off += r * c
    torch.cuda.synchronize()
    return blob


# ---- the scheduler-only pass: exact per-step work record of the whole job -------------------------------------------
def scheduler_trace(R, wl, L, snap_steps, mode=0):
    """Run the library's own scheduler without the model (ROLLOUT_DEBUG_NO_MODEL: same kernels, same page accounting)
    over the whole workload.  Returns (per-step work arrays, final stats, {step: snapshot}) where a snapshot lists the
    rollouts running / queued before that step with their generated lengths."""
    m = wl.model
    offs = np.arange(wl.n_prompts + 1, dtype=np.uint32) * wl.prompt_len
    toks = np.zeros(wl.n_prompts * wl.prompt_len, np.int32)
    stale = wl.max_staleness if mode == 0 else -1

    def mk():
        cfg = R.make_cfg(m, max_slots=wl.max_slots, max_prompt_len=wl.prompt_len, max_new_tokens=wl.cap,
                         max_seqs=wl.n_prompts, kv_pool_bytes=wl.kv_pool_bytes, max_staleness=stale, mode=mode,
                         debug_flags=R.ROLLOUT_DEBUG_NO_MODEL)
        c = R.rollout_init(np.zeros(1, np.uint16), cfg)
        R.rollout_submit(c, toks, offs, L.astype(np.uint32))
        return c

    def snapshot(c, step):
        running, queued = [], []
        for sid in range(wl.n_prompts):
            tk, _, state, slot = R.rollout_peek(c, sid, wl.cap)
            if state == 1:
                running.append((slot, sid, len(tk)))
            elif state == 0:
                queued.append((0 if len(tk) else 1, sid, len(tk)))   # resumed rollouts wait ahead of fresh prompts
        return dict(step=step, running=[(sid, g) for _, sid, g in sorted(running)],
                    queued=[(sid, g) for _, sid, g in sorted(queued)])

    def run(c, snaps_at):
        rec = dict(ran=[], rows=[], ctx=[], pf_tok=[], pf_pairs=[], queued=[], active=[])
        snaps = {}
        s = 0
        while True:
            if s in snaps_at:
                snaps[s] = snapshot(c, s)
            i = R.rollout_step(c)
            rec["ran"].append(i.n_ran); rec["rows"].append(i.n_decode_rows); rec["ctx"].append(i.decode_ctx_tokens)
            rec["pf_tok"].append(i.prefill_tokens); rec["pf_pairs"].append(i.prefill_ctx_pairs)
            rec["queued"].append(i.n_queued); rec["active"].append(i.n_active)
            if i.n_finished_unharvested >= wl.harvest:
                R.rollout_harvest(c, wl.harvest, 0, want_logp=False)
            s += 1
            if i.n_active == 0 and i.n_queued == 0:
                break
        st = R.rollout_stats(c)
        R.rollout_destroy(c)
        return {k: np.array(v, np.float64) for k, v in rec.items()}, st, snaps

    return run(mk(), set(snap_steps))


def cpu_baseline(wl, ctx_lens, budget_s=24.0):
    """The oracle as it stands (numpy, fp32), timed on this host: per-token decode time of 1- and 2-layer slices at
    full widths, extrapolated linearly to all layers; once with the BLAS threads numpy picks, once with one."""
    import workloads as W
    from oracle import ContiguousKV, OracleModel
    try:
        import threadpoolctl
    except Exception:
        threadpoolctl = None

    def measure(n_threads, budget):
        t_of = {}
        g = np.random.default_rng(0)
        n_done = 0
        for nl in (1, 2):
            m = wl.model.with_layers(nl)
            w = {}
            for name, r, c in W.weight_layout(m):
                w[name] = np.ones((r, c), np.float32) if name.endswith("norm") else \
                    g.standard_normal((r, c), dtype=np.float32) * np.float32(0.02)
            model = OracleModel(m, w, np.float32)
            times = []
            t_start = time.time()
            for L in ctx_lens:
                cache = ContiguousKV(nl)
                for l in range(nl):
                    cache.k[l] = list(g.standard_normal((L, m.n_kv_heads, m.head_dim), dtype=np.float32))
                    cache.v[l] = list(g.standard_normal((L, m.n_kv_heads, m.head_dim), dtype=np.float32))
                t0 = time.time()
                if threadpoolctl is not None and n_threads:
                    with threadpoolctl.threadpool_limits(limits=n_threads):
                        model.token_forward(int(g.integers(0, m.vocab - 1)), int(L), cache)
                else:
                    model.token_forward(int(g.integers(0, m.vocab - 1)), int(L), cache)
                times.append(time.time() - t0)
                if time.time() - t_start > budget / 2:
                    break
            t_of[nl] = float(np.mean(times))
            n_done = len(times)
            del model, w
        return 1.0 / (t_of[1] + (wl.model.n_layers - 1) * max(t_of[2] - t_of[1], 0.0)), n_done

    blas_threads = 1
    if threadpoolctl is not None and threadpoolctl.threadpool_info():
        blas_threads = max(int(i.get("num_threads", 1)) for i in threadpoolctl.threadpool_info())
    v_all, n_all = measure(0, budget_s * 0.6)
    v_one, n_one = (measure(1, budget_s * 0.4) if threadpoolctl is not None else (None, 0))
    return dict(value=v_all, unit="tokens/s", cores=blas_threads, kind="oracle",
                single_thread=dict(value=v_one, cores=1, contexts=n_one),
                host_cores=os.cpu_count(),
                sample=f"numpy fp32 oracle, one decode token at {n_all} in-flight contexts "
                       f"(mean {int(np.mean(ctx_lens[:max(1, n_all)]))} tokens), 1- and 2-layer slices at full widths, "
                       f"extrapolated to {wl.model.n_layers} layers; `cores` = BLAS threads used by the matrix-vector "
                       f"products, the rest of the oracle is single-threaded Python")


def attention_alone(torch, R, iters=20):
    """The decode-attention kernel alone on the 256-sequence long-tail case: HIP-event time per launch."""
    import workloads as W
    a = W.ATTN_CASE
    Hq, Hkv, d, n = a["n_q_heads"], a["n_kv_heads"], a["head_dim"], a["n_seqs"]
    lens = W.make_kv_lengths(n, a["median"], a["sigma"], a["cap"], a["seed_lengths"])
    table, n_pool = W.make_page_table(lens, 16, a["seed_pages"])
    dev = torch.device("cuda:0")
    g = torch.Generator(device="cuda:0")
    g.manual_seed(a["seed_values"])
    pools = []
    for _ in range(3):   # rotate pools so no launch finds its KV in the 256 MB last-level cache
        p = torch.empty(R.rollout_attn_pool_bytes(n_pool, Hkv, d) // 2, dtype=torch.bfloat16, device=dev)
        p.normal_(0.0, 1.0, generator=g)
        pools.append(p)
    q = torch.empty((n, Hq, d), dtype=torch.bfloat16, device=dev).normal_(0.0, 1.0, generator=g)
    tab = torch.from_numpy(np.maximum(table, 0).astype(np.int32)).to(dev)
    ws_bytes = R.rollout_attn_workspace_bytes(n, int(lens.sum()), Hq, d)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
    n_work, chunk = R.rollout_attn_plan(lens, Hq, Hkv, d, ws.data_ptr(), ws_bytes)
    out = torch.empty((n, Hq, d), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def launch(i):
        R.rollout_attn_decode(pools[i % 3].data_ptr(), Hq, Hkv, d, q.data_ptr(), tab.data_ptr(), table.shape[1], n,
                              n_work, chunk, out.data_ptr(), 0, ws.data_ptr(), stream.cuda_stream)
    for i in range(3):
        launch(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        launch(i)
        e1.record(stream)
    torch.cuda.synchronize()
    ms = np.array([e0.elapsed_time(e1) for e0, e1 in evs])
    # practical ceiling: a pure 16-byte-per-lane read of the same pools (rotated), same event timing
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    pool_bytes = pools[0].numel() * 2 // 16 * 16
    rd = []
    for i in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        R.rollout_stream_read(pools[i % 3].data_ptr(), pool_bytes, sink.data_ptr(), stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        rd.append(pool_bytes / e0.elapsed_time(e1) / 1e6)
    # one plain copy of known size (1 GiB read + 1 GiB written): the dispatch the memory counters are calibrated on
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_(generator=g)
    cal_dst = torch.empty_like(cal_src)
    R.rollout_stream_copy(cal_src.data_ptr(), cal_dst.data_ptr(), cal_src.numel() * 4, stream.cuda_stream)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    bytes_per = int(lens.sum()) * Hkv * 2 * d * 2 + 2 * n * Hq * d * 2 + int(((lens + 15) // 16).sum()) * 4
    return dict(median_ms=float(np.median(ms)), gbps=bytes_per / np.median(ms) / 1e6, bytes=bytes_per,
                kv_tokens=int(lens.sum()), frac_of_8TBps=bytes_per / np.median(ms) / 1e6 / 8000.0,
                pure_read_ceiling_gbps=float(np.median(rd[2:])))


def pool_bytes_for(wl, m):
    page_bytes = wl.model.n_layers * wl.model.n_kv_heads * 2 * 16 * wl.model.head_dim * 2
    pb = wl.kv_pool_bytes or min(120 * 10**9, wl.max_slots * ((wl.prompt_len + wl.cap + 15) // 16) * page_bytes)
    return pb * m.n_layers // wl.model.n_layers


class Window:
    """A short run of real steps from a recreated mid-run state: every step's wall time with the work it did."""

    def __init__(self, torch, R, W, wl, m, L, blob, snap, label):
        self.R, self.torch, self.wl, self.m, self.label, self.snap = R, torch, wl, m, label, snap
        order = snap["running"] + snap["queued"]
        g = W.rng(wl.seed_prompts)
        prompts = [g.integers(0, m.vocab - 1, size=wl.prompt_len + gl, dtype=np.int64).astype(np.int32) for _, gl in order]
        targets = np.array([int(L[sid]) - gl for sid, gl in order], np.uint32)
        # the warm start inflates max_prompt_len, so never let the library size the pool for the worst case: use the
        # workload's pool, else the worst case of the ORIGINAL workload capped at 120 GB (the 32B weights need the rest)
        cfg = R.make_cfg(m, max_slots=wl.max_slots, max_prompt_len=wl.prompt_len + max(gl for _, gl in order),
                         max_new_tokens=int(targets.max()), max_seqs=len(order), kv_pool_bytes=pool_bytes_for(wl, m),
                         weights_on_device=1, max_staleness=wl.max_staleness, debug_flags=R.ROLLOUT_DEBUG_TIME_ATTN)
        self.ctx = R.rollout_init((blob.data_ptr(), blob.numel() * 2), cfg)
        offs = np.zeros(len(prompts) + 1, np.uint32)
        offs[1:] = np.cumsum([len(p) for p in prompts])
        R.rollout_submit(self.ctx, np.concatenate(prompts), offs, targets)
        self.samples = []     # (rows, ctx, pf_tokens, pf_pairs, seconds, n_ran)
        # algorithmic HBM bytes of one step (what the method must move): every weight once (the embedding table is
        # gathered, not streamed), the cached K/V of every decode row, the new K/V rows and the fp32 logits rows
        self.weight_bytes = 2 * (W.weight_count(m) - m.vocab * m.d_model)
        self.kv_bytes_per_tok = m.n_layers * m.n_kv_heads * 2 * m.head_dim * 2
        self.model_bytes = 0

    def step(self):
        R, wl, m = self.R, self.wl, self.m
        t0 = time.perf_counter()
        i = R.rollout_step(self.ctx)
        if i.n_finished_unharvested >= wl.harvest:
            R.rollout_harvest(self.ctx, wl.harvest, 0, want_logp=True)
        dt = time.perf_counter() - t0
        self.samples.append((i.n_decode_rows, i.decode_ctx_tokens, i.prefill_tokens, i.prefill_ctx_pairs, dt, i.n_ran))
        self.model_bytes += self.weight_bytes + (i.decode_ctx_tokens + i.prefill_tokens) * self.kv_bytes_per_tok + \
            i.n_ran * m.vocab * 4
        return i

    def close(self):
        self.R.rollout_destroy(self.ctx)
        self.torch.cuda.empty_cache()


def fit_cost_model(samples):
    """Least squares (relative residuals) of the step time on its work: decode steps t = a + b rows + c ctx; steps that
    also prefill add g + alpha tokens + beta pairs on top of the decode model."""
    S = np.array(samples, np.float64)
    rows, ctx, pft, pfp, t = S[:, 0], S[:, 1], S[:, 2], S[:, 3], S[:, 4]
    dec = pft == 0
    A = np.stack([np.ones(dec.sum()), rows[dec], ctx[dec]], 1)
    w = 1.0 / t[dec]
    d_coef, *_ = np.linalg.lstsq(A * w[:, None], t[dec] * w, rcond=None)
    d_coef = np.maximum(d_coef, 0.0)

    def t_dec(r, c):
        return (d_coef[0] + d_coef[1] * r + d_coef[2] * c) * (r > 0)
    pf = ~dec
    p_coef = np.zeros(3)
    if pf.sum() >= 3:
        resid = t[pf] - t_dec(rows[pf], ctx[pf])
        B = np.stack([np.ones(pf.sum()), pft[pf], pfp[pf]], 1)
        wp = 1.0 / np.maximum(t[pf], 1e-6)
        p_coef, *_ = np.linalg.lstsq(B * wp[:, None], resid * wp, rcond=None)
        p_coef = np.maximum(p_coef, 0.0)

    def predict(r, c, tok, pairs):
        return t_dec(r, c) + (p_coef[0] + p_coef[1] * tok + p_coef[2] * pairs) * (tok > 0)
    pred = predict(rows, ctx, pft, pfp)
    rel = (pred - t) / t
    return predict, dict(decode=dict(per_step_s=d_coef[0], per_row_s=d_coef[1], per_cached_token_s=d_coef[2]),
                         prefill=dict(per_refill_step_s=p_coef[0], per_token_s=p_coef[1], per_query_key_pair_s=p_coef[2]),
                         fit_rms_rel=float(np.sqrt(np.mean(rel ** 2))), fit_max_rel=float(np.max(np.abs(rel))),
                         n_decode_samples=int(dec.sum()), n_prefill_samples=int(pf.sum()))


def full_run(torch, R, W, wl, m, L, mode="partial"):
    """Whole job, cold start to drain: every prompt prefilled, every token decoded, harvest whenever a group is ready
    (with the boundary work that entails), tail drain included.  Reports whole-job tokens/s and the three bubble ratios.
    mode: "partial" (the default operating mode, with the workload's staleness bound), "onpolicy" (unfinished rollouts
    are terminated and their tokens discarded at every update boundary) or "sync" (the canonical baseline: a batch is
    admitted only when every slot is empty).  tokens/s counts harvested tokens only, so discarded work lowers it."""
    mode_id = {"partial": R.ROLLOUT_MODE_PARTIAL, "onpolicy": R.ROLLOUT_MODE_ONPOLICY, "sync": R.ROLLOUT_MODE_SYNC}[mode]
    stale = wl.max_staleness if mode == "partial" else -1
    blob = device_weights(torch, m, wl.seed_weights)
    cfg = R.make_cfg(m, max_slots=wl.max_slots, max_prompt_len=wl.prompt_len, max_new_tokens=wl.cap, max_seqs=wl.n_prompts,
                     kv_pool_bytes=pool_bytes_for(wl, m), weights_on_device=1,
                     max_staleness=stale, mode=mode_id, debug_flags=R.ROLLOUT_DEBUG_TIME_ATTN)
    ctx = R.rollout_init((blob.data_ptr(), blob.numel() * 2), cfg)
    del blob
    torch.cuda.empty_cache()
    prompts = W.make_prompts(wl.n_prompts, wl.prompt_len, m.vocab, wl.seed_prompts)
    offs = np.arange(wl.n_prompts + 1, dtype=np.uint32) * wl.prompt_len
    R.rollout_submit(ctx, prompts.reshape(-1), offs, L.astype(np.uint32))
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    idle_time = 0.0
    harvested = steps = 0
    last_print = t_start
    while True:
        t0 = time.perf_counter()
        i = R.rollout_step(ctx)
        dt = time.perf_counter() - t0
        idle_time += (wl.max_slots - i.n_ran) * dt
        steps += 1
        if i.n_finished_unharvested >= wl.harvest:
            ng, recs, tk, lp = R.rollout_harvest(ctx, wl.harvest, 0, want_logp=True)
            harvested += len(recs)
        if i.n_active == 0 and i.n_queued == 0:
            break
        if time.perf_counter() - last_print > 30:
            last_print = time.perf_counter()
            print(f"[full-run] step {steps} active {i.n_active} queued {i.n_queued} harvested {harvested} "
                  f"elapsed {last_print - t_start:.0f}s", file=sys.stderr, flush=True)
    ng, recs, tk, lp = R.rollout_harvest(ctx, wl.harvest, R.ROLLOUT_FLUSH, want_logp=True)
    harvested += len(recs)
    torch.cuda.synchronize()
    T = time.perf_counter() - t_start
    st = R.rollout_stats(ctx)
    R.rollout_destroy(ctx)
    useful = int(st.gen_tokens - st.discarded_tokens)
    assert harvested == wl.n_prompts and useful == int(L.sum())
    kvb = m.n_kv_heads * 2 * m.head_dim * 2
    out = dict(metric=f"rollout tokens/s, whole job ({wl.name}, {mode} mode)", value=useful / T, unit="tokens/s", n_gpus=1,
               steps=int(st.steps), warmup=0, ms_per_step=1e3 * T / st.steps, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload=f"{wl.name}: whole job from a cold start to drain, {m.n_layers} layers, Q={wl.max_slots}, "
                                    f"{wl.n_prompts} prompts x {wl.prompt_len}, cap {wl.cap}, harvest {wl.harvest}, "
                                    f"max_staleness {stale}, {mode} mode",
                           wall_s=T, gen_tokens=int(st.gen_tokens), discarded_tokens=int(st.discarded_tokens),
                           prefill_tokens=int(st.prefill_tokens),
                           n_stale=int(st.n_stale), n_preempt=int(st.n_preempt)),
               bubble_ratio=dict(steps=st.idle / (wl.max_slots * st.steps),
                                 steps_while_queue_non_empty=(st.idle_q / (wl.max_slots * st.steps_q)) if st.steps_q else 0.0,
                                 wall_time_weighted=idle_time / (wl.max_slots * T)),
               roofline=dict(bound="hbm", kernel="k_decode_attn, all decode launches of the job",
                             achieved=(st.attn_kv_tokens * kvb) / max(st.attn_ms, 1e-9) / 1e6, peak=8000.0, unit="GB/s",
                             frac=(st.attn_kv_tokens * kvb) / max(st.attn_ms, 1e-9) / 1e6 / 8000.0, traffic=None,
                             launches=int(st.attn_launches)))
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="8b_long")
    ap.add_argument("--layers", type=int, default=0, help="debug: override the layer count (invalidates the result)")
    ap.add_argument("--at-step", type=int, default=-1,
                    help="debug: start the timed window from this scheduler step instead of the mean-context one "
                         "(e.g. a late step to look at the tail drain; changes what the result means)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-attn-alone", action="store_true")
    ap.add_argument("--no-whole-job", action="store_true", help="skip the extra windows and the whole-job estimate")
    ap.add_argument("--full-run", action="store_true",
                    help="run the whole workload from a cold start to drain and report whole-job tokens/s "
                         "(minutes of GPU time; not the default bench line)")
    ap.add_argument("--mode", choices=["partial", "onpolicy", "sync"], default="partial",
                    help="operating mode of a --full-run (the default window always runs partial mode)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2603_23414_amd as R
    import workloads as W
    wl = W.CONFIGS[args.workload]
    m = wl.model if not args.layers else wl.model.with_layers(args.layers)
    L = W.make_target_lengths(wl.n_prompts, wl.len_mu, wl.len_sigma, wl.cap, wl.seed_lengths)
    if args.full_run:
        return full_run(torch, R, W, wl, m, L, args.mode)

    # ---- scheduler-only passes: the job's exact work record, the bubble ratios, the states to time ------------------
    t0 = time.time()
    rec0, st0, _ = scheduler_trace(R, wl, L, set())
    n_steps = len(rec0["ran"])
    q_empty = int(np.nonzero(rec0["queued"] == 0)[0][0]) if (rec0["queued"] == 0).any() else n_steps - 1
    tail = n_steps - q_empty
    # the headline state: the step (with a non-empty queue) whose in-flight context is closest to the mean over such steps
    steady = np.nonzero((rec0["queued"] > 0) & (rec0["rows"] > 0))[0]
    if len(steady) == 0:
        steady = np.nonzero(rec0["rows"] > 0)[0]
    mean_ctx_sum = float(rec0["ctx"][steady].mean())
    head_step = int(steady[np.argmin(np.abs(rec0["ctx"][steady] - mean_ctx_sum))]) if args.at_step < 0 else args.at_step
    extra = {} if args.no_whole_job else {
        "cold start": 0,
        "late steady state": max(1, int(q_empty * 0.85)),
        "tail drain 15%": q_empty + int(tail * 0.15),
        "tail drain 45%": q_empty + int(tail * 0.45),
        "tail drain 80%": q_empty + int(tail * 0.80),
    }
    rec, st, snaps = scheduler_trace(R, wl, L, {head_step, *extra.values()})
    assert np.array_equal(rec["ran"], rec0["ran"])
    _, st_sync, _ = scheduler_trace(R, wl, L, set(), mode=2)
    full = dict(steps=int(st.steps), bubble=st.idle / (wl.max_slots * st.steps), n_stale=int(st.n_stale),
                n_preempt=int(st.n_preempt), prefill_tokens=int(st.prefill_tokens), gen_tokens=int(st.gen_tokens),
                bubble_sync_baseline=st_sync.idle / (wl.max_slots * st_sync.steps), queue_empty_at_step=q_empty)
    snap = snaps[head_step]
    snap["mean_ctx_sum"] = mean_ctx_sum
    print(f"[bench] scheduler-only passes: {full} headline snapshot step {snap['step']} ({time.time() - t0:.1f}s)",
          file=sys.stderr)

    attn = None if args.no_attn_alone else attention_alone(torch, R)
    if attn:
        print(f"[bench] attention alone: {attn}", file=sys.stderr)

    blob = device_weights(torch, m, wl.seed_weights)

    # ---- the headline window: W warm-up steps (incl. the warm-start prefill), then exactly K timed steps --------------
    win = Window(torch, R, W, wl, m, L, blob, snap, "headline")
    t0 = time.time()
    for _ in range(args.warmup):
        win.step()
    torch.cuda.synchronize()
    print(f"[bench] warm-up ({args.warmup} steps incl. warm-start prefill): {time.time() - t0:.1f}s", file=sys.stderr)
    s0 = R.rollout_stats(win.ctx)
    win.model_bytes = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = 0
    for _ in range(args.steps):
        tokens += win.step().n_ran
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    s1 = R.rollout_stats(win.ctx)
    model_bytes = win.model_bytes
    win.close()
    samples = list(win.samples)

    launches = s1.attn_launches - s0.attn_launches
    kv_tok = s1.attn_kv_tokens - s0.attn_kv_tokens
    attn_ms = s1.attn_ms - s0.attn_ms
    kv_bytes_tok = m.n_kv_heads * 2 * m.head_dim * 2
    dec_rows = sum(s[0] for s in win.samples[args.warmup:])
    alg_bytes = kv_tok * kv_bytes_tok + dec_rows * m.n_layers * (2 * m.n_q_heads * m.head_dim * 2)
    achieved = alg_bytes / max(attn_ms, 1e-9) / 1e6 if launches else 0.0
    # HBM traffic per launch: the counters' FETCH_SIZE + WRITE_SIZE (scaled by the copy-kernel calibration) relative to
    # the algorithmic bytes, as recorded in the tracked profile of this same command, times this run's algorithmic bytes
    ratio = recorded("bench_8b_long_hbm_traffic_pmc.txt", "traffic_over_algorithmic") if wl.name == "8b_long" and not args.layers else None
    roofline = dict(bound="hbm", kernel="k_decode_attn (ragged paged GQA decode attention, in situ)",
                    achieved=achieved, peak=8000.0, unit="GB/s", frac=achieved / 8000.0,
                    traffic=(ratio * alg_bytes / max(1, launches)) if ratio else None,
                    traffic_source="profiles/bench_8b_long_hbm_traffic_pmc.txt: traffic_over_algorithmic x this run's "
                                   "algorithmic bytes per launch" if ratio else None,
                    launches=int(launches), avg_launch_ms=attn_ms / max(1, launches),
                    alg_bytes_per_launch=alg_bytes / max(1, launches))

    # ---- the other windows and the whole-job estimate ------------------------------------------------------------
    whole = None
    if extra:
        t0 = time.time()
        windows = [dict(label="headline", step=snap["step"], steps=len(win.samples),
                        ms_per_decode_step=1e3 * float(np.mean([s[4] for s in win.samples if s[2] == 0])),
                        rows=float(np.mean([s[0] for s in win.samples if s[2] == 0])))]
        for label, s_at in extra.items():
            w2 = Window(torch, R, W, wl, m, L, blob, snaps[s_at], label)
            n_w = 12 if s_at else 8
            for _ in range(n_w):
                w2.step()
            w2.close()
            dec = [s for s in w2.samples if s[2] == 0]
            windows.append(dict(label=label, step=s_at, steps=n_w, rows=float(np.mean([s[0] for s in dec])) if dec else 0.0,
                                ms_per_decode_step=1e3 * float(np.mean([s[4] for s in dec])) if dec else None,
                                warm_start=dict(prefill_tokens=int(w2.samples[0][2]), seconds=w2.samples[0][4])))
            samples += w2.samples
        predict, model = fit_cost_model(samples)
        t_step = predict(rec["rows"], rec["ctx"], rec["pf_tok"], rec["pf_pairs"])
        T_est = float(t_step.sum())
        useful = int(L.sum())
        pf_part = float((t_step - predict(rec["rows"], rec["ctx"], 0 * rec["pf_tok"], 0 * rec["pf_pairs"])).sum())
        whole = dict(tokens_per_s=useful / T_est, wall_s=T_est, tokens=useful, steps=n_steps,
                     method="per-step cost model fitted to the timed steps of all windows, summed over the scheduler-only "
                            "trace of the whole job (every step's rows, cached tokens, prefill tokens and pairs)",
                     seconds_in_prefill=pf_part, seconds_in_tail_drain=float(t_step[q_empty:].sum()),
                     bubble_wall_time_weighted=float(((wl.max_slots - rec["ran"]) * t_step).sum() / (wl.max_slots * T_est)),
                     cost_model=model, windows=windows,
                     recorded_full_run=dict(tokens_per_s=recorded(f"full_run_{wl.name}.txt", "whole_job_tokens_per_s"),
                                            wall_s=recorded(f"full_run_{wl.name}.txt", "wall_s"),
                                            bubble_wall_time_weighted=recorded(f"full_run_{wl.name}.txt", "bubble_wall_time_weighted"),
                                            source=f"profiles/full_run_{wl.name}.txt (bench.py --workload {wl.name} --full-run)"))
        print(f"[bench] whole-job estimate: {whole['tokens_per_s']:.0f} tokens/s over {T_est:.0f}s "
              f"(windows {time.time() - t0:.1f}s)", file=sys.stderr)
    del blob

    shape_name = 'LLaMA-3.1-8B' if m.d_model == 4096 else 'Qwen-2.5-32B' if m.d_model == 5120 else 'tiny'
    out = dict(metric="rollout tokens/s (8B shape, 16k-cap lengths)" if wl.name == "8b_long" else f"rollout tokens/s ({wl.name})",
               value=tokens / dt, unit="tokens/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=1e3 * dt / args.steps, higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload=f"{wl.name}: {shape_name} shape ({m.n_layers} layers), Q={wl.max_slots}, "
                                    f"{wl.n_prompts} prompts x {wl.prompt_len}, LogNormal(median {math.exp(wl.len_mu):.0f}, "
                                    f"sigma {wl.len_sigma}) cap {wl.cap}, KV pool "
                                    f"{(str(round(wl.kv_pool_bytes / 1e9)) + ' GB') if wl.kv_pool_bytes else 'worst-case'}, harvest {wl.harvest}, "
                                    f"max_staleness {wl.max_staleness}; timed window from scheduler step "
                                    f"{snap['step']} ({'mean in-flight context' if args.at_step < 0 else 'chosen by --at-step'})",
                           window_only=True,
                           window_note="`value` is the rate inside the timed window (full batch at the mean in-flight context); "
                                       "the whole job, with its re-prefills and tail drain, is `whole_job.tokens_per_s`",
                           mean_inflight_ctx=snap.get("mean_ctx_sum", 0.0) / wl.max_slots,
                           prefill_tokens_in_window=int(s1.prefill_tokens - s0.prefill_tokens),
                           stale_evictions_in_window=int(s1.n_stale - s0.n_stale)),
               roofline=roofline,
               bubble_ratio=dict(whole_run_steps=full["bubble"], sync_baseline_steps=full["bubble_sync_baseline"],
                                 wall_time_weighted=whole["bubble_wall_time_weighted"] if whole else None,
                                 window=(s1.idle - s0.idle) / max(1, wl.max_slots * (s1.steps - s0.steps)),
                                 whole_run_n_steps=full["steps"], n_stale=full["n_stale"], n_preempt=full["n_preempt"]),
               whole_job=whole,
               end_to_end_hbm=dict(alg_bytes_per_step=model_bytes / args.steps, achieved=model_bytes / dt / 1e9,
                                   peak=8000.0, unit="GB/s", frac=model_bytes / dt / 1e9 / 8000.0,
                                   note="weights once + cached K/V of every decode row + new K/V + fp32 logits, "
                                        "per step, over the wall time of the timed steps (prefill flops not counted)"),
               attn_alone=attn)
    if not args.no_cpu_baseline:
        live = [wl.prompt_len + gl for _, gl in snap["running"]]
        out["cpu_baseline"] = cpu_baseline(wl, live[:: max(1, len(live) // 12)])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
