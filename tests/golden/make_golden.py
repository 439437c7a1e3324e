"""Writes the stored expected values under tests/golden/ from the CPU oracle alone (never from the HIP path).

    python tests/golden/make_golden.py

Each fixture names the passage of the paper its quantities come from.  tests/test_golden.py checks that the oracle
still reproduces them (a guard against silent drift of the reference), and the GPU suite checks the engine against
the same files."""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import workloads as W                                   # noqa: E402
from oracle import OracleModel, OracleRollout, PagedKV   # noqa: E402


def schedule_fixture(name, *, Q, n, P, cap, G, pool_pages, stale, mode, len_mu, len_sigma, seed, k=1):
    L = W.make_target_lengths(n * k, len_mu, len_sigma, cap, seed)
    o = OracleRollout(max_slots=Q, page_tokens=16, n_pages=pool_pages, max_new_tokens=cap, eos_id=99,
                      max_staleness=stale, mode=mode, page_seed=seed)
    o.submit([np.zeros(P, np.int32)] * n, L, n_responses=k)
    groups = o.run_to_completion(G)
    return dict(
        source="Sec. 3.1 (oversubscription, early harvest, length-ordered groups), Sec. 3.2-3.3 (update boundaries, "
               "cached partial rollouts), eq. 4 (bubble ratio with one decode step as the time unit)",
        config=dict(max_slots=Q, n_prompts=n, responses_per_prompt=k, prompt_len=P, cap=cap, harvest=G,
                    pool_pages=pool_pages, max_staleness=stale, mode=mode, len_mu=len_mu, len_sigma=len_sigma,
                    seed=seed),
        target_len=[int(x) for x in L],
        groups=[[s.seq_id for s in g] for g in groups],
        completion_step=[s.completion_step for s in o.seqs],
        last_slot=[s.last_slot for s in o.seqs],
        n_preempt=[s.n_preempt for s in o.seqs],
        stats=o.stats(),
        bubble_ratio=o.bubble_ratio(),
    ), name


def model_fixture():
    """Config 1 (tiny policy, fp64 oracle on the bf16-rounded weights): greedy rollouts of 6 tokens and the first
    logits row of every prompt, to 1e-9."""
    c = W.CONFIGS["tiny"]
    m = c.model
    blob = W.make_weights(m, c.seed_weights)
    w = {k: W.bf16_bits_to_f32(v) for k, v in W.split_weights(blob, m).items()}
    model = OracleModel(m, w, np.float64)
    prompts = list(W.make_prompts(c.n_prompts, c.prompt_len, m.vocab, c.seed_prompts))
    n_pages = c.max_slots * ((c.prompt_len + c.cap + 15) // 16)
    o = OracleRollout(max_slots=c.max_slots, page_tokens=16, n_pages=n_pages, max_new_tokens=c.cap, eos_id=m.vocab - 1,
                      model=model, kv_pool=PagedKV(m.n_layers, n_pages, 16, m.n_kv_heads, m.head_dim, np.float64))
    o.submit(prompts, [6] * c.n_prompts)
    o.step()
    first = {int(slot): [round(float(x), 9) for x in lg[:8]] for slot, lg in o.last_logits.items()}
    o.run_to_completion(c.harvest)
    return dict(
        source="decoder-only forward pass of the policy (Sec. 4.1 names the model families; shapes of configuration 1), "
               "greedy decoding with the sixth token forced to EOS (Sec. 4.4.1 fixes per-sample lengths)",
        tokens=[s.tokens for s in o.seqs],
        logp=[[round(float(x), 9) for x in s.logp] for s in o.seqs],
        first_step_logits_0_8={str(k): v for k, v in sorted(first.items())},
    ), "tiny_model_rollout"


def main():
    out = [
        schedule_fixture("schedule_partial_refill", Q=8, n=40, P=20, cap=120, G=4, pool_pages=8 * 9, stale=-1, mode=0,
                         len_mu=3.0, len_sigma=0.6, seed=3),
        schedule_fixture("schedule_stale_preempt", Q=6, n=36, P=30, cap=150, G=5, pool_pages=30, stale=1, mode=0,
                         len_mu=3.4, len_sigma=0.8, seed=11),
        schedule_fixture("schedule_on_policy", Q=6, n=24, P=10, cap=80, G=4, pool_pages=6 * 6, stale=-1, mode=1,
                         len_mu=3.0, len_sigma=0.7, seed=12),
        schedule_fixture("schedule_sync_baseline", Q=6, n=24, P=10, cap=80, G=6, pool_pages=6 * 6, stale=-1, mode=2,
                         len_mu=3.0, len_sigma=0.7, seed=12),
        schedule_fixture("schedule_shared_prompt", Q=6, n=8, P=50, cap=60, G=4, pool_pages=28, stale=1, mode=0,
                         len_mu=2.8, len_sigma=0.7, seed=13, k=4),
        model_fixture(),
    ]
    for data, name in out:
        with open(os.path.join(HERE, name + ".json"), "w") as f:
            json.dump(data, f, indent=1, sort_keys=True)
            f.write("\n")
        print("wrote", name)


if __name__ == "__main__":
    main()
