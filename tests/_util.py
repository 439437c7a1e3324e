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
