"""ctypes binding of include/rollout.h: same names, argument marshalling only.

There is no fallback: if librollout.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

__all__ = [
    "LIB_PATH", "lib", "RolloutError", "rollout_cfg", "rollout_step_info", "rollout_traj", "rollout_stats_t",
    "rollout_init", "rollout_submit", "rollout_step", "rollout_step_forced", "rollout_harvest", "rollout_stats",
    "rollout_peek", "rollout_slot_pages", "rollout_destroy", "rollout_last_error",
    "rollout_attn_pool_bytes", "rollout_attn_write_kv", "rollout_attn_workspace_bytes", "rollout_attn_plan",
    "rollout_attn_decode", "rollout_gemm_workspace_bytes", "rollout_gemm_bf16", "rollout_stream_copy",
    "rollout_stream_read", "rollout_gemm_packed_bytes", "rollout_gemm_pack_weights", "rollout_update_weights",
    "rollout_submit_n", "rollout_gemm_swiglu_bf16", "rollout_gemm_kernel_name", "rollout_gemm_splits",
    "rollout_gemm_bf16_static", "rollout_gemm_static_scratch_bytes", "make_cfg",
    "ROLLOUT_FLUSH", "ROLLOUT_DEBUG_NO_MODEL", "ROLLOUT_DEBUG_TIME_ATTN", "ROLLOUT_MODE_PARTIAL",
    "ROLLOUT_MODE_ONPOLICY", "ROLLOUT_MODE_SYNC", "ROLLOUT_EOS_FORCED_ONLY", "ROLLOUT_EOS_NATURAL_OR_FORCED",
    "EXPORTS",
]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librollout.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not built: run `python -m paper_2603_23414_amd.build` "
                      "(or __graft_entry__.build()); there is no fallback path")
lib = C.CDLL(LIB_PATH)

ROLLOUT_FLUSH = 1
ROLLOUT_DEBUG_NO_MODEL, ROLLOUT_DEBUG_TIME_ATTN = 1, 2
ROLLOUT_MODE_PARTIAL, ROLLOUT_MODE_ONPOLICY, ROLLOUT_MODE_SYNC = 0, 1, 2
ROLLOUT_EOS_FORCED_ONLY, ROLLOUT_EOS_NATURAL_OR_FORCED = 0, 1
_ERR = {-1: "EINVAL", -2: "ENOMEM", -3: "EBUSY", -4: "ERANGE", -5: "EDEVICE"}

EXPORTS = [
    "rollout_init", "rollout_submit", "rollout_step", "rollout_harvest", "rollout_stats", "rollout_step_forced",
    "rollout_peek", "rollout_slot_pages", "rollout_last_error", "rollout_destroy", "rollout_attn_pool_bytes",
    "rollout_attn_write_kv", "rollout_attn_workspace_bytes", "rollout_attn_plan", "rollout_attn_decode",
    "rollout_gemm_workspace_bytes", "rollout_gemm_bf16", "rollout_stream_copy", "rollout_stream_read",
    "rollout_gemm_packed_bytes", "rollout_gemm_pack_weights", "rollout_update_weights", "rollout_submit_n",
    "rollout_gemm_swiglu_bf16", "rollout_gemm_kernel_name", "rollout_gemm_splits", "rollout_gemm_bf16_static",
    "rollout_gemm_static_scratch_bytes",
]


class RolloutError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR.get(code, code)}: {msg}")
        self.code = code


class rollout_cfg(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("qkv_bias", C.c_uint32), ("weight_dtype", C.c_uint32),
        ("weights_on_device", C.c_uint32), ("max_slots", C.c_uint32), ("page_tokens", C.c_uint32),
        ("kv_pool_bytes", C.c_uint64), ("max_prompt_len", C.c_uint32), ("max_new_tokens", C.c_uint32),
        ("max_seqs", C.c_uint32), ("eos_id", C.c_int32), ("eos_mode", C.c_uint32), ("mode", C.c_uint32),
        ("max_staleness", C.c_int32), ("grouped_loading", C.c_uint32), ("debug_flags", C.c_uint32),
        ("page_seed", C.c_uint64), ("device", C.c_int32), ("reserved", C.c_uint32), ("temperature", C.c_float),
        ("reserved2", C.c_uint32), ("sample_seed", C.c_uint64)]


class rollout_step_info(C.Structure):
    _fields_ = [("step", C.c_uint64)] + [(n, C.c_uint32) for n in
                ("n_ran", "n_active", "n_finished_unharvested", "n_queued", "free_pages", "n_admitted",
                 "n_finished_step", "n_preempted_step")] + [("ctx_tokens", C.c_uint64), ("n_decode_rows", C.c_uint32),
                                                            ("prefill_tokens", C.c_uint32),
                                                            ("decode_ctx_tokens", C.c_uint64),
                                                            ("prefill_ctx_pairs", C.c_uint64)]


class rollout_traj(C.Structure):
    _fields_ = [("seq_id", C.c_uint64), ("slot", C.c_uint32), ("completion_step", C.c_uint32),
                ("gen_len", C.c_uint32), ("group_idx", C.c_uint32), ("tok_off", C.c_uint64),
                ("n_preempt", C.c_uint32), ("policy_version", C.c_uint32)]


class rollout_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("steps", "busy", "idle", "steps_q", "idle_q", "gen_tokens", "discarded_tokens", "prefill_tokens",
                 "n_preempt", "n_stale", "version", "n_pages", "max_pages_used", "attn_launches",
                 "attn_kv_tokens")] + [("attn_ms", C.c_double), ("wall_ms_steps", C.c_double)]


_vp, _u32, _u64, _i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32
lib.rollout_init.argtypes = [C.POINTER(_vp), _vp, C.c_size_t, C.POINTER(rollout_cfg)]
lib.rollout_update_weights.argtypes = [_vp, _vp, C.c_size_t]
lib.rollout_submit.argtypes = [_vp, _vp, _vp, _vp, _u32, C.POINTER(_u64)]
lib.rollout_submit_n.argtypes = [_vp, _vp, _vp, _vp, _u32, _u32, C.POINTER(_u64)]
lib.rollout_step.argtypes = [_vp, C.POINTER(rollout_step_info)]
lib.rollout_step_forced.argtypes = [_vp, _vp, _vp, C.POINTER(rollout_step_info)]
lib.rollout_harvest.argtypes = [_vp, _u32, _u32, _vp, _u32, _vp, _vp, _u64, C.POINTER(_u32), C.POINTER(_u32),
                                C.POINTER(_u64)]
lib.rollout_stats.argtypes = [_vp, C.POINTER(rollout_stats_t)]
lib.rollout_peek.argtypes = [_vp, _u64, _vp, _vp, _u32, C.POINTER(_u32), C.POINTER(_u32), C.POINTER(_i32)]
lib.rollout_slot_pages.argtypes = [_vp, _u32, _vp, _u32, C.POINTER(_u32)]
lib.rollout_last_error.argtypes = [_vp]
lib.rollout_last_error.restype = C.c_char_p
lib.rollout_destroy.argtypes = [_vp]
lib.rollout_destroy.restype = None
lib.rollout_attn_pool_bytes.argtypes = [_u32, _u32, _u32]
lib.rollout_attn_pool_bytes.restype = _u64
lib.rollout_attn_write_kv.argtypes = [_vp, _u32, _u32, _vp, _vp, _vp, _vp, _vp, _u32, _u64, _vp]
lib.rollout_attn_workspace_bytes.argtypes = [_u32, _u64, _u32, _u32]
lib.rollout_attn_workspace_bytes.restype = _u64
lib.rollout_attn_plan.argtypes = [_vp, _u32, _u32, _u32, _u32, _vp, _u64, C.POINTER(_u32), C.POINTER(_u32)]
lib.rollout_attn_decode.argtypes = [_vp, _u32, _u32, _u32, _vp, _vp, _u32, _u32, _u32, _u32, _vp, C.c_int, _vp, _vp]
lib.rollout_gemm_workspace_bytes.argtypes = [_u32, _u32, _u32]
lib.rollout_gemm_workspace_bytes.restype = _u64
lib.rollout_gemm_bf16.argtypes = [_vp, _vp, _vp, _u32, _u32, _u32, _vp, _u64, _vp]


lib.rollout_gemm_packed_bytes.argtypes = [_u32, _u32]
lib.rollout_gemm_packed_bytes.restype = _u64
lib.rollout_gemm_pack_weights.argtypes = [_vp, _vp, _u32, _u32, _vp]
lib.rollout_gemm_bf16_static.argtypes = [_vp, _vp, _vp, _u32, _u32, _u32, _vp]
lib.rollout_gemm_static_scratch_bytes.argtypes = []
lib.rollout_gemm_static_scratch_bytes.restype = _u64
lib.rollout_gemm_swiglu_bf16.argtypes = [_vp, _vp, _vp, _u32, _u32, _u32, _vp]
lib.rollout_gemm_kernel_name.argtypes = [_u32, _u32, _u32, _u32, C.c_int]
lib.rollout_gemm_splits.argtypes = [_u32, _u32, _u32]
lib.rollout_gemm_splits.restype = _u32
lib.rollout_gemm_kernel_name.restype = C.c_char_p
lib.rollout_stream_copy.argtypes = [_vp, _vp, _u64, _vp]
lib.rollout_stream_read.argtypes = [_vp, _u64, _vp, _vp]


def rollout_last_error(ctx=None) -> str:
    s = lib.rollout_last_error(ctx)
    return s.decode() if s else ""


def _check(rc: int, ctx=None) -> None:
    if rc != 0:
        raise RolloutError(rc, rollout_last_error(ctx))


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def make_cfg(shape, *, max_slots, max_prompt_len, max_new_tokens, max_seqs, kv_pool_bytes=0, weight_dtype=1,
             weights_on_device=0, eos_mode=0, mode=0, max_staleness=-1, grouped_loading=0, debug_flags=0,
             page_seed=0, device=0, temperature=0.0, sample_seed=0) -> rollout_cfg:
    """Fill a rollout_cfg from a model shape object (fields as in workloads.ModelShape)."""
    c = rollout_cfg()
    for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "qkv_bias"):
        setattr(c, n, int(getattr(shape, n)))
    c.rms_eps, c.rope_theta = float(shape.rms_eps), float(shape.rope_theta)
    c.weight_dtype, c.weights_on_device = weight_dtype, weights_on_device
    c.max_slots, c.page_tokens, c.kv_pool_bytes = max_slots, 16, int(kv_pool_bytes)
    c.max_prompt_len, c.max_new_tokens, c.max_seqs = max_prompt_len, max_new_tokens, max_seqs
    c.eos_id, c.eos_mode, c.mode, c.max_staleness = int(shape.vocab) - 1, eos_mode, mode, max_staleness
    c.grouped_loading, c.debug_flags, c.page_seed, c.device = grouped_loading, debug_flags, page_seed, device
    c.temperature, c.sample_seed = float(temperature), int(sample_seed)
    return c


def rollout_init(weights, cfg: rollout_cfg):
    """weights: numpy array (host blob) or (device_ptr:int, nbytes:int) when cfg.weights_on_device."""
    ctx = _vp()
    if isinstance(weights, tuple):
        ptr, nbytes = weights
        rc = lib.rollout_init(C.byref(ctx), _vp(ptr), nbytes, C.byref(cfg))
    else:
        w = np.ascontiguousarray(weights)
        rc = lib.rollout_init(C.byref(ctx), w.ctypes.data_as(_vp), w.nbytes, C.byref(cfg))
    _check(rc)
    return ctx


def rollout_update_weights(ctx, weights) -> None:
    if isinstance(weights, tuple):
        ptr, nbytes = weights
        _check(lib.rollout_update_weights(ctx, _vp(ptr), nbytes), ctx)
    else:
        w = np.ascontiguousarray(weights)
        _check(lib.rollout_update_weights(ctx, w.ctypes.data_as(_vp), w.nbytes), ctx)


def rollout_submit(ctx, tokens, offsets, target_len) -> int:
    t, o, L = _np(tokens, np.int32), _np(offsets, np.uint32), _np(target_len, np.uint32)
    first = _u64()
    _check(lib.rollout_submit(ctx, t.ctypes.data_as(_vp), o.ctypes.data_as(_vp), L.ctypes.data_as(_vp), len(L),
                              C.byref(first)), ctx)
    return first.value


def rollout_submit_n(ctx, tokens, offsets, target_len, k) -> int:
    t, o, L = _np(tokens, np.int32), _np(offsets, np.uint32), _np(target_len, np.uint32)
    n = len(o) - 1
    if len(L) != n * k:
        raise ValueError("target_len needs one entry per (prompt, response)")
    first = _u64()
    _check(lib.rollout_submit_n(ctx, t.ctypes.data_as(_vp), o.ctypes.data_as(_vp), L.ctypes.data_as(_vp), n, k,
                                C.byref(first)), ctx)
    return first.value


def rollout_step(ctx) -> rollout_step_info:
    info = rollout_step_info()
    _check(lib.rollout_step(ctx, C.byref(info)), ctx)
    return info


def rollout_step_forced(ctx, forced_tok, logits_out: Optional[np.ndarray]) -> rollout_step_info:
    info = rollout_step_info()
    f = _np(forced_tok, np.int32)
    lp = logits_out.ctypes.data_as(_vp) if logits_out is not None else None
    _check(lib.rollout_step_forced(ctx, f.ctypes.data_as(_vp), lp, C.byref(info)), ctx)
    return info


def rollout_harvest(ctx, group_size: int, flags: int = 0, want_logp: bool = True):
    """Returns (n_groups, recs: list[rollout_traj], tokens int32, logp float32 or None)."""
    ng, nr, need = _u32(), _u32(), _u64()
    rc = lib.rollout_harvest(ctx, group_size, flags, None, 0, None, None, 0, C.byref(ng), C.byref(nr), C.byref(need))
    if rc == 0:
        return 0, [], np.zeros(0, np.int32), (np.zeros(0, np.float32) if want_logp else None)
    if rc != -4:
        _check(rc, ctx)
    recs = (rollout_traj * nr.value)()
    toks = np.zeros(max(1, need.value), np.int32)
    logp = np.zeros(max(1, need.value), np.float32) if want_logp else None
    _check(lib.rollout_harvest(ctx, group_size, flags, recs, nr.value, toks.ctypes.data_as(_vp),
                               logp.ctypes.data_as(_vp) if want_logp else None, toks.size, C.byref(ng),
                               C.byref(nr), C.byref(need)), ctx)
    return ng.value, list(recs), toks[:need.value], (logp[:need.value] if want_logp else None)


def rollout_stats(ctx) -> rollout_stats_t:
    s = rollout_stats_t()
    _check(lib.rollout_stats(ctx, C.byref(s)), ctx)
    return s


def rollout_peek(ctx, seq_id: int, cap: int) -> Tuple[np.ndarray, np.ndarray, int, int]:
    toks, logp = np.zeros(max(1, cap), np.int32), np.zeros(max(1, cap), np.float32)
    g, st, sl = _u32(), _u32(), _i32()
    _check(lib.rollout_peek(ctx, seq_id, toks.ctypes.data_as(_vp), logp.ctypes.data_as(_vp), cap, C.byref(g),
                            C.byref(st), C.byref(sl)), ctx)
    return toks[:g.value], logp[:g.value], st.value, sl.value


def rollout_slot_pages(ctx, slot: int, cap: int) -> np.ndarray:
    pages = np.zeros(max(1, cap), np.int32)
    n = _u32()
    _check(lib.rollout_slot_pages(ctx, slot, pages.ctypes.data_as(_vp), cap, C.byref(n)), ctx)
    return pages[:n.value]


def rollout_destroy(ctx) -> None:
    lib.rollout_destroy(ctx)


# ---- standalone kernels: device pointers are plain ints (e.g. torch.Tensor.data_ptr()) -----------------------
def rollout_attn_pool_bytes(n_pages, n_kv_heads, head_dim) -> int:
    return lib.rollout_attn_pool_bytes(n_pages, n_kv_heads, head_dim)


def rollout_attn_write_kv(pool_dev, n_kv_heads, head_dim, k_dev, v_dev, tok_seq_dev, tok_pos_dev, page_table_dev,
                          max_pages, n_tok, stream=0) -> None:
    _check(lib.rollout_attn_write_kv(pool_dev, n_kv_heads, head_dim, k_dev, v_dev, tok_seq_dev, tok_pos_dev,
                                     page_table_dev, max_pages, n_tok, stream))


def rollout_attn_workspace_bytes(n, total_ctx, n_q_heads, head_dim) -> int:
    return lib.rollout_attn_workspace_bytes(n, total_ctx, n_q_heads, head_dim)


def rollout_attn_plan(ctx_len, n_q_heads, n_kv_heads, head_dim, workspace_dev, workspace_bytes) -> Tuple[int, int]:
    """Returns (n_work, chunk_tokens)."""
    L = _np(ctx_len, np.int32)
    nw, ch = _u32(), _u32()
    _check(lib.rollout_attn_plan(L.ctypes.data_as(_vp), len(L), n_q_heads, n_kv_heads, head_dim, workspace_dev,
                                 workspace_bytes, C.byref(nw), C.byref(ch)))
    return nw.value, ch.value


def rollout_attn_decode(pool_dev, n_q_heads, n_kv_heads, head_dim, q_dev, page_table_dev, max_pages, n, n_work,
                        chunk_tokens, out_dev, out_fp32, workspace_dev, stream=0) -> None:
    _check(lib.rollout_attn_decode(pool_dev, n_q_heads, n_kv_heads, head_dim, q_dev, page_table_dev, max_pages, n,
                                   n_work, chunk_tokens, out_dev, int(out_fp32), workspace_dev, stream))


def rollout_gemm_workspace_bytes(M, N, K) -> int:
    return lib.rollout_gemm_workspace_bytes(M, N, K)


def rollout_gemm_bf16(a_dev, w_dev, c_dev, M, N, K, workspace_dev, workspace_bytes, stream=0) -> None:
    _check(lib.rollout_gemm_bf16(a_dev, w_dev, c_dev, M, N, K, workspace_dev, workspace_bytes, stream))


def rollout_stream_copy(src_dev, dst_dev, nbytes, stream=0) -> None:
    _check(lib.rollout_stream_copy(src_dev, dst_dev, nbytes, stream))


def rollout_stream_read(src_dev, nbytes, sink_dev, stream=0) -> None:
    _check(lib.rollout_stream_read(src_dev, nbytes, sink_dev, stream))


def rollout_gemm_packed_bytes(N, K) -> int:
    return lib.rollout_gemm_packed_bytes(N, K)


def rollout_gemm_pack_weights(w_dev, packed_dev, N, K, stream=0) -> None:
    _check(lib.rollout_gemm_pack_weights(w_dev, packed_dev, N, K, stream))


def rollout_gemm_swiglu_bf16(a_dev, w_packed_dev, act_dev, M, F, K, stream=0) -> None:
    _check(lib.rollout_gemm_swiglu_bf16(a_dev, w_packed_dev, act_dev, M, F, K, stream))


def rollout_gemm_kernel_name(M, N, K, splits=0, swiglu=False) -> str:
    return lib.rollout_gemm_kernel_name(M, N, K, splits, int(bool(swiglu))).decode()


def rollout_gemm_splits(M, N, K) -> int:
    return lib.rollout_gemm_splits(M, N, K)


def rollout_gemm_bf16_static(a_dev, w_dev, c_dev, M, N, K, stream=0) -> None:
    _check(lib.rollout_gemm_bf16_static(a_dev, w_dev, c_dev, M, N, K, stream))


def rollout_gemm_static_scratch_bytes() -> int:
    return lib.rollout_gemm_static_scratch_bytes()
