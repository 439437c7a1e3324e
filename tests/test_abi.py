"""The C-ABI library loads and exports every function include/rollout.h declares (no compute without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "rollout.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(rollout_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    import paper_2603_23414_amd as R
    names = _declared()
    assert {"rollout_init", "rollout_submit", "rollout_step", "rollout_harvest"} <= set(names)
    for n in names:
        assert hasattr(R.lib, n), n
    assert sorted(R.EXPORTS) == names


def test_struct_layouts_match_the_header():
    import paper_2603_23414_amd as R
    assert ctypes.sizeof(R.rollout_cfg) == 136 and ctypes.sizeof(R.rollout_traj) == 40
    assert ctypes.sizeof(R.rollout_step_info) == 72 and ctypes.sizeof(R.rollout_stats_t) == 136
    assert R.rollout_cfg.kv_pool_bytes.offset == 56 and R.rollout_cfg.page_seed.offset == 104


def test_argument_errors_are_reported_without_a_gpu():
    import numpy as np
    import workloads as W
    import paper_2603_23414_amd as R
    m = W.CONFIGS["tiny"].model
    cfg = R.make_cfg(m, max_slots=8, max_prompt_len=16, max_new_tokens=64, max_seqs=8)
    cfg.page_tokens = 8
    try:
        R.rollout_init(np.zeros(4, np.uint16), cfg)
        assert False
    except R.RolloutError as e:
        assert e.code == -1 and "page_tokens" in str(e)
    cfg.page_tokens = 16
    cfg.head_dim = 48
    try:
        R.rollout_init(np.zeros(4, np.uint16), cfg)
        assert False
    except R.RolloutError as e:
        assert e.code == -1
    assert R.rollout_attn_pool_bytes(10, 8, 128) == 10 * 8 * 2 * 16 * 128 * 2
    assert R.rollout_gemm_workspace_bytes(256, 4096, 4096) >= 256 * 4096 * 4
