"""Host-side launch planning of the projection GEMM (no GPU needed: rollout_gemm_splits / rollout_gemm_kernel_name are
plain host arithmetic in the library): which kernel instantiation and how many K splits each projection of the 8B and
32B shapes gets at the row counts the workloads run, and the invariants the split rule promises."""
import pytest

import workloads as W


def _shapes(m):
    qd = m.n_q_heads * m.head_dim
    nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
    return dict(qkv=(nqkv, m.d_model), o=(m.d_model, qd), down=(m.d_model, m.d_ffn), lm_head=(m.vocab, m.d_model))


@pytest.mark.parametrize("name,rows,kernel,splits", [
    # a full batch of the headline workload: one workgroup per CU on the deep kernel
    ("8b_long", 256, "k_gemm_bf16_deep<0>", dict(qkv=5, o=8, down=8)),
    # the tail drain and the smaller workloads: never more workgroups than CUs, at least 10 k blocks per split
    ("8b_long", 9, "k_gemm_bf16<1,0,true>", dict(qkv=5, o=6, down=8)),
    ("8b_long", 32, "k_gemm_bf16<1,0,true>", dict(qkv=5, o=6, down=8)),
    ("8b", 128, "k_gemm_bf16<4,0,true>", dict(qkv=5, o=6, down=8)),
    ("32b", 64, "k_gemm_bf16<2,0,true>", dict(qkv=4, o=6, down=6)),
])
def test_projection_plan_of_the_workloads(name, rows, kernel, splits):
    import paper_2603_23414_amd as R
    m = W.CONFIGS[name].model
    sh = _shapes(m)
    for proj, want in splits.items():
        N, K = sh[proj]
        assert R.rollout_gemm_splits(rows, N, K) == want, proj
        assert R.rollout_gemm_kernel_name(rows, N, K) == kernel, proj
        tiles = (N + 127) // 128
        assert want * tiles <= 256                      # one workgroup per CU at most
    # the gate/up projection and the LM head are never split (their epilogues are not linear)
    assert R.rollout_gemm_splits(rows, 2 * m.d_ffn, m.d_model) == 1
    assert R.rollout_gemm_splits(rows, m.vocab, m.d_model) == 1
    mi = 1 if rows <= 32 else 2 if rows <= 64 else 4 if rows <= 128 else 8
    gu = R.rollout_gemm_kernel_name(rows, 2 * m.d_ffn, m.d_model, swiglu=True)
    assert gu == ("k_gemm_bf16_deep<1>" if rows > 128 else f"k_gemm_bf16<{mi},1,true>")
    assert R.rollout_gemm_kernel_name(rows, m.vocab, m.d_model, splits=1) == f"k_gemm_bf16<{mi},0,true>"


def test_split_rule_invariants():
    import paper_2603_23414_amd as R
    g = W.rng(77)
    for _ in range(4000):
        M, N, K = int(g.integers(1, 5000)), int(g.integers(1, 40000)), 64 * int(g.integers(1, 500))
        S = R.rollout_gemm_splits(M, N, K)
        nkb = K // 64
        tiles = ((N + 127) // 128) * ((M + 255) // 256)
        assert 1 <= S <= 8 and S <= max(1, nkb // 4)
        if S > 1:
            assert S * tiles <= 256
            per = -(-nkb // S)
            assert (S - 1) * per < nkb                  # no empty split
            if M <= 128:
                assert nkb // S >= 10 or S == 1


def test_prefill_passes_take_the_several_row_block_kernel():
    import paper_2603_23414_amd as R
    m = W.CONFIGS["8b_long"].model
    sh = _shapes(m)
    for proj in ("qkv", "o", "down"):
        N, K = sh[proj]
        assert R.rollout_gemm_kernel_name(4096, N, K).startswith("k_gemm_bf16_big<0,")
        assert R.rollout_gemm_splits(4096, N, K) == 1
    assert R.rollout_gemm_kernel_name(4096, 2 * m.d_ffn, m.d_model, swiglu=True).startswith("k_gemm_bf16_big<1,")
