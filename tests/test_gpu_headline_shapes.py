"""Parity of the kernel instantiations the benchmark times: the decode chain with a FULL batch of rows at the real
widths (256 rows of the 8B shape, 64 rows of the 32B shape, and an odd 130), and the projection kernels those row
counts select, each against the oracle / a float64 product.  Every test states which instantiation it reaches
(rollout_gemm_kernel_name goes through the same selection as the launches)."""
import numpy as np
import pytest

import workloads as W
from tests._util import LogitError, flat_prompts, lockstep_teacher_forced, make_engine, make_oracle

pytestmark = pytest.mark.gpu


def _names(R, m, rows):
    qd = m.n_q_heads * m.head_dim
    nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim
    return dict(qkv=R.rollout_gemm_kernel_name(rows, nqkv, m.d_model),
                o=R.rollout_gemm_kernel_name(rows, m.d_model, qd),
                gate_up=R.rollout_gemm_kernel_name(rows, 2 * m.d_ffn, m.d_model, swiglu=True),
                down=R.rollout_gemm_kernel_name(rows, m.d_model, m.d_ffn),
                lm_head=R.rollout_gemm_kernel_name(rows, m.vocab, m.d_model, splits=1))


@pytest.mark.parametrize("name,Q,vocab,expect", [
    # the headline batch: 256 rows, one workgroup per CU for the four layer projections, > 256 workgroups for the LM head
    ("8b", 256, 33024, dict(qkv="k_gemm_bf16_deep<0>", o="k_gemm_bf16_deep<0>", gate_up="k_gemm_bf16_deep<1>",
                            down="k_gemm_bf16_deep<0>", lm_head="k_gemm_bf16<8,0,true>")),
    # a ragged 130 rows: the 256-row kernels with clamped rows
    ("8b", 130, 2048, dict(qkv="k_gemm_bf16_deep<0>", o="k_gemm_bf16_deep<0>", gate_up="k_gemm_bf16_deep<1>",
                           down="k_gemm_bf16_deep<0>", lm_head="k_gemm_bf16_deep<0>")),
    # the 32B batch: 64 rows, group of 5 query heads, QKV bias, 6-way split of the down projection
    ("32b", 64, 2048, dict(qkv="k_gemm_bf16<2,0,true>", o="k_gemm_bf16<2,0,true>", gate_up="k_gemm_bf16<2,1,true>",
                           down="k_gemm_bf16<2,0,true>", lm_head="k_gemm_bf16<2,0,true>")),
])
def test_full_batch_one_layer_slice_teacher_forced(name, Q, vocab, expect):
    """One layer at the real widths with every slot running: prompts of 1-2 tokens, three generated tokens each (one
    from the prefill pass, two from full-batch decode steps), every logits row against the fp32 oracle.  The vocabulary
    is cut down so the oracle stays affordable (33024 columns still give the LM head more than 256 workgroups)."""
    import dataclasses
    import paper_2603_23414_amd as R
    m = dataclasses.replace(W.CONFIGS[name].model.with_layers(1), vocab=vocab)
    assert _names(R, m, Q) == expect
    if name == "32b":
        assert R.rollout_gemm_splits(Q, m.d_model, m.d_ffn) == 6
    blob = W.make_weights(m, 11)
    g = W.rng(12)
    prompts = [g.integers(0, m.vocab - 1, int(k)).astype(np.int32) for k in g.integers(1, 3, Q)]
    L = np.full(Q, 3, np.uint32)
    orc = make_oracle(m, max_slots=Q, max_prompt_len=2, cap=3, weights_blob=blob, dtype=np.float32)
    ctx = make_engine(m, blob, max_slots=Q, max_prompt_len=2, cap=3, max_seqs=Q)
    try:
        toks, offs = flat_prompts(prompts)
        R.rollout_submit(ctx, toks, offs, L)
        orc.submit(prompts, L)
        err = LogitError(0.02 * np.sqrt(m.d_model))
        rows_per_step = []
        lockstep_teacher_forced(R, ctx, orc, Q, m.vocab, Q, err, on_step=lambda io, ig: rows_per_step.append(ig.n_ran))
        assert rows_per_step == [Q, Q, Q] and err.rows == 3 * Q      # steps 2 and 3 are decode steps of Q rows
        err.check(f"{name} widths, {Q} rows")
    finally:
        R.rollout_destroy(ctx)


def _gemm_inputs(M, N, K, seed):
    g = W.rng(seed)
    a = W.f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))
    w = W.f32_to_bf16_bits(g.standard_normal((N, K), dtype=np.float32) * np.float32(0.05))
    return a, w


@pytest.mark.parametrize("M,N,K,kernel", [
    (256, 128256, 128, "k_gemm_bf16<8,0,true>"),     # the 8B LM head's row and column counts (shallow K keeps the check cheap)
    (129, 33024, 256, "k_gemm_bf16<8,0,true>"),
    (256, 33000, 4096, "k_gemm_bf16<8,0,true>"),     # full depth, a column count that is not a tile multiple
    (64, 152064, 5120, "k_gemm_bf16<2,0,true>"),     # the 32B LM head at its batch
    (256, 6144, 4096, "k_gemm_bf16_deep<0>"),        # 8B QKV, 5 splits
    (256, 4096, 14336, "k_gemm_bf16_deep<0>"),       # 8B down, 8 splits
    (64, 5120, 27648, "k_gemm_bf16<2,0,true>"),      # 32B down, 6 splits
])
def test_projection_shapes_of_the_timed_step(M, N, K, kernel):
    import torch
    import paper_2603_23414_amd as R
    assert R.rollout_gemm_kernel_name(M, N, K) == kernel
    a, w = _gemm_inputs(M, N, K, M + N)
    dev = torch.device("cuda:0")
    a_d = torch.from_numpy(a.view(np.int16)).to(dev)
    w_d = torch.from_numpy(w.view(np.int16)).to(dev)
    c_d = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    ws_bytes = R.rollout_gemm_workspace_bytes(M, N, K)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    wp = torch.full((R.rollout_gemm_packed_bytes(N, K) // 2,), 0x7FC0, dtype=torch.int16, device=dev)
    R.rollout_gemm_pack_weights(w_d.data_ptr(), wp.data_ptr(), N, K)
    R.rollout_gemm_bf16(a_d.data_ptr(), wp.data_ptr(), c_d.data_ptr(), M, N, K, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    got = c_d.cpu().numpy()
    af = W.bf16_bits_to_f32(a).astype(np.float64)
    worst = 0.0
    for n0 in range(0, N, 16384):                       # float64 reference in column slabs (bounded host memory)
        ref = af @ W.bf16_bits_to_f32(w[n0:n0 + 16384]).astype(np.float64).T
        worst = max(worst, float(np.abs(got[:, n0:n0 + 16384] - ref).max()))
    # products of bf16 are exact in fp32; only the fp32 accumulation order differs
    assert worst < 1e-4 * np.sqrt(K) * 0.05 + 1e-6, worst


@pytest.mark.parametrize("M,F,K,kernel", [
    (256, 14336, 4096, "k_gemm_bf16_deep<1>"),       # the 8B gate/up projection at the headline batch
    (130, 14336, 4096, "k_gemm_bf16_deep<1>"),
    (200, 1000 * 16, 320, "k_gemm_bf16_deep<1>"),    # short K (5 blocks: shorter than the pipeline is deep), ragged rows
    (256, 48, 64, "k_gemm_bf16_deep<1>"),            # one k block, one partly filled column tile
    (64, 27648, 5120, "k_gemm_bf16<2,1,true>"),      # the 32B gate/up projection at its batch
    (24, 512, 128, "k_gemm_bf16<1,1,true>"),
    (8, 512, 64 * 9, "k_gemm_bf16<1,1,true>"),       # k-block counts that end inside a ring group and inside an activation stage
    (40, 512, 64 * 6, "k_gemm_bf16<2,1,true>"),
    (100, 512, 64 * 7, "k_gemm_bf16<4,1,true>"),
    (200, 512, 64 * 7, "k_gemm_bf16_deep<1>"),
    (700, 14336, 512, "k_gemm_bf16_big<1,3,true>"),  # several row blocks (prefill)
])
def test_swiglu_projection_against_float64(M, F, K, kernel):
    """act = silu(a Wg^T) * (a Wu^T) through the fused epilogue, on the instantiation each batch size selects."""
    import torch
    import paper_2603_23414_amd as R
    assert R.rollout_gemm_kernel_name(M, 2 * F, K, swiglu=True) == kernel
    g = W.rng(M * 3 + F)
    a = W.f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))
    wg = W.f32_to_bf16_bits(g.standard_normal((F, K), dtype=np.float32) * np.float32(0.05))
    wu = W.f32_to_bf16_bits(g.standard_normal((F, K), dtype=np.float32) * np.float32(0.05))
    inter = np.empty((2 * F, K), np.uint16)             # gate and up rows interleaved in blocks of 16
    inter.reshape(F // 16, 2, 16, K)[:, 0] = wg.reshape(F // 16, 16, K)
    inter.reshape(F // 16, 2, 16, K)[:, 1] = wu.reshape(F // 16, 16, K)
    dev = torch.device("cuda:0")
    a_d = torch.from_numpy(a.view(np.int16)).to(dev)
    w_d = torch.from_numpy(inter.view(np.int16)).to(dev)
    wp = torch.full((R.rollout_gemm_packed_bytes(2 * F, K) // 2,), 0x7FC0, dtype=torch.int16, device=dev)
    R.rollout_gemm_pack_weights(w_d.data_ptr(), wp.data_ptr(), 2 * F, K)
    act = torch.full((M, F), -1, dtype=torch.int16, device=dev)        # 0xFFFF = a NaN pattern: unwritten cells show
    R.rollout_gemm_swiglu_bf16(a_d.data_ptr(), wp.data_ptr(), act.data_ptr(), M, F, K)
    torch.cuda.synchronize()
    got = W.bf16_bits_to_f32(act.cpu().numpy().view(np.uint16)).astype(np.float64)
    af = W.bf16_bits_to_f32(a).astype(np.float64)
    gate = af @ W.bf16_bits_to_f32(wg).astype(np.float64).T
    up = af @ W.bf16_bits_to_f32(wu).astype(np.float64).T
    ref = gate / (1.0 + np.exp(-gate)) * up
    assert np.isfinite(got).all()
    # the output is rounded to bf16 (relative 2^-9) after fp32 accumulation and a fast exponential
    tol = np.abs(ref) * 2.0 ** -8 + 1e-4 * np.sqrt(K) * 0.05 * (1.0 + np.abs(up) + np.abs(gate)) + 1e-6
    assert (np.abs(got - ref) <= tol).all(), float(np.abs(got - ref).max())
