"""Parity of the ragged paged GQA decode-attention kernel (C ABI: rollout_attn_*) against the oracle."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _run_case(lens, Hq, Hkv, d, seed, out_fp32=True, poison=True, repeat=1):
    import torch
    import paper_2603_23414_amd as R
    from oracle import paged_decode_attention
    lens = np.asarray(lens, np.int32)
    n = len(lens)
    q, k, v, offs = W.make_attention_case(lens, Hq, Hkv, d, seed)
    table, n_pool = W.make_page_table(lens, 16, seed + 1)
    dev = torch.device("cuda:0")
    pool_bytes = R.rollout_attn_pool_bytes(n_pool, Hkv, d)
    pool = torch.empty(pool_bytes // 2, dtype=torch.int16, device=dev)
    pool.fill_(0x7FC0 if poison else 0)          # bf16 NaN in every byte that is never written
    tok_seq = np.repeat(np.arange(n, dtype=np.int32), lens)
    tok_pos = np.concatenate([np.arange(L, dtype=np.int32) for L in lens])
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    k_d, v_d = t(k.view(np.int16)), t(v.view(np.int16))
    ts_d, tp_d, tab_d = t(tok_seq), t(tok_pos), t(np.maximum(table, 0).astype(np.int32))
    R.rollout_attn_write_kv(pool.data_ptr(), Hkv, d, k_d.data_ptr(), v_d.data_ptr(), ts_d.data_ptr(), tp_d.data_ptr(),
                            tab_d.data_ptr(), table.shape[1], int(lens.sum()))
    ws_bytes = R.rollout_attn_workspace_bytes(n, int(lens.sum()), Hq, d)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    n_work, chunk = R.rollout_attn_plan(lens, Hq, Hkv, d, ws.data_ptr(), ws_bytes)
    # one work item (workgroup per kv head) per four consecutive chunks of a row
    assert chunk % 64 == 0 and 128 <= chunk <= 1024 and n_work == int(((((lens + chunk - 1) // chunk) + 3) // 4).sum())
    q_d = t(q.view(np.int16))
    out = torch.full((n, Hq, d), float("nan"), dtype=torch.float32 if out_fp32 else torch.bfloat16, device=dev)
    first = None
    for it in range(repeat):     # the same plan serves every launch: the arrival counters must be back at zero each time
        out.fill_(float("nan"))
        R.rollout_attn_decode(pool.data_ptr(), Hq, Hkv, d, q_d.data_ptr(), tab_d.data_ptr(), table.shape[1], n, n_work,
                              chunk, out.data_ptr(), out_fp32, ws.data_ptr())
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().astype(np.float64)
        if first is None:
            first = got
        assert np.array_equal(first, got)          # and the merge order is fixed: bit-identical results
    # oracle on the same bf16-exact operands, contiguous pools built by the oracle's own addressing
    kp = np.zeros((n_pool, 16, Hkv, d))
    vp = np.zeros((n_pool, 16, Hkv, d))
    kf, vf = W.bf16_bits_to_f32(k).astype(np.float64), W.bf16_bits_to_f32(v).astype(np.float64)
    for i, L in enumerate(lens):
        for p in range((L + 15) // 16):
            a, b = p * 16, min(L, p * 16 + 16)
            kp[table[i, p], : b - a] = kf[offs[i] + a: offs[i] + b]
            vp[table[i, p], : b - a] = vf[offs[i] + a: offs[i] + b]
    ref = paged_decode_attention(W.bf16_bits_to_f32(q).astype(np.float64), kp, vp, table, lens)
    return got, ref


# fp32 softmax + fp32 accumulation of bf16 operands; probabilities are rounded to bf16 before the value product:
# |err| <= 2^-9 * max|v| * (small factor).  With N(0,1) values (max ~4.5) 2e-2 is the same bar as the logits gate.
TOL = 2e-2


@pytest.mark.parametrize("Hq,Hkv,d", [(32, 8, 128), (40, 8, 128), (4, 4, 32), (8, 8, 128), (8, 2, 32), (10, 2, 32)])
def test_ragged_lengths_span_pages_chunks_and_tails(Hq, Hkv, d):
    lens = [1, 2, 15, 16, 17, 63, 64, 65, 255, 256, 257, 300, 511, 513, 777, 1024, 1500]
    got, ref = _run_case(lens, Hq, Hkv, d, seed=10 + Hq)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max(axis=(1, 2))
    assert err.max() < TOL, err
    # length-1 context returns v (bf16-exact, so exactly)
    assert np.abs(got[0] - ref[0]).max() < 1e-6


def test_bf16_output_and_single_sequence():
    got, ref = _run_case([1000], 32, 8, 128, seed=3, out_fp32=False)
    assert np.abs(got - ref).max() < TOL + 2e-2   # + one bf16 rounding of the output


def test_long_tail_mix_like_the_benchmark_case():
    a = W.ATTN_CASE
    lens = W.make_kv_lengths(24, a["median"], a["sigma"], a["cap"], seed=11)
    lens[0] = 16384
    lens[1] = 1
    got, ref = _run_case(lens, 32, 8, 128, seed=12)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() < TOL


@pytest.mark.parametrize("Hq,Hkv,d", [(32, 8, 128), (40, 8, 128), (8, 2, 32)])
def test_group_boundaries_of_the_workgroup_merge(Hq, Hkv, d):
    """A workgroup merges four token spans in LDS and rows longer than four chunks are merged by their last-arriving workgroup:
    contexts just below, at and above one, four, five, eight and sixteen chunks of the smallest chunk size (128),
    whose last spans hold anything from a single token to a full tile."""
    lens = [127, 128, 129, 255, 256, 257, 511, 512, 513, 575, 576, 577, 641, 1023, 1024, 1025, 2047, 2048, 2049, 4097, 5000]
    got, ref = _run_case(lens, Hq, Hkv, d, seed=20 + Hq)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max(axis=(1, 2)).max() < TOL


def test_repeated_launches_on_one_plan_and_many_groups_per_row():
    """Rows of 1 to 30 work items (the last-arriving workgroup of a row merges the others' partial results), launched
    four times from one plan."""
    lens = [16000, 9000, 4097, 2049, 1537, 1536, 1535, 600, 3, 12000, 513]
    got, ref = _run_case(lens, 32, 8, 128, seed=77, repeat=4)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() < TOL
    got, ref = _run_case(lens[:6], 10, 2, 32, seed=78, repeat=3)
    assert np.abs(got - ref).max() < TOL


@pytest.mark.parametrize("seed", range(12))
def test_random_length_mixes_and_head_layouts(seed):
    """Row counts, head layouts and length mixes drawn at random: all-short batches, a single row, lengths that sit on
    page / tile / chunk boundaries, and one row far longer than the rest."""
    g = W.rng(300 + seed)
    d = int(g.choice([32, 128]))
    group = int(g.choice([1, 4, 5]))
    Hkv = int(g.integers(1, 5))
    n = int(g.integers(1, 33))
    kind = int(g.integers(0, 4))
    if kind == 0:
        lens = g.integers(1, 40, n)
    elif kind == 1:
        lens = np.minimum(6000, np.ceil(g.lognormal(np.log(300), 1.2, n))).astype(np.int64)
    elif kind == 2:
        lens = g.choice([1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 511, 512, 513, 1023, 1024, 1025], n)
    else:
        lens = g.integers(1, 200, n)
        lens[int(g.integers(0, n))] = int(g.integers(3000, 9000))
    got, ref = _run_case(np.maximum(1, lens), Hkv * group, Hkv, d, seed=400 + seed, out_fp32=bool(g.integers(0, 2)))
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() < TOL + 2e-2    # + one bf16 rounding when the output is bf16
