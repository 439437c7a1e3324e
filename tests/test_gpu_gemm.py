"""Parity of the bf16 MFMA projection GEMM (C ABI: rollout_gemm_bf16) against a float64 matmul."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (8, 384, 128), (33, 512, 512), (128, 6144, 4096), (256, 4096, 4096),
                                   (250, 1000, 1024), (300, 256, 14336 // 7), (700, 640, 256), (64, 128256 // 4, 128),
                                   (333, 384, 128), (333, 128, 128), (2, 256, 128), (437, 256, 64), (4096, 128, 128),
                                   (256, 4096, 192)])
def test_gemm_matches_float64(M, N, K):
    _check_gemm(M, N, K)


@pytest.mark.parametrize("seed", range(24))
def test_gemm_random_shapes(seed):
    """Row counts on both sides of every kernel variant's limits (32, 64, 128, 256 rows; several row blocks), column
    counts that are not tile multiples, depths from one k block to a few hundred."""
    g = W.rng(900 + seed)
    M = int(g.choice([int(g.integers(1, 33)), int(g.integers(33, 129)), int(g.integers(129, 257)), int(g.integers(257, 1100))]))
    N = int(g.choice([int(g.integers(1, 300)), 32 * int(g.integers(1, 40)), int(g.integers(300, 3000))]))
    K = 64 * int(g.choice([1, 2, 3, int(g.integers(4, 40)), int(g.integers(40, 130))]))
    _check_gemm(M, N, K)


@pytest.mark.parametrize("M,N,kernel", [
    (8, 384, "k_gemm_bf16<1,0,true>"), (40, 384, "k_gemm_bf16<2,0,true>"), (100, 384, "k_gemm_bf16<4,0,true>"),
    (200, 384, "k_gemm_bf16_deep<0>"), (600, 384, "k_gemm_bf16_deep<0>"), (256, 33024, "k_gemm_bf16<8,0,true>"),
    (600, 12000, "k_gemm_bf16_big<0,"),
])
def test_gemm_every_loop_tail(M, N, kernel):
    """The k loops run full groups of ring-depth blocks (and, for the activation tile, stages of several blocks) without
    a test between the blocks, then the last one to three blocks behind theirs, and prefetches past the last block go
    against an empty buffer descriptor: every k-block count from 1 to 13 (all remainders of 3- and 4-deep rings, stages
    ending inside a group, launches shorter than the prologue) on each kernel variant."""
    import paper_2603_23414_amd as R
    for nkb in range(1, 14):
        K = 64 * nkb
        assert R.rollout_gemm_kernel_name(M, N, K).startswith(kernel), (nkb, R.rollout_gemm_kernel_name(M, N, K))
        _check_gemm(M, N, K)


def _check_gemm(M, N, K):
    import torch
    import paper_2603_23414_amd as R
    g = W.rng(M * 7 + N)
    a = W.f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))
    w = W.f32_to_bf16_bits(g.standard_normal((N, K), dtype=np.float32) * np.float32(0.05))
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
    got = c_d.cpu().numpy().astype(np.float64)
    ref = W.bf16_bits_to_f32(a).astype(np.float64) @ W.bf16_bits_to_f32(w).astype(np.float64).T
    # products of bf16 are exact in fp32; only the fp32 accumulation order differs: ~K^0.5 * 2^-24 * |terms|
    scale = np.sqrt(K) * 0.05
    assert np.abs(got - ref).max() < 1e-4 * scale + 1e-6


def test_gemm_rejects_sizes_whose_offsets_would_not_fit_32_bits():
    import torch
    import paper_2603_23414_amd as R
    t = torch.zeros(64, dtype=torch.int16, device="cuda:0")
    c = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    for M, N, K in [(1, 32, (1 << 20) + 64), ((1 << 24) + 1, 32, 64), (1, (1 << 24) + 1, 64), (1, 32, 100)]:
        with pytest.raises(R.RolloutError) as e:
            R.rollout_gemm_bf16(t.data_ptr(), t.data_ptr(), c.data_ptr(), M, N, K, t.data_ptr(), 0)
        assert e.value.code == -1      # EINVAL
