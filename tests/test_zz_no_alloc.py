"""The projection GEMM's entry point that allocates nothing (split-K partials in the library's static device array)
against the workspace entry point: same kernels, so the outputs must agree bit for bit.  Two calls in a row, the
second with a smaller input, so stale contents of the shared array would show."""
import numpy as np
import pytest

import workloads as W

gpu = pytest.mark.gpu


def test_static_scratch_symbol_is_in_the_device_image_dynamic_symbol_table():
    """hipGetSymbolAddress finds a device variable by name in the code object's dynamic symbol table; a file-scope
    static array only gets there when host code ODR-uses it and nothing (e.g. a `used` attribute) pins its internal
    linkage.  Checked on the built object, no GPU needed."""
    import os
    import shutil
    import subprocess
    import tempfile
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    obj = os.path.join(root, "paper_2603_23414_amd", "_build", "engine.o")
    bundler = "/opt/rocm/llvm/bin/clang-offload-bundler"
    if not (os.path.exists(obj) and os.path.exists(bundler) and shutil.which("objcopy") and shutil.which("readelf")):
        pytest.skip("object file or binutils / offload bundler not available")
    with tempfile.TemporaryDirectory() as d:
        fat, dev = os.path.join(d, "fat.bin"), os.path.join(d, "dev.o")
        subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", obj, fat], check=True)
        subprocess.run([bundler, "--unbundle", "--type=o", f"--input={fat}",
                        "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={dev}"], check=True)
        syms = subprocess.run(["readelf", "--dyn-syms", "-W", dev], check=True, capture_output=True, text=True).stdout
    line = [l for l in syms.splitlines() if l.strip().endswith("scratch")]
    assert len(line) == 1 and "GLOBAL" in line[0] and "OBJECT" in line[0], syms
    assert int(line[0].split()[2], 0) == 32 << 20


def _run_both(R, torch, M, N, K, seed):
    g = W.rng(seed)
    a = W.f32_to_bf16_bits(g.standard_normal((M, K), dtype=np.float32))
    w = W.f32_to_bf16_bits(g.standard_normal((N, K), dtype=np.float32) * np.float32(0.05))
    dev = torch.device("cuda:0")
    a_d = torch.from_numpy(a.view(np.int16)).to(dev)
    w_d = torch.from_numpy(w.view(np.int16)).to(dev)
    wp = torch.zeros(R.rollout_gemm_packed_bytes(N, K) // 2, dtype=torch.int16, device=dev)
    R.rollout_gemm_pack_weights(w_d.data_ptr(), wp.data_ptr(), N, K)
    ws_bytes = R.rollout_gemm_workspace_bytes(M, N, K)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    ref = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    got = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    R.rollout_gemm_bf16(a_d.data_ptr(), wp.data_ptr(), ref.data_ptr(), M, N, K, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    R.rollout_gemm_bf16_static(a_d.data_ptr(), wp.data_ptr(), got.data_ptr(), M, N, K)
    torch.cuda.synchronize()
    ref_h, got_h = ref.cpu().numpy(), got.cpu().numpy()
    assert np.isfinite(got_h).all()
    assert np.array_equal(ref_h, got_h), float(np.abs(ref_h - got_h).max())
    exact = W.bf16_bits_to_f32(a).astype(np.float64) @ W.bf16_bits_to_f32(w).astype(np.float64).T
    assert np.abs(got_h - exact).max() < 1e-4 * np.sqrt(K) * 0.05 + 1e-6


@gpu
def test_static_scratch_gemm_equals_the_workspace_gemm_on_two_calls_in_a_row():
    import torch
    import paper_2603_23414_amd as R
    assert R.rollout_gemm_static_scratch_bytes() == 32 << 20
    assert R.rollout_gemm_splits(256, 4096, 4096) == 8 and R.rollout_gemm_splits(100, 640, 2560) > 1
    _run_both(R, torch, 256, 4096, 4096, 1)     # 8 splits x 256 x 4096 fp32 = the whole 32 MiB
    _run_both(R, torch, 100, 640, 2560, 2)      # smaller, right after: the array still holds the first call's partials
    _run_both(R, torch, 64, 33024, 128, 3)      # one split: no scratch at all


def test_static_scratch_holds_the_partial_sums_of_every_shape():
    """The split rule never launches more workgroups than 256 (splits x column tiles x row blocks), so the partial sums
    of any shape stay within 256 x 256 x 128 fp32 = the array's 32 MiB; the entry point's size check is a second line
    of defence.  Host arithmetic only: no GPU needed."""
    import paper_2603_23414_amd as R
    cap = R.rollout_gemm_static_scratch_bytes()
    g = W.rng(5)
    worst = 0
    shapes = [(256, 4096, 4096), (256, 4096, 14336), (128, 384, 1 << 19), (256, 384, 1 << 19), (8192, 128, 4096),
              (64, 5120, 27648), (257, 2048, 8192), (4096, 384, 4096)]
    shapes += [(int(g.integers(1, 9000)), int(g.integers(1, 30000)), 64 * int(g.integers(1, 600))) for _ in range(3000)]
    for M, N, K in shapes:
        S = R.rollout_gemm_splits(M, N, K)
        assert 1 <= S <= 8
        if S > 1:
            worst = max(worst, S * M * N * 4)
    assert 0 < worst <= cap
    assert R.rollout_gemm_splits(256, 4096, 4096) * 256 * 4096 * 4 == cap       # the O projection at the headline batch fills it


@gpu
def test_static_scratch_gemm_rejects_bad_sizes():
    import torch
    import paper_2603_23414_amd as R
    t = torch.zeros(64, dtype=torch.int16, device="cuda:0")
    with pytest.raises(R.RolloutError) as e:
        R.rollout_gemm_bf16_static(t.data_ptr(), t.data_ptr(), t.data_ptr(), 1, 32, 100)          # K not a multiple of 64
    assert e.value.code == -1
    with pytest.raises(R.RolloutError) as e:
        R.rollout_gemm_bf16_static(t.data_ptr(), t.data_ptr(), t.data_ptr(), 8, 128, 1 << 21)      # beyond the stated maximum
    assert e.value.code == -1 and "too large" in str(e.value)
