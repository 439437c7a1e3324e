"""The C ABI used from plain C: tests/c/example.c is compiled as strict C99 against include/rollout.h, linked with
librollout.so and run as a program of its own (no Python in the loop, no torch)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIBDIR = os.path.join(ROOT, "paper_2603_23414_amd")


def _build(tmp_path):
    exe = str(tmp_path / "example_c")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "example.c"), "-L", LIBDIR, "-lrollout", "-lm", f"-Wl,-rpath,{LIBDIR}", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def test_header_is_plain_c_and_the_program_links(tmp_path):
    import torch
    exe = _build(tmp_path)
    if not torch.cuda.is_available():
        # no CPU fallback: without a GPU the very first call reports a device error and the program gives up
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        assert r.returncode == 1 and "rollout_init -> -5" in r.stderr, (r.returncode, r.stderr)


@pytest.mark.gpu
def test_c_program_runs_a_whole_job(tmp_path):
    exe = _build(tmp_path)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert r.stdout.startswith("ok: 8 rollouts in 3 groups"), r.stdout
