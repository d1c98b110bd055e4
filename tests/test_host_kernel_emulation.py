"""Runs the pack and scatter kernel SOURCE on the CPU, thread by thread, under AddressSanitizer
(tests/emu): every address the kernels compute is bounds-checked against exactly sized buffers and
the results are compared with plain memcpy expectations. No GPU involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.fixture(scope="module")
def emu(tmp_path_factory):
    if not os.path.exists(CLANG):
        pytest.skip("ROCm clang not present")
    exe = str(tmp_path_factory.mktemp("emu") / "emu_pack")
    cmd = [CLANG, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "tests", "emu"), "-o", exe,
           os.path.join(ROOT, "tests", "emu", "emu_pack.cpp"), os.path.join(ROOT, "paper_2406_10707_amd", "csrc", "plan.cpp")]
    subprocess.run(cmd, check=True, cwd=os.path.join(ROOT, "tests", "emu"))
    return exe


@pytest.mark.parametrize("seed,n", [(1, 300), (2, 300), (7, 40), (11, 700)])
def test_pack_and_scatter_stay_in_bounds_and_move_the_right_bytes(emu, seed, n):
    r = subprocess.run([emu, str(seed), str(n)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert r.stdout.startswith("ok seed")
