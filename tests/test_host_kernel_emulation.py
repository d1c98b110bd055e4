"""Runs the library's SOURCE on the CPU (tests/emu). The pack and scatter kernels run thread by thread
under AddressSanitizer: every address they compute is bounds-checked against exactly sized buffers
and the results are compared with plain memcpy expectations. The whole engine runs against a model of
streams and events under ThreadSanitizer: files, restore, retention and error paths are checked, and
any pair of accesses the engine's event graph leaves unordered is reported as a race. No GPU involved."""
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


def _build_emu_engine(tmp_path_factory, sanitizer):
    if not os.path.exists(CLANG):
        pytest.skip("ROCm clang not present")
    exe = str(tmp_path_factory.mktemp("emu") / "emu_engine")
    csrc = os.path.join(ROOT, "paper_2406_10707_amd", "csrc")
    cmd = [CLANG, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=" + sanitizer, "-fno-omit-frame-pointer", "-pthread",
           "-I", os.path.join(ROOT, "tests", "emu"), "-o", exe, os.path.join(ROOT, "tests", "emu", "emu_engine.cpp"),
           *[os.path.join(csrc, f) for f in ("engine.cpp", "submit.cpp", "io_threads.cpp", "restore.cpp", "second_tier.cpp", "plan.cpp",
                                             "pack_kernels.hip")]]
    subprocess.run(cmd, check=True, cwd=os.path.join(ROOT, "tests", "emu"))
    return exe


@pytest.fixture(scope="module")
def emu_engine(tmp_path_factory):
    return _build_emu_engine(tmp_path_factory, "thread")


@pytest.fixture(scope="module")
def emu_engine_asan(tmp_path_factory):
    return _build_emu_engine(tmp_path_factory, "address,undefined")


def _run_scenarios(exe, seed, tmp_path, forbidden):
    r = subprocess.run([exe, str(tmp_path), str(seed)], capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "FAILED" not in out and not any(w in out for w in forbidden), out[-6000:]
    assert out.count("ok policy") == 12 and out.count("snapshots copied") == 3


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_engine_event_graph_under_thread_sanitizer(emu_engine, seed, tmp_path):
    _run_scenarios(emu_engine, seed, tmp_path, ["ThreadSanitizer"])


def test_engine_host_memory_under_address_sanitizer(emu_engine_asan, tmp_path):
    """The same scenarios with AddressSanitizer, LeakSanitizer and UBSan: every buffer the engine's host code
    indexes (header, capture buffers, ring slots, mappings) and every object it frees."""
    _run_scenarios(emu_engine_asan, 4, tmp_path, ["AddressSanitizer", "LeakSanitizer", "runtime error"])
