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
                                             "pack_kernels.hip", "pack_image.hip", "derive_kernels.hip")]]
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


def test_failed_chunk_write_never_yields_a_named_file(emu_engine, tmp_path):
    """One chunk write of a snapshot fails; the caller takes the latched error through a call about another
    iteration; the snapshot's remaining chunks are then written. The file must not get its final name (plain
    files and recycled spares), the snapshot must keep reporting its failure, and the context must go on working."""
    r = subprocess.run([emu_engine, "--failed-chunk", str(tmp_path)], capture_output=True, text=True, timeout=300)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "FAILED" not in out and "ThreadSanitizer" not in out, out[-6000:]
    assert out.count("ok failed chunk") == 2


def test_nothing_is_enqueued_before_the_device_reaches_the_boundary(emu_engine, tmp_path):
    """The caller's host requests a snapshot while its stream still has the whole step to run. Until the device
    reaches the boundary the library must keep its own streams empty (work parked behind an unsignalled event
    slows every kernel launch of the caller on the GPU); afterwards the file is the state at the boundary."""
    r = subprocess.run([emu_engine, "--held-boundary", str(tmp_path)], capture_output=True, text=True, timeout=300)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "FAILED" not in out and "ThreadSanitizer" not in out, out[-6000:]
    assert out.count("ok held boundary") == 2


def _crash_expected(it):
    """The file the oracle writes for iteration `it` of the crash child's shard (tests/emu/emu_engine.cpp: crash_byte)."""
    import numpy as np
    from oracle import oracle
    ts = []
    for k in range(12):
        n = 30000 + 9973 * k
        j = np.arange(n, dtype=np.uint64)
        data = (((j * np.uint64(2654435761) + np.uint64(k * 40503 + it * 97)) >> np.uint64(8)) & np.uint64(0xFF)).astype(np.uint8)
        ts.append((f"t{k}", 4, (n,), data))
    return ts, oracle.serialize_bytes(ts, it)


@pytest.mark.parametrize("variant", [0, 1, 2], ids=["plain", "recycled-spares", "second-tier"])
def test_kill_during_flush_leaves_no_torn_named_file(emu_engine, variant, tmp_path):
    """The engine's process is killed (SIGKILL, by itself, at its k-th file write) at points spread over the
    whole run. Afterwards every file that carries a final name, in either tier, is exactly the oracle's file of
    its iteration; ckpt_find_latest finds the newest of them and the oracle's restore accepts it."""
    import random
    import numpy as np
    from oracle import oracle
    from paper_2406_10707_amd import binding as B
    full = tmp_path / "full"
    full.mkdir()
    r = subprocess.run([emu_engine, "--crash", str(full), str(variant), str(10 ** 9)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "survived with" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
    total = int(r.stdout.split("survived with")[1].split()[0])
    assert total > 40
    rng = random.Random(1000 + variant)
    kills = sorted({1, 2, total // 2, total - 1, total} | {rng.randrange(1, total + 1) for _ in range(5)})
    expected = {it: _crash_expected(it) for it in range(1, 6)}
    died, leftovers, named = 0, 0, 0
    for k in kills:
        d = tmp_path / f"kill{k}"
        d.mkdir()
        r = subprocess.run([emu_engine, "--crash", str(d), str(variant), str(k)], capture_output=True, text=True, timeout=300)
        assert r.returncode == -9, (k, r.returncode, r.stdout[-2000:], r.stderr[-2000:])     # it did end in the middle
        died += 1
        newest = 0
        for tier in (d, d / "tier2"):
            if not tier.is_dir():
                continue
            for f in sorted(os.listdir(tier)):
                if f.endswith(".tmp") or f.startswith(".spare_"):
                    leftovers += 1
                    continue
                if not f.startswith("ckpt_iter"):
                    continue
                it = int(f[len("ckpt_iter"):-len(".dsl")])
                assert (tier / f).read_bytes() == expected[it][1], f"kill at write {k}: {tier / f} is torn"
                named += 1
                if tier == d:
                    newest = max(newest, it)
        if newest:
            it, path = B.find_latest(str(d))
            assert it == newest
            blank = [(n, dt, s, np.zeros(len(x), dtype=np.uint8)) for n, dt, s, x in expected[it][0]]
            assert oracle.restore_file(path, blank) == it
            assert all(np.array_equal(b[3], e[3]) for b, e in zip(blank, expected[it][0]))
        else:
            with pytest.raises(B.CkptError):
                B.find_latest(str(d))
    assert died == len(kills) and leftovers > 0 and named > 0


@pytest.mark.parametrize("which", ["thread", "address"])
def test_derived_tensors_through_the_engine(which, emu_engine, emu_engine_asan, tmp_path):
    """Data reduction through the whole engine on the CPU (ThreadSanitizer, then AddressSanitizer): the
    derivation check and both kernels run from the library's source; snapshots whose pairs hold are version-2
    files, the one with a single wrong bit is a version-1 file, both restore, recycled spares of the wrong size
    are replaced, and a registration without the declaration refuses the version-2 file."""
    exe = emu_engine if which == "thread" else emu_engine_asan
    r = subprocess.run([exe, "--derived", str(tmp_path)], capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "FAILED" not in out, out[-6000:]
    assert not any(w in out for w in ("ThreadSanitizer", "AddressSanitizer", "LeakSanitizer", "runtime error")), out[-6000:]
    assert out.count("ok derived tensors") == 4
