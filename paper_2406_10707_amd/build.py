"""Builds libdsllm_ckpt.so (HIP kernels + engine + C ABI) in-tree for gfx950 with hipcc."""
import hashlib
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsllm_ckpt.so")
SOURCES = ["plan.cpp", "engine.cpp", "submit.cpp", "io_threads.cpp", "restore.cpp", "second_tier.cpp", "pack_kernels.hip",
           "pack_image.hip", "derive_kernels.hip", "proxy_kernels.hip"]
HEADERS = ["plan.hpp", "engine_internal.hpp", "tile_batch.hpp", "kernel_util.hpp", os.path.join("..", "..", "include", "ckpt.h"), os.path.join("..", "..", "include", "ckpt_proxy.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result",
    # packed fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


STAMP = LIB + ".stamp"


def _fingerprint() -> str:
    """Hash of everything the library is built from (sources, headers, flags): file times do not survive
    a copy of the tree to another machine, contents do."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for s in SOURCES + HEADERS:
        with open(os.path.join(CSRC, s), "rb") as f:
            h.update(s.encode() + b"\0" + f.read())
    return h.hexdigest()


def _stale() -> bool:
    """True when there is no library, or the one that is there was built from other sources than today's."""
    if not os.path.exists(LIB) or not os.path.exists(STAMP):
        return True
    with open(STAMP) as f:
        return f.read().strip() != _fingerprint()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    fingerprint = _fingerprint()     # of the sources as they are now, before the minutes of compiling
    objs = []
    for s in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc, "-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj] + HIPCC_FLAGS
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs + ["-lpthread"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    with open(STAMP, "w") as f:
        f.write(fingerprint + "\n")
    return LIB


def ensure_built() -> str:
    """For tests, the smoke run and the benchmark: load what is built, but never a library that was built
    from other sources than the ones in the tree. A missing or outdated library is rebuilt here (and said so
    on stderr), so a run can never silently measure yesterday's kernels. The binding itself never builds."""
    if not _stale():
        return LIB
    print("[build] libdsllm_ckpt.so is %s: building" % ("missing" if not os.path.exists(LIB) else "older than its sources"),
          file=sys.stderr, flush=True)
    return build(force=True)


if __name__ == "__main__":
    print(build(verbose=True))
