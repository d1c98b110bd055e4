"""Builds libdsllm_ckpt.so (HIP kernels + engine + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsllm_ckpt.so")
SOURCES = ["plan.cpp", "engine.cpp", "submit.cpp", "io_threads.cpp", "restore.cpp", "second_tier.cpp", "pack_kernels.hip",
           "proxy_kernels.hip"]
HEADERS = ["plan.hpp", "engine_internal.hpp", os.path.join("..", "..", "include", "ckpt.h"), os.path.join("..", "..", "include", "ckpt_proxy.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result",
    # packed fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
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
    return LIB


def ensure_built() -> str:
    """For tests, the smoke run and the benchmark: compile only when no library is there at all (they never
    rebuild one that exists; after a change to a source, build explicitly). The binding itself never builds."""
    return LIB if os.path.exists(LIB) else build(force=True)


if __name__ == "__main__":
    print(build(verbose=True))
