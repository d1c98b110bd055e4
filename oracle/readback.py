"""The oracle's own way to device memory: blocking hipMemcpy calls made straight on the HIP runtime
through ctypes. TEST INFRASTRUCTURE ONLY, and independent of the library under test: the bytes the
oracle serializes (read back at an iteration boundary) and the bytes it compares after a restore never
pass through code of libdsllm_ckpt.so.

This is step 2 of the oracle's algorithm (the blocking baseline the paper calls the default engine:
stop, copy every tensor to the host, write): pageable host memory, one blocking copy per tensor, no
streams, no pinned buffers.

One process holds one HIP runtime: the shim binds to the libamdhip64 that is already mapped (the one the
library under test, or PyTorch, brought in) and only otherwise loads the system's.
"""
import ctypes as C
import os

import numpy as np

_H2D, _D2H = 1, 2
_hip = None


def _loaded_runtime():
    try:
        with open("/proc/self/maps") as f:
            for line in f:
                path = line.rsplit(" ", 1)[-1].strip()
                if os.path.basename(path).startswith("libamdhip64.so"):
                    return path
    except OSError:
        pass
    return None


def hip():
    global _hip
    if _hip is None:
        path = _loaded_runtime() or os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib", "libamdhip64.so")
        L = C.CDLL(path)
        L.hipMemcpy.restype = C.c_int
        L.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        L.hipDeviceSynchronize.restype = C.c_int
        L.hipDeviceSynchronize.argtypes = []
        L.hipGetErrorString.restype = C.c_char_p
        L.hipGetErrorString.argtypes = [C.c_int]
        _hip = L
    return _hip


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what}: {hip().hipGetErrorString(rc).decode()}")


def device_synchronize():
    """Everything enqueued on the device so far has run (the oracle's 'stop')."""
    _check(hip().hipDeviceSynchronize(), "hipDeviceSynchronize")


def d2h(dev_ptr, nbytes):
    """nbytes bytes at device address dev_ptr as a fresh uint8 array (blocking, pageable destination)."""
    out = np.empty(int(nbytes), dtype=np.uint8)
    if nbytes:
        _check(hip().hipMemcpy(out.ctypes.data, dev_ptr, int(nbytes), _D2H), "hipMemcpy device to host")
    return out


def h2d(dev_ptr, data):
    """The restore-oracle's last step: host bytes back to device address dev_ptr (blocking)."""
    a = np.ascontiguousarray(data).view(np.uint8).reshape(-1)
    if a.nbytes:
        _check(hip().hipMemcpy(dev_ptr, a.ctypes.data, a.nbytes, _H2D), "hipMemcpy host to device")
