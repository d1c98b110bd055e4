"""Device-side scaffolding shared by the GPU tests, the smoke check and the benchmark: puts a
synthetic shard (shards.py) into HBM, drives the proxy kernels, reads tensors back with blocking
copies. Everything goes through the C ABI of libdsllm_ckpt.so (proxy_* for memory, streams and
events); no other GPU package is involved, so the process runs on the system HIP runtime."""
import numpy as np

from . import binding as B
from . import shards


class Stream:
    """A non-blocking HIP stream of default priority, created by the library."""

    def __init__(self):
        self.handle = B.proxy_stream_create()

    @property
    def cuda_stream(self):          # same attribute name as a framework stream object
        return self.handle

    def synchronize(self):
        B.proxy_stream_synchronize(self.handle)


class NullStream:
    handle = 0
    cuda_stream = 0

    def synchronize(self):
        B.proxy_stream_synchronize(0)


class Event:
    def __init__(self):
        self.handle = B.proxy_event_create()

    def record(self, stream):
        B.proxy_event_record(self.handle, stream.handle)

    def synchronize(self):
        B.proxy_event_synchronize(self.handle)

    def elapsed_time(self, later):
        return B.proxy_event_elapsed_ms(self.handle, later.handle)

    def __del__(self):
        try:
            B.proxy_event_destroy(self.handle)
        except Exception:
            pass


class DevBuf:
    """One device allocation (hipMalloc)."""

    def __init__(self, nbytes):
        self.nbytes = int(nbytes)
        self.ptr = B.proxy_device_alloc(max(self.nbytes, 1))

    def upload(self, arr):
        a = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
        assert a.nbytes == self.nbytes
        B.proxy_copy_h2d(self.ptr, a.ctypes.data, a.nbytes)

    def download(self, offset=0, nbytes=None):
        n = self.nbytes - offset if nbytes is None else nbytes
        out = np.empty(n, dtype=np.uint8)
        if n:
            B.proxy_copy_d2h(out.ctypes.data, self.ptr + offset, n)
        return out

    def free(self):
        if self.ptr:
            B.proxy_device_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def make_compute_stream():
    return Stream()


def synchronize():
    B.proxy_device_synchronize()


class DeviceShard:
    """The tensors of a ShardSpec in device memory.

    Configs 1-4: every state tensor is an allocation of its own (naturally >= 256-byte aligned).
    Config 5: a few flat buffers; tensors are sub-ranges at element-size-aligned offsets."""

    def __init__(self, spec: shards.ShardSpec):
        self.spec = spec
        self.flat = [DevBuf(n) for n in spec.flat_buffers]
        self.own = {}          # tensor index -> DevBuf
        self.ptrs = []
        for k, t in enumerate(spec.tensors):
            if t.buffer >= 0:
                self.ptrs.append(self.flat[t.buffer].ptr + t.offset)
            else:
                self.own[k] = DevBuf(t.nbytes)
                self.ptrs.append(self.own[k].ptr)

    def free(self):
        for b in list(self.own.values()) + self.flat:
            b.free()

    # ---- description for ckpt_register_tensors
    def descs(self):
        return [(t.name, t.dtype, t.shape, p, t.nbytes) for t, p in zip(self.spec.tensors, self.ptrs)]

    # ---- contents
    def upload_host_values(self):
        """Small shards: values come from shards.host_values (includes special bit patterns)."""
        for k, t in enumerate(self.spec.tensors):
            v = np.ascontiguousarray(shards.host_values(self.spec, k))
            B.proxy_copy_h2d(self.ptrs[k], v.ctypes.data, t.nbytes)
        synchronize()

    def poison(self, byte=0xA5):
        for b in list(self.own.values()) + self.flat:
            B.proxy_device_fill_async(b.ptr, byte, b.nbytes, 0)
        synchronize()

    def _param_groups(self):
        ts = self.spec.tensors
        k = 0
        while k < len(ts):
            if ts[k].role == "p_bf16":
                yield k // 4, k
                k += 4
            else:
                k += 1

    def fill_device(self, stream):
        """Seeded fill on the device (proxy_fill_state / proxy_fill_words)."""
        s = stream.handle
        for i, f in enumerate(self.flat):
            B.proxy_fill_words(f.ptr, f.nbytes // 4, self.spec.seed + 1000 * i, s)
        for pid, k in self._param_groups():
            n = self.spec.tensors[k].numel
            B.proxy_fill_state(self.ptrs[k], self.ptrs[k + 1], self.ptrs[k + 2], self.ptrs[k + 3], n, self.spec.seed, pid, s)

    def update(self, step, stream):
        """The mutating phase: Adam on every parameter's four tensors, or the word mutator on flat buffers."""
        s = stream.handle
        for f in self.flat:
            B.proxy_mutate_words(f.ptr, f.nbytes // 4, step, s)
        for pid, k in self._param_groups():
            n = self.spec.tensors[k].numel
            B.proxy_adam_step(self.ptrs[k], self.ptrs[k + 1], self.ptrs[k + 2], self.ptrs[k + 3], n, self.spec.seed, pid, step, s)

    # ---- blocking read-back (what the oracle is fed)
    def readback(self, k) -> np.ndarray:
        n = self.spec.tensors[k].nbytes
        out = np.empty(n, dtype=np.uint8)
        B.proxy_copy_d2h(out.ctypes.data, self.ptrs[k], n)
        return out

    def readback_all(self):
        synchronize()
        return [self.readback(k) for k in range(len(self.ptrs))]

    def clone_all(self, stream):
        """Device-side copies of every tensor, ordered on `stream` (they capture the state at this
        point of the stream without stopping it). Returns DevBufs to be downloaded later."""
        out = []
        for t, p in zip(self.spec.tensors, self.ptrs):
            b = DevBuf(t.nbytes)
            B.proxy_copy_d2d_async(b.ptr, p, t.nbytes, stream.handle)
            out.append(b)
        return out

    def oracle_tensors(self, host_arrays):
        return [(t.name, t.dtype, t.shape, a) for t, a in zip(self.spec.tensors, host_arrays)]


class GemmProxy:
    """The forward/backward stand-in: repeated bf16 GEMMs of a fixed size on the matrix cores."""

    def __init__(self, n=4096, seed=1):
        g = np.random.default_rng(seed)
        self.n = n
        self.host_a = shards.f32_to_bf16_rne((g.standard_normal((n, n), dtype=np.float32) * np.float32(0.05)))
        self.host_b = shards.f32_to_bf16_rne((g.standard_normal((n, n), dtype=np.float32) * np.float32(0.05)))
        self.a, self.b, self.c = DevBuf(2 * n * n), DevBuf(2 * n * n), DevBuf(2 * n * n)
        self.a.upload(self.host_a)
        self.b.upload(self.host_b)
        self.flops_per_launch = 2.0 * n * n * n

    def run(self, launches, stream):
        s = stream.handle
        for _ in range(launches):
            B.proxy_gemm_bf16(self.a.ptr, self.b.ptr, self.c.ptr, self.n, self.n, self.n, s)

    def calibrate(self, target_ms, stream):
        """Number of launches whose total duration is about target_ms, and the measured ms per launch."""
        self.run(3, stream)
        e0, e1 = Event(), Event()
        e0.record(stream)
        self.run(10, stream)
        e1.record(stream)
        e1.synchronize()
        per = e0.elapsed_time(e1) / 10.0
        return max(1, int(round(target_ms / per))), per
