"""Device-side scaffolding shared by the GPU tests, the smoke check and the benchmark: puts a
synthetic shard (shards.py) into HBM with PyTorch as the allocator, drives the proxy kernels, and
reads tensors back with blocking copies. PyTorch is used for device memory, streams and events
only; every byte the checkpoint path moves is moved by libdsllm_ckpt.so."""
import numpy as np
import torch

from . import binding as B
from . import shards


def make_compute_stream(device="cuda:0"):
    """A torch stream object around a stream created by the library (proxy_stream_create), so that it
    does not come from PyTorch's pool of 32+ streams, which would spread over all hardware queues and
    end up sharing one with the checkpoint library's own streams."""
    torch.cuda.set_device(device)
    torch.cuda.current_stream().synchronize()      # HIP is initialised and the null stream has its queue
    return torch.cuda.ExternalStream(B.proxy_stream_create(), device=device)


class DeviceShard:
    """The tensors of a ShardSpec in device memory.

    Configs 1-4: every state tensor is an allocation of its own (naturally >= 256-byte aligned).
    Config 5: a few flat uint8 buffers; tensors are sub-ranges at element-size-aligned offsets."""

    def __init__(self, spec: shards.ShardSpec, device="cuda:0"):
        self.spec = spec
        self.device = torch.device(device)
        self.flat = [torch.empty(n, dtype=torch.uint8, device=self.device) for n in spec.flat_buffers]
        self.bufs = []      # one uint8 view per tensor
        for t in spec.tensors:
            if t.buffer >= 0:
                self.bufs.append(self.flat[t.buffer][t.offset:t.offset + t.nbytes])
            else:
                self.bufs.append(torch.empty(t.nbytes, dtype=torch.uint8, device=self.device))

    # ---- description for ckpt_register_tensors
    def descs(self):
        return [(t.name, t.dtype, t.shape, b.data_ptr(), t.nbytes) for t, b in zip(self.spec.tensors, self.bufs)]

    # ---- contents
    def upload_host_values(self):
        """Small shards: values come from shards.host_values (includes special bit patterns)."""
        for k, b in enumerate(self.bufs):
            b.copy_(torch.from_numpy(shards.host_values(self.spec, k).copy()))
        torch.cuda.synchronize(self.device)

    def poison(self, byte=0xA5):
        for f in self.flat:
            f.fill_(byte)
        for t, b in zip(self.spec.tensors, self.bufs):
            if t.buffer < 0:
                b.fill_(byte)
        torch.cuda.synchronize(self.device)

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
        """Seeded fill on the device (proxy_fill_state / proxy_fill_words); `stream` is a torch stream."""
        s = stream.cuda_stream
        if self.flat:
            for i, f in enumerate(self.flat):
                B.proxy_fill_words(f.data_ptr(), f.numel() // 4, self.spec.seed + 1000 * i, s)
        for pid, k in self._param_groups():
            n = self.spec.tensors[k].numel
            B.proxy_fill_state(self.bufs[k].data_ptr(), self.bufs[k + 1].data_ptr(), self.bufs[k + 2].data_ptr(),
                               self.bufs[k + 3].data_ptr(), n, self.spec.seed, pid, s)

    def update(self, step, stream):
        """The mutating phase: Adam on every parameter's four tensors, or the word mutator on flat buffers."""
        s = stream.cuda_stream
        if self.flat:
            for f in self.flat:
                B.proxy_mutate_words(f.data_ptr(), f.numel() // 4, step, s)
        for pid, k in self._param_groups():
            n = self.spec.tensors[k].numel
            B.proxy_adam_step(self.bufs[k].data_ptr(), self.bufs[k + 1].data_ptr(), self.bufs[k + 2].data_ptr(),
                              self.bufs[k + 3].data_ptr(), n, self.spec.seed, pid, step, s)

    # ---- blocking read-back (what the oracle is fed)
    def readback(self, k) -> np.ndarray:
        return self.bufs[k].cpu().numpy()

    def readback_all(self):
        torch.cuda.synchronize(self.device)
        return [self.readback(k) for k in range(len(self.bufs))]

    def clone_all(self):
        """Device-side copies of every tensor, ordered on the current torch stream."""
        return [b.clone() for b in self.bufs]

    def oracle_tensors(self, host_arrays):
        return [(t.name, t.dtype, t.shape, a) for t, a in zip(self.spec.tensors, host_arrays)]


class GemmProxy:
    """The forward/backward stand-in: repeated bf16 GEMMs of a fixed size on the matrix cores."""

    def __init__(self, n=4096, device="cuda:0", seed=1):
        g = torch.Generator(device="cpu").manual_seed(seed)
        self.n = n
        self.a = (torch.randn(n, n, generator=g) * 0.05).to(torch.bfloat16).to(device)
        self.b = (torch.randn(n, n, generator=g) * 0.05).to(torch.bfloat16).to(device)
        self.c = torch.empty(n, n, dtype=torch.bfloat16, device=device)
        self.flops_per_launch = 2.0 * n * n * n

    def run(self, launches, stream):
        s = stream.cuda_stream
        for _ in range(launches):
            B.proxy_gemm_bf16(self.a.data_ptr(), self.b.data_ptr(), self.c.data_ptr(), self.n, self.n, self.n, s)

    def calibrate(self, target_ms, stream):
        """Number of launches whose total duration is about target_ms, and the measured ms per launch."""
        with torch.cuda.stream(stream):
            self.run(3, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            self.run(10, stream)
            e1.record(stream)
        e1.synchronize()
        per = e0.elapsed_time(e1) / 10.0
        return max(1, int(round(target_ms / per))), per
