"""The snapshot path in the setting where PyTorch owns the device memory and the stream, and with it the HIP
runtime of the process (PyTorch ships its own). Run as a program, in a process of its own:

    python -m paper_2406_10707_amd.torch_runtime_probe [--config 1] [--snapshots 4]

PyTorch is imported first, so the library binds to PyTorch's runtime. A GPT-2-small-shaped shard (workload 1)
lives in torch tensors; a matmul loop on a torch stream stands in for forward/backward; snapshots are requested
on that stream. Prints one JSON line: the rate of the timed copy ckpt_init makes, the pinned-copy peak measured
with torch, device-to-host rate and pack kernel rate of the snapshots. Whether the copies ran on the copy
engines or as kernels on the compute units shows in a profiler trace of this program (memory-copy records versus
copy kernels); in-process it shows as the copy rate and as the pack kernel's rate collapsing."""
import argparse
import json
import os
import shutil
import sys
import tempfile

import torch  # first on purpose: one process, one HIP runtime, here PyTorch's

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2406_10707_amd import binding as B  # noqa: E402
from paper_2406_10707_amd import shards  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--snapshots", type=int, default=4)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    spec = shards.make_shard(args.config)
    dt = {shards.BF16: torch.bfloat16, shards.F32: torch.float32}
    state = [torch.empty(t.shape if t.shape else (), dtype=dt[t.dtype], device=dev).normal_(0, 0.02) for t in spec.tensors]
    descs = [(t.name, t.dtype, t.shape, x.data_ptr(), x.numel() * x.element_size()) for t, x in zip(spec.tensors, state)]
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    out_dir = tempfile.mkdtemp(prefix="dsllm_torch_", dir=base)
    stream = torch.cuda.Stream()
    try:
        # pinned-copy peak as PyTorch itself reaches it
        n = 1 << 30
        d = torch.empty(n, dtype=torch.uint8, device=dev)
        h = torch.empty(n, dtype=torch.uint8, pin_memory=True)
        peak = 0.0
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(stream):
                e0.record(stream)
                h.copy_(d, non_blocking=True)
                e1.record(stream)
            e1.synchronize()
            peak = max(peak, n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del d, h
        data_upper = spec.payload_bytes + 4096 * len(spec.tensors)
        # a shard of under 2 GB that is checkpointed every step: 64 MiB copies (the pipeline starts sooner) and a ring of twice
        # the shard, so that a snapshot's copies never wait for the previous snapshot's slots to be written out
        chunk = 64 << 20
        ring = min(16 << 30, 2 * (-(-data_upper // chunk) * chunk))
        ck = B.Checkpointer(B.make_config(out_dir=out_dir, host_ring_bytes=ring, dma_chunk_bytes=chunk, n_io_threads=6, keep_last=1,
                                          prealloc_files=2))
        ck.register_tensors(descs)
        a = torch.randn(4096, 4096, device=dev, dtype=torch.bfloat16)
        f32 = [x for x in state if x.dtype == torch.float32]
        for it in range(1, args.snapshots + 2):
            with torch.cuda.stream(stream):
                for _ in range(40):                                # forward/backward stand-in
                    torch.mm(a, a)
                ck.wait_immutable_window_end(stream.cuda_stream)
                torch._foreach_add_(f32, 1e-3)                     # the update: mutates the state
                ck.snapshot_async(it, stream.cuda_stream)
        ck.flush()
        stream.synchronize()
        rows = [ck.stats(it) for it in range(2, args.snapshots + 2)]   # the first snapshot warms everything up
        lay = ck.layout()
        pack_bytes = lay["payload_bytes"] + lay["data_bytes"]
        d2h = sum(r["data_bytes"] for r in rows) / (sum(r["d2h_span_ms"] for r in rows) * 1e-3) / 1e9
        pack = pack_bytes * len(rows) / (sum(r["pack_ms_sum"] for r in rows) * 1e-3) / 1e9
        init = ck.init_probe()
        ck.destroy()
        print(json.dumps({
            "workload": spec.name, "torch": torch.__version__, "hip_of_torch": torch.version.hip, "snapshots": len(rows),
            "init_probe_d2h_gbps": round(init, 2), "torch_pinned_copy_peak_d2h_gbps": round(peak, 2),
            "snapshot_d2h_gbps": round(d2h, 2), "d2h_frac_of_torch_peak": round(d2h / peak, 4),
            "pack_kernel_gbps": round(pack, 1), "pack_frac_of_hbm_peak": round(pack / 8000.0, 4),
            "copy_path_suspected": "copy engines" if init > 40.0 and pack > 2000.0 else "kernels on the compute units"}), flush=True)
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)


if __name__ == "__main__":
    main()
