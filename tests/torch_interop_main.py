"""Run as a program by tests/test_gpu_torch_interop.py (a process of its own: PyTorch has to be imported
before the library, so that the process holds one HIP runtime, PyTorch's).

PyTorch owns the device memory and the stream; the library gets raw pointers and the stream handle.
A few steps of a toy training loop with snapshots in between, files compared with the CPU oracle on
clones taken at each boundary, then a restore into overwritten tensors."""
import sys
import tempfile

import torch  # noqa: E402  (first on purpose)

from oracle import oracle  # noqa: E402
from paper_2406_10707_amd import binding as B  # noqa: E402

DT = {torch.bfloat16: B.CKPT_BF16, torch.float32: B.CKPT_F32}


def as_bytes(t):
    return t.detach().contiguous().flatten().view(torch.uint8).cpu().numpy()


def main():
    dev = torch.device("cuda:0")
    torch.manual_seed(7)
    shapes = [(513, 257), (1000,), (64, 64, 33), (3,), (2048, 1024)]
    state, names = [], []
    for k, shp in enumerate(shapes):
        master = (torch.randn(*shp) * 0.02).to(dev)
        for role, t in (("p_bf16", master.to(torch.bfloat16)), ("master", master), ("m", torch.zeros_like(master)),
                        ("v", torch.zeros_like(master))):
            state.append(t)
            names.append(f"param{k}.{role}")
    descs = [(n, DT[t.dtype], tuple(t.shape), t.data_ptr(), t.numel() * t.element_size()) for n, t in zip(names, state)]
    out_dir = tempfile.mkdtemp(prefix="dsllm_torch_")
    ck = B.Checkpointer(B.make_config(out_dir=out_dir, dma_chunk_bytes=256 << 10, pack_superchunk_bytes=1 << 20, host_ring_bytes=2 << 20))
    ck.register_tensors(descs)
    stream = torch.cuda.Stream()
    a = torch.randn(1024, 1024, device=dev)
    clones = {}
    with torch.cuda.stream(stream):
        for it in range(1, 5):
            b = a @ a                                            # forward/backward stand-in on the same stream
            ck.wait_immutable_window_end(stream.cuda_stream)     # before anything mutates the state
            for k in range(len(shapes)):
                p, master, m, v = state[4 * k:4 * k + 4]
                grad = torch.full_like(master, 1e-3 * it)
                m.mul_(0.9).add_(grad, alpha=0.1)
                v.mul_(0.999).addcmul_(grad, grad, value=0.001)
                master.addcdiv_(m, v.sqrt() + 1e-8, value=-1e-3)
                p.copy_(master)
            clones[it] = [t.clone() for t in state]
            ck.snapshot_async(it, stream.cuda_stream)
            del b
    ck.flush()
    stream.synchronize()
    for it in range(1, 5):
        tensors = [(n, DT[t.dtype], tuple(t.shape), as_bytes(c)) for n, t, c in zip(names, state, clones[it])]
        bad = oracle.compare_file(tensors, it, ck.file_name(it))
        assert bad is None, f"iteration {it}: {bad}"
    with torch.cuda.stream(stream):
        for t in state:
            t.fill_(7.0)
        assert ck.restore(ck.file_name(2), stream.cuda_stream) == 2
    stream.synchronize()
    for t, c in zip(state, clones[2]):
        assert torch.equal(t, c)
    ck.destroy()
    print("torch interop ok:", torch.__version__, "hip", torch.version.hip, flush=True)


if __name__ == "__main__":
    sys.exit(main())
