"""Read-back helpers of the GPU tests: every byte that is handed to the oracle or compared with its
output comes off the device through the oracle's own blocking hipMemcpy shim (oracle/readback.py),
not through the library under test."""
from oracle import readback as rb


def readback(shard, k):
    """Tensor k of a harness.DeviceShard as host bytes."""
    return rb.d2h(shard.ptrs[k], shard.spec.tensors[k].nbytes)


def readback_all(shard):
    rb.device_synchronize()
    return [rb.d2h(p, t.nbytes) for p, t in zip(shard.ptrs, shard.spec.tensors)]


def download(buf, offset=0, nbytes=None):
    """A harness.DevBuf (or a part of it) as host bytes."""
    n = buf.nbytes - offset if nbytes is None else nbytes
    return rb.d2h(buf.ptr + offset, n)
