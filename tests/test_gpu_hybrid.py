"""Parity of the hybrid path (large tensors copied by the DMA engines straight out of, and on
restore into, their own memory; only small ones packed) with the CPU oracle, through the C ABI.
The file format does not know how a byte travelled: the expected files are the same as without
direct copies, bit for bit."""
import os
import shutil
import tempfile

import numpy as np
import pytest

from oracle import oracle
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness, shards
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

SMALL = dict(dma_chunk_bytes=64 << 10, pack_superchunk_bytes=128 << 10, host_ring_bytes=256 << 10)


def _say(msg):
    print(msg, flush=True)


@pytest.fixture
def big_dir():
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="dsllm_", dir=base)
    yield d
    shutil.rmtree(d, ignore_errors=True)


@pytest.mark.parametrize("direct_min", [4096, 65536])
@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_tiny_shard_file_equals_oracle(config, direct_min, tmp_path):
    _say(f"hybrid tiny config {config} direct_min {direct_min}")
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), direct_min_bytes=direct_min, **SMALL))
    ck.register_tensors(shard.descs())
    lay = ck.layout()
    n_big = sum(1 for t in spec.tensors if t.nbytes >= direct_min)
    assert lay["n_direct_tensors"] == n_big and lay["n_chunks"] > 4
    if direct_min == 4096:
        assert n_big > 0
    ck.snapshot_async(3, stream.cuda_stream)
    ck.wait_immutable_window_end(stream.cuda_stream)
    ck.flush(3)
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    assert open(ck.file_name(3), "rb").read() == oracle.serialize_bytes(shard.oracle_tensors(host), 3)
    # restore into poisoned memory: payload back, guard bytes between flat-buffer fragments untouched
    shard.poison(0xA5)
    assert ck.restore(ck.file_name(3), stream.cuda_stream) == 3
    stream.synchronize()
    for k, got in enumerate(gu.readback_all(shard)):
        assert np.array_equal(got, host[k]), spec.tensors[k].name
    if shard.flat:
        used = [np.zeros(n, dtype=bool) for n in spec.flat_buffers]
        for t in spec.tensors:
            used[t.buffer][t.offset:t.offset + t.nbytes] = True
        for f, u in zip(shard.flat, used):
            assert np.all(gu.download(f)[~u] == 0xA5)
    with pytest.raises(B.CkptError):
        ck.set_window_policy(B.CKPT_WINDOW_PACK)        # direct copies read the tensors until the last one has landed
    ck.destroy()


@pytest.mark.parametrize("config", [1, 5])
def test_every_iteration_with_mutation(config, tmp_path):
    """Snapshots every iteration while the update mutates everything, with stream order only: the
    direct copies must start after the boundary and the update must wait for the last of them."""
    _say(f"hybrid every-iteration config {config}")
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    gemm = harness.GemmProxy(1024)
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), direct_min_bytes=16384, **SMALL))
    ck.register_tensors(shard.descs())
    assert 0 < ck.layout()["n_direct_tensors"] < len(spec.tensors)
    clones = {}
    for it in range(1, 7):
        gemm.run(4, stream)
        ck.wait_immutable_window_end(stream.cuda_stream)
        shard.update(it, stream)
        clones[it] = shard.clone_all(stream)
        ck.snapshot_async(it, stream.cuda_stream)
    ck.flush()
    stream.synchronize()
    files = set()
    for it in range(1, 7):
        host = [gu.download(c) for c in clones[it]]
        assert oracle.compare_file(shard.oracle_tensors(host), it, ck.file_name(it)) is None, f"iteration {it}"
        files.add(open(ck.file_name(it), "rb").read())
    assert len(files) == 6
    ck.destroy()


def test_gpt2_full_size_hybrid_equals_plain_and_oracle(big_dir):
    """Workload 1 at full size with the default chunking: the hybrid file, the plain file and the
    oracle's file of the same read-back state are one and the same."""
    _say("hybrid gpt2 full size")
    spec = shards.make_shard(1)
    shard = harness.DeviceShard(spec)
    stream = harness.Stream()
    shard.fill_device(stream)
    stream.synchronize()
    images, names = [], []
    for direct_min in (1 << 20, 0):
        d = os.path.join(big_dir, f"d{direct_min}")
        os.mkdir(d)
        ck = B.Checkpointer(B.make_config(out_dir=d, host_ring_bytes=1 << 30, direct_min_bytes=direct_min))
        ck.register_tensors(shard.descs())
        ck.snapshot_async(9, stream.cuda_stream)
        ck.flush(9)
        names.append(ck.file_name(9))
        images.append(open(names[-1], "rb").read())
        if direct_min:
            lay = ck.layout()
            assert 0 < lay["n_direct_tensors"] < len(spec.tensors) and lay["n_tiles"] < lay["data_bytes"] // lay["tile_bytes"]
            want = gu.readback_all(shard)
            shard.poison(0x5A)
            assert ck.restore(ck.file_name(9), stream.cuda_stream) == 9
            stream.synchronize()
            assert all(np.array_equal(g, w) for g, w in zip(gu.readback_all(shard), want))
        ck.destroy()
    assert images[0] == images[1]
    assert oracle.compare_file(shard.oracle_tensors(gu.readback_all(shard)), 9, names[0]) is None
