"""Full-size parity: workloads 2-5 at their real sizes (94 / 91 / 61 / 40 GB) in the launch
configuration bench.py times (64 MiB chunks, 1 GiB super-chunks, 16 GiB ring, 12 I/O threads, tmpfs
sink). EVERY byte of every file is compared with the oracle: the header, each tensor's bytes at the
oracle's offset and the zero padding behind it. The oracle's input is a device-side clone of the whole
shard taken on the stream at the boundary (with the next update enqueued right behind the window), read
back with the oracle's own blocking copies and fed to its piecewise comparison a few GB at a time, so
the host never holds the shard a second time. After a restore into poisoned memory every tensor is read
back and compared with the same file the same way, and for the fragmented workload every byte between
the fragments must still hold the poison."""
import os
import shutil
import tempfile
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import oracle, readback
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness, shards

pytestmark = pytest.mark.gpu

PAYLOAD = {2: 94_337_818_624, 3: 91_113_953_280, 4: 60_816_752_640}
PIECE_BYTES = 2 << 30      # host bytes per comparison piece
WORKERS = 6                # pieces in flight (each: blocking read-back, then the oracle's comparison)


def _say(msg):
    print(msg, flush=True)


def _clone(shard, stream):
    """Device-side copy of the whole shard, ordered on `stream`. Returns (device address per tensor, buffers)."""
    spec = shard.spec
    if shard.flat:
        bufs = [harness.DevBuf(f.nbytes) for f in shard.flat]
        for b, f in zip(bufs, shard.flat):
            B.proxy_copy_d2d_async(b.ptr, f.ptr, f.nbytes, stream.handle)
        return [bufs[t.buffer].ptr + t.offset for t in spec.tensors], bufs
    bufs = shard.clone_all(stream)
    return [b.ptr for b in bufs], bufs


def _pieces(spec):
    out, first, acc = [], 0, 0
    for k, t in enumerate(spec.tensors):
        acc += t.nbytes
        if acc >= PIECE_BYTES:
            out.append((first, k + 1))
            first, acc = k + 1, 0
    if first < len(spec.tensors):
        out.append((first, len(spec.tensors)))
    return out


def _whole_file_equals(spec, ptrs, it, path, cmp):
    """Every byte of the file at `path` against the oracle fed from device addresses `ptrs`. Returns the
    first differing offset of the lowest piece that differs, or None."""
    def one(piece):
        a, b = piece
        arrays = [readback.d2h(ptrs[k], spec.tensors[k].nbytes) for k in range(a, b)]
        return cmp.compare(it, a, arrays, path)

    readback.device_synchronize()
    with ThreadPoolExecutor(WORKERS) as pool:
        diffs = [d for d in pool.map(one, _pieces(spec)) if d is not None]
    return min(diffs) if diffs else None


def _gaps_hold(shard, byte):
    """Fragmented workload: every byte of the flat buffers that belongs to no tensor still holds `byte`."""
    spec = shard.spec
    for b, f in enumerate(shard.flat):
        whole = readback.d2h(f.ptr, f.nbytes)
        pos = 0
        for t in sorted((t for t in spec.tensors if t.buffer == b), key=lambda t: t.offset):
            if not np.all(whole[pos:t.offset] == byte):
                return False
            pos = t.offset + t.nbytes
        if not np.all(whole[pos:] == byte):
            return False
    return True


def _poison(shard, stream, byte=0xA5):
    for buf in list(shard.own.values()) + shard.flat:
        B.proxy_device_fill_async(buf.ptr, byte, buf.nbytes, stream.handle)


def _config(d, direct_min=0, keep_last=1):
    return B.make_config(out_dir=d, host_ring_bytes=16 << 30, dma_chunk_bytes=256 << 20, pack_superchunk_bytes=1 << 30,
                         n_dma_streams=2, n_io_threads=12, keep_last=keep_last, direct_min_bytes=direct_min)


@pytest.mark.parametrize("config,direct_min", [(2, 0), (3, 0), (4, 0), (5, 0), (5, 1 << 20)])
def test_full_size_snapshot_and_restore(config, direct_min):
    """direct_min > 0: the hybrid path on the fragmented workload (6,606 of its 20,000 tensors, most of
    them at unaligned addresses, go by DMA straight from and to their own memory)."""
    _say(f"full size workload {config} direct_min {direct_min}")
    spec = shards.make_shard(config)
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="dsllm_full_", dir=base)
    shard = harness.DeviceShard(spec)
    ck, bufs = None, []
    try:
        stream = harness.Stream()
        shard.fill_device(stream)
        shard.update(1, stream)
        ck = B.Checkpointer(_config(d, direct_min))
        ck.register_tensors(shard.descs())
        assert (ck.layout()["n_direct_tensors"] > 1000) == (direct_min > 0)
        ots = [(t.name, t.dtype, t.shape, None) for t in spec.tensors]
        cmp = oracle.SpanComparer(ots)
        # the boundary: clone of the whole shard on the stream between update 1 and update 2
        ptrs, bufs = _clone(shard, stream)
        ck.snapshot_async(1, stream.cuda_stream)
        ck.wait_immutable_window_end(stream.cuda_stream)
        shard.update(2, stream)                       # the update right behind the window must not leak into file 1
        _say("  snapshot requested")
        ck.flush(1)
        st = ck.stats(1)
        _say(f"  flushed: d2h {st['data_bytes'] / st['d2h_span_ms'] / 1e6:.1f} GB/s")
        path = ck.file_name(1)
        assert os.path.getsize(path) == oracle.header_bytes(ots) + oracle.data_bytes(ots) == ck.layout()["file_bytes"]
        if config in PAYLOAD:
            assert spec.payload_bytes == PAYLOAD[config]
        assert _whole_file_equals(spec, ptrs, 1, path, cmp) is None
        _say("  every byte of the file equals the oracle's")
        # update 2 did run behind the window: the live state no longer matches the file
        k = min(range(len(ptrs)), key=lambda j: abs(spec.tensors[j].nbytes - (1 << 20)))
        assert not np.array_equal(readback.d2h(shard.ptrs[k], spec.tensors[k].nbytes), readback.d2h(ptrs[k], spec.tensors[k].nbytes))
        # restore file 1 into poisoned memory: every tensor is again what the file holds (= the boundary state)
        _poison(shard, stream)
        assert ck.restore(path, stream.cuda_stream) == 1
        stream.synchronize()
        _say("  restored")
        assert _whole_file_equals(spec, shard.ptrs, 1, path, cmp) is None
        if shard.flat:
            assert _gaps_hold(shard, 0xA5)
        _say("  every restored tensor equals the file; bytes between fragments untouched")
        if config == 5 and direct_min == 0:
            # round trip: a snapshot of the restored state is file 1 again but for the iteration field
            ck.snapshot_async(2, stream.cuda_stream)
            ck.flush(2)
            assert _whole_file_equals(spec, ptrs, 2, ck.file_name(2), cmp) is None
            _say("  re-snapshot of the restored state equals the oracle's file of the boundary state")
    finally:
        if ck is not None:
            ck.destroy()
        for b in bufs:
            b.free()
        shard.free()
        shutil.rmtree(d, ignore_errors=True)


def test_full_size_every_iteration_with_mutation():
    """Workload 5 at full size, three consecutive snapshots with the update mutating every word between
    them and nothing but stream order between the phases; every byte of all three files against the oracle
    on the clone taken at each boundary."""
    _say("full size workload 5, three snapshots in a row")
    spec = shards.make_shard(5)
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="dsllm_full_", dir=base)
    shard = harness.DeviceShard(spec)
    ck, clones = None, {}
    try:
        stream = harness.Stream()
        shard.fill_device(stream)
        gemm = harness.GemmProxy(4096)
        ck = B.Checkpointer(_config(d, keep_last=0))
        ck.register_tensors(shard.descs())
        cmp = oracle.SpanComparer([(t.name, t.dtype, t.shape, None) for t in spec.tensors])
        for it in (1, 2, 3):
            gemm.run(200, stream)                                # forward/backward stand-in (reads nothing of the shard)
            ck.wait_immutable_window_end(stream.cuda_stream)     # before the update
            shard.update(it, stream)
            clones[it] = _clone(shard, stream)
            ck.snapshot_async(it, stream.cuda_stream)
        ck.flush()
        stream.synchronize()
        for it in (1, 2, 3):
            assert _whole_file_equals(spec, clones[it][0], it, ck.file_name(it), cmp) is None, f"iteration {it}"
            _say(f"  file {it} equals the oracle's, every byte")
            os.unlink(ck.file_name(it))
        # the three states really differ (the comparison has something to tell apart)
        a, b = readback.d2h(clones[1][0][7], 4096), readback.d2h(clones[2][0][7], 4096)
        assert not np.array_equal(a, b)
    finally:
        if ck is not None:
            ck.destroy()
        for _, bufs in clones.values():
            for b in bufs:
                b.free()
        shard.free()
        shutil.rmtree(d, ignore_errors=True)
