"""Parity of the HIP snapshot/restore path with the CPU oracle, through the C ABI, on a real GPU.
Bit-exact: checkpointing is byte movement, so there is exactly one correct file per (registration,
iteration) and one correct device state after a restore."""
import os
import shutil
import tempfile

import numpy as np
import pytest

from oracle import oracle
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness, shards
from tests import gpu_util as gu
from tests import format_reader as fr

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture
def big_dir():
    """Directory for multi-GB files: tmpfs when there is one."""
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="dsllm_", dir=base)
    yield d
    shutil.rmtree(d, ignore_errors=True)


SMALL = dict(dma_chunk_bytes=64 << 10, pack_superchunk_bytes=128 << 10, host_ring_bytes=256 << 10)


@pytest.mark.parametrize("policy", [B.CKPT_WINDOW_D2H, B.CKPT_WINDOW_PACK])
@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_tiny_shard_file_equals_oracle(config, policy, tmp_path):
    """Small chunks and a ring of 4 slots: many super-chunks, ragged last chunk, ring much smaller
    than the shard (streaming flush and back-pressure are on the path)."""
    _say(f"tiny config {config} policy {policy}")
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), window_policy=policy, **SMALL))
    ck.register_tensors(shard.descs())
    lay = ck.layout()
    assert lay["n_superchunks"] > 2 and lay["n_chunks"] > 4
    ck.snapshot_async(3, stream.cuda_stream)
    ck.wait_immutable_window_end(stream.cuda_stream)
    ck.flush(3)
    data = open(ck.file_name(3), "rb").read()
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    assert data == oracle.serialize_bytes(shard.oracle_tensors(host), 3)           # oracle on the generator's bytes
    assert oracle.compare_file(shard.oracle_tensors(gu.readback_all(shard)), 3, ck.file_name(3)) is None   # and on the read-back
    it, table = fr.parse(data)                                                     # third opinion on the structure
    assert it == 3 and len(table) == len(spec.tensors)
    assert not os.path.exists(ck.file_name(3) + ".tmp")
    st = ck.stats(3)
    assert st["d2h_done"] == 1 and st["committed"] == 1 and st["pack_launches"] == lay["n_superchunks"]
    assert st["payload_bytes"] == spec.payload_bytes and st["d2h_span_ms"] > 0
    ck.destroy()


@pytest.mark.parametrize("mode", ["pwrite", "o_direct", "mmap+fsync"])
def test_sink_modes_write_the_same_file(mode, tmp_path):
    _say(f"sink mode {mode}")
    spec = shards.make_shard(5, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    kw = dict(pwrite=dict(io_mode=B.CKPT_IO_PWRITE), o_direct=dict(o_direct=1, fsync_on_commit=1),
              **{"mmap+fsync": dict(io_mode=B.CKPT_IO_MMAP, fsync_on_commit=1)})[mode]
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), n_io_threads=3, n_dma_streams=1, **SMALL, **kw))
    ck.register_tensors(shard.descs())
    for it in (1, 2):
        ck.snapshot_async(it, stream.cuda_stream)
        ck.flush(it)
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    for it in (1, 2):
        assert open(ck.file_name(it), "rb").read() == oracle.serialize_bytes(shard.oracle_tensors(host), it)
    shard.poison()
    assert ck.restore(ck.file_name(2), stream.cuda_stream) == 2
    stream.synchronize()
    assert all(np.array_equal(g, h) for g, h in zip(gu.readback_all(shard), host))
    ck.destroy()


@pytest.mark.parametrize("io_mode", [B.CKPT_IO_MMAP, B.CKPT_IO_PWRITE])
def test_retention_recycles_files_in_place(io_mode, tmp_path):
    """keep_last=2 with one pre-allocated spare: only the two newest files keep their names, retired
    files are overwritten in place, and every byte of a recycled file is rewritten (the spare starts
    as zeros, later spares hold an older iteration's bytes)."""
    _say(f"retention io_mode {io_mode}")
    spec = shards.make_shard(5, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), keep_last=2, prealloc_files=1, io_mode=io_mode, **SMALL))
    ck.register_tensors(shard.descs())
    assert len([f for f in os.listdir(tmp_path) if f.startswith(".spare_")]) == 1
    want = {}
    for it in range(1, 7):
        shard.update(it, stream)
        ck.snapshot_async(it, stream.cuda_stream)
        ck.wait_immutable_window_end(stream.cuda_stream, host_block=True)
        want[it] = oracle.serialize_bytes(shard.oracle_tensors(gu.readback_all(shard)), it)
        ck.flush(it)
        names = sorted(f for f in os.listdir(tmp_path) if not f.startswith("."))
        assert names == [os.path.basename(ck.file_name(j)) for j in range(max(1, it - 1), it + 1)], names
        assert open(ck.file_name(it), "rb").read() == want[it]
        if it > 1:
            assert open(ck.file_name(it - 1), "rb").read() == want[it - 1]
    assert ck.stats(1)["committed"] == 1          # measurements of retired snapshots stay available
    ck.destroy()
    assert not [f for f in os.listdir(tmp_path) if f.startswith(".spare_")]


@pytest.mark.parametrize("policy,staging", [(B.CKPT_WINDOW_D2H, 0), (B.CKPT_WINDOW_PACK, 0), (B.CKPT_WINDOW_PACK, 64 << 20)],
                         ids=["d2h", "pack-2-staging-slots", "pack-full-staging"])
@pytest.mark.parametrize("config", [1, 5])
def test_every_iteration_with_mutation(config, policy, staging, tmp_path):
    """Snapshot every iteration while the update keeps mutating everything, with nothing but stream
    order between the phases (no host synchronisation inside the loop). The oracle's input for
    iteration i is a device-side clone taken right after update i on the compute stream. Under the
    paper's rule the update waits for the last copy; under policy PACK only for the last pack kernel,
    while the copies drain from staging behind it: with two staging slots (fewer than super-chunks, so
    packs depend on copies) and with staging that holds the whole data region (consecutive snapshots
    reuse it while the previous one's copies may still be reading it)."""
    _say(f"every-iteration config {config} policy {policy} staging {staging}")
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    gemm = harness.GemmProxy(1024)
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), window_policy=policy, dev_staging_bytes=staging, **SMALL))
    ck.register_tensors(shard.descs())
    assert ck.layout()["n_superchunks"] > 2
    clones = {}
    for it in range(1, 7):
        gemm.run(4, stream)                                  # forward/backward stand-in
        ck.wait_immutable_window_end(stream.cuda_stream)     # before the update
        shard.update(it, stream)
        clones[it] = shard.clone_all(stream)
        ck.snapshot_async(it, stream.cuda_stream)
    ck.flush()
    stream.synchronize()
    files = {}
    for it in range(1, 7):
        host = [gu.download(c) for c in clones[it]]
        assert oracle.compare_file(shard.oracle_tensors(host), it, ck.file_name(it)) is None, f"iteration {it}"
        files[it] = open(ck.file_name(it), "rb").read()
    assert len(set(files.values())) == 6          # the update really changed the state every time
    ck.destroy()


def test_update_inside_the_window_is_detected(big_dir):
    """Negative control: if the update runs before the window is closed, the file no longer equals
    the state at the boundary. Shows the parity check can see a late copy."""
    _say("negative control")
    spec = shards.make_shard(1)          # 1.7 GB: copies take tens of milliseconds
    shard = harness.DeviceShard(spec)
    stream = harness.Stream()
    shard.fill_device(stream)
    stream.synchronize()
    ck = B.Checkpointer(B.make_config(out_dir=big_dir, dma_chunk_bytes=16 << 20, pack_superchunk_bytes=64 << 20,
                                      host_ring_bytes=2 << 30))
    ck.register_tensors(shard.descs())
    clones = shard.clone_all(stream)
    ck.snapshot_async(1, stream.cuda_stream)
    shard.update(1, stream)                                  # too early, on purpose
    ck.wait_immutable_window_end(stream.cuda_stream)
    ck.flush(1)
    stream.synchronize()
    host = [gu.download(c) for c in clones]
    assert oracle.compare_file(shard.oracle_tensors(host), 1, ck.file_name(1)) is not None
    ck.destroy()


@pytest.mark.parametrize("config", [1, 5])
def test_restore_and_resnapshot_round_trip(config, tmp_path):
    _say(f"restore config {config}")
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), **SMALL))
    ck.register_tensors(shard.descs())
    ck.snapshot_async(10, stream.cuda_stream)
    ck.flush(10)
    first = open(ck.file_name(10), "rb").read()
    # guard bytes around the flat-buffer fragments must survive a restore untouched
    shard.poison(0xA5)
    assert ck.restore(ck.file_name(10), stream.cuda_stream) == 10
    stream.synchronize()
    for k, got in enumerate(gu.readback_all(shard)):
        assert np.array_equal(got, shards.host_values(spec, k)), spec.tensors[k].name
    if shard.flat:
        used = [np.zeros(n, dtype=bool) for n in spec.flat_buffers]
        for t in spec.tensors:
            used[t.buffer][t.offset:t.offset + t.nbytes] = True
        for f, u in zip(shard.flat, used):
            assert np.all(gu.download(f)[~u] == 0xA5)
    # the oracle's restore agrees (file -> host arrays)
    blank = [np.zeros(t.nbytes, dtype=np.uint8) for t in spec.tensors]
    assert oracle.restore_file(ck.file_name(10), shard.oracle_tensors(blank)) == 10
    for k, b in enumerate(blank):
        assert np.array_equal(b, shards.host_values(spec, k))
    ck.snapshot_async(11, stream.cuda_stream)
    ck.flush(11)
    second = open(ck.file_name(11), "rb").read()
    assert first[:16] == second[:16] and first[24:] == second[24:] and second[16:24] == (11).to_bytes(8, "little")
    ck.destroy()


def test_restore_rejects_bad_files(tmp_path):
    _say("restore errors")
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), **SMALL))
    ck.register_tensors(shard.descs())
    ck.snapshot_async(1, stream.cuda_stream)
    ck.flush(1)
    good = open(ck.file_name(1), "rb").read()
    bad = str(tmp_path / "bad.dsl")

    def expect(code, blob):
        open(bad, "wb").write(blob)
        with pytest.raises(B.CkptError) as e:
            ck.restore(bad, stream.cuda_stream)
        assert e.value.code == code, e.value

    expect(B.CKPT_EFORMAT, good[:-4096])                         # truncated
    expect(B.CKPT_EFORMAT, b"NOTACKPT" + good[8:])               # magic
    expect(B.CKPT_EFORMAT, good[:100])                           # shorter than a header unit
    renamed = bytearray(good); renamed[66] ^= 1                  # first tensor's name
    expect(B.CKPT_EMISMATCH, bytes(renamed))
    with pytest.raises(B.CkptError) as e:
        ck.restore(str(tmp_path / "missing.dsl"), stream.cuda_stream)
    assert e.value.code == B.CKPT_EIO
    # a file of another registration
    other = shards.make_shard(2, tiny=True)
    oshard = harness.DeviceShard(other)
    oshard.upload_host_values()
    ck2 = B.Checkpointer(B.make_config(out_dir=str(tmp_path / "."), **SMALL))
    ck2.register_tensors(oshard.descs())
    with pytest.raises(B.CkptError) as e:
        ck2.restore(ck.file_name(1), stream.cuda_stream)
    assert e.value.code == B.CKPT_EMISMATCH
    # after all those failures the context still works
    shard.poison()
    assert ck.restore(ck.file_name(1), stream.cuda_stream) == 1
    stream.synchronize()
    assert all(np.array_equal(g, shards.host_values(spec, k)) for k, g in enumerate(gu.readback_all(shard)))
    ck.snapshot_async(2, stream.cuda_stream)
    ck.flush(2)
    assert open(ck.file_name(2), "rb").read()[24:] == good[24:]
    ck.destroy(); ck2.destroy()


def test_call_order_and_argument_errors(tmp_path):
    _say("state errors")
    with pytest.raises(B.CkptError) as e:
        B.Checkpointer(B.make_config(out_dir=str(tmp_path / "nope")))
    assert e.value.code == B.CKPT_EIO
    with pytest.raises(B.CkptError) as e:
        B.Checkpointer(B.make_config(out_dir=str(tmp_path), device=99))
    assert e.value.code == B.CKPT_EINVAL
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), **SMALL))
    with pytest.raises(B.CkptError) as e:
        ck.snapshot_async(1, stream.cuda_stream)
    assert e.value.code == B.CKPT_ESTATE                         # nothing registered
    host_arr = np.zeros(64, dtype=np.uint8)
    with pytest.raises(B.CkptError) as e:
        ck.register_tensors([("h", B.CKPT_U8, (64,), host_arr.ctypes.data, 64)])
    assert e.value.code == B.CKPT_EINVAL                         # not device memory
    ck.register_tensors(shard.descs())
    with pytest.raises(B.CkptError) as e:
        ck.register_tensors(shard.descs())
    assert e.value.code == B.CKPT_ESTATE
    ck.wait_immutable_window_end(stream.cuda_stream)             # no pending snapshot: no-op
    ck.snapshot_async(1, stream.cuda_stream)
    with pytest.raises(B.CkptError) as e:
        ck.snapshot_async(2, stream.cuda_stream)                 # window of 1 never closed
    assert e.value.code == B.CKPT_ESTATE
    ck.wait_immutable_window_end(stream.cuda_stream, host_block=True)
    ck.snapshot_async(2, stream.cuda_stream)
    with pytest.raises(B.CkptError) as e:
        ck.flush(99)
    assert e.value.code == B.CKPT_EINVAL
    ck.flush()
    assert os.path.exists(ck.file_name(1)) and os.path.exists(ck.file_name(2))
    ck.destroy()


def test_io_error_is_latched_and_reported(tmp_path):
    """The output directory disappears: the flush threads cannot create the file; the error comes
    back from ckpt_flush, the context stays usable."""
    _say("io error")
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    out = tmp_path / "out"
    out.mkdir()
    ck = B.Checkpointer(B.make_config(out_dir=str(out), **SMALL))
    ck.register_tensors(shard.descs())
    shutil.rmtree(out)
    ck.snapshot_async(1, stream.cuda_stream)
    with pytest.raises(B.CkptError) as e:
        ck.flush(1)
    assert e.value.code == B.CKPT_EIO
    out.mkdir()
    ck.snapshot_async(2, stream.cuda_stream)
    ck.flush(2)
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    assert open(ck.file_name(2), "rb").read() == oracle.serialize_bytes(shard.oracle_tensors(host), 2)
    ck.destroy()


def test_default_stream_and_default_config(big_dir):
    """The null stream as compute stream, library defaults for every size (64 MiB chunks, 1 GiB
    super-chunks): config 1 at full size, whole file compared by the oracle's streaming comparison."""
    _say("config 1 full size, default config")
    spec = shards.make_shard(1)
    shard = harness.DeviceShard(spec)
    shard.fill_device(harness.NullStream())
    ck = B.Checkpointer(B.make_config(out_dir=big_dir))
    ck.register_tensors(shard.descs())
    shard.update(1, harness.NullStream())
    ck.snapshot_async(1, 0)
    ck.wait_immutable_window_end(0, host_block=True)
    host = gu.readback_all(shard)
    ck.flush(1)
    assert os.path.getsize(ck.file_name(1)) == ck.layout()["file_bytes"] == 1_742_157_312 + 600_576 + ck.layout()["header_bytes"]
    assert oracle.compare_file(shard.oracle_tensors(host), 1, ck.file_name(1)) is None
    st = ck.stats(1)
    assert ck.init_probe() > 5.0 and st["init_d2h_gbps"] == ck.init_probe()      # the timed copy of ckpt_init: a plausible link rate
    assert st["host_window_wait_ms"] > 0 and st["format_version"] == 1 and st["verify_ms"] == -1
    ck.destroy()


def test_edge_sizes_and_a_tensor_beyond_4_gib(big_dir):
    """Sizes around every internal boundary (16 B word, 4 KiB unit, 32 KiB tile), a one-byte tensor, a
    scalar, and one tensor larger than 4 GiB (offsets and tile counts beyond 32 bits), all carved at odd
    offsets out of one flat buffer. Whole file compared by the oracle's streaming comparison."""
    _say("edge sizes")
    sizes = [1, 2, 15, 16, 17, 4095, 4096, 4097, 32767, 32768, 32769, 65535, (4 << 30) + 4097 + 3]
    tensors, off = [], 3
    for i, n in enumerate(sizes):
        tensors.append(shards.TensorSpec(f"edge{i}_{n}", shards.U8, (n,), buffer=0, offset=off, role="raw"))
        off += n + (i % 7) + 1
    tensors.append(shards.TensorSpec("scalar", shards.I64, (), buffer=0, offset=(off + 7) // 8 * 8, role="raw"))
    off = tensors[-1].offset + 8
    spec = shards.ShardSpec("edges", 99, tensors, flat_buffers=[(off + 255) // 256 * 256])
    shard = harness.DeviceShard(spec)
    stream = harness.Stream()
    shard.fill_device(stream)                      # seeded words over the whole flat buffer
    stream.synchronize()
    ck = B.Checkpointer(B.make_config(out_dir=big_dir, host_ring_bytes=1 << 30, dma_chunk_bytes=32 << 20,
                                      pack_superchunk_bytes=512 << 20, n_io_threads=8))
    ck.register_tensors(shard.descs())
    lay = ck.layout()
    assert lay["n_superchunks"] >= 9 and lay["data_bytes"] > (4 << 30)
    ck.snapshot_async(7, stream.cuda_stream)
    ck.wait_immutable_window_end(stream.cuda_stream)
    host = gu.readback_all(shard)
    ck.flush(7)
    assert oracle.compare_file(shard.oracle_tensors(host), 7, ck.file_name(7)) is None
    whole = gu.download(shard.flat[0])
    shard.poison(0x5A)
    assert ck.restore(ck.file_name(7), stream.cuda_stream) == 7
    stream.synchronize()
    after = gu.download(shard.flat[0])
    used = np.zeros(spec.flat_buffers[0], dtype=bool)
    for t in tensors:
        used[t.offset:t.offset + t.nbytes] = True
    assert np.array_equal(after[used], whole[used]) and np.all(after[~used] == 0x5A)
    ck.destroy()
    shard.free()
