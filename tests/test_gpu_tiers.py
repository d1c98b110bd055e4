"""The second storage tier on a real GPU: files committed to the fast directory are copied on to a
slower one in the background; what arrives there is bit-exact against the CPU oracle, the newest
snapshot always arrives, and a restore can be fed from either tier."""
import os

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


@pytest.mark.parametrize("keep_last,io_mode,o_direct,mode", [(1, B.CKPT_IO_MMAP, 0, B.CKPT_TIER2_NEWEST), (0, B.CKPT_IO_PWRITE, 0, B.CKPT_TIER2_NEWEST),
                                                             (2, B.CKPT_IO_MMAP, 1, B.CKPT_TIER2_NEWEST), (1, B.CKPT_IO_MMAP, 1, B.CKPT_TIER2_EVERY),
                                                             (0, B.CKPT_IO_PWRITE, 0, B.CKPT_TIER2_EVERY)])
def test_second_tier_receives_the_newest_snapshot(keep_last, io_mode, o_direct, mode, tmp_path):
    """mode NEWEST: the newest snapshot always arrives, older ones are copied or skipped; mode EVERY: all arrive."""
    _say(f"second tier keep_last {keep_last} io_mode {io_mode} o_direct {o_direct} mode {mode}")
    fast, slow = tmp_path / "fast", tmp_path / "slow"
    fast.mkdir()
    slow.mkdir()
    spec = shards.make_shard(5, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(fast), keep_last=keep_last, prealloc_files=1 if keep_last else 0, io_mode=io_mode, **SMALL))
    ck.register_tensors(shard.descs())
    with pytest.raises(B.CkptError):
        ck.wait_second_tier()                               # none enabled
    ck.enable_second_tier(str(slow), n_threads=3, o_direct=o_direct, keep_last=2, mode=mode)
    clones = {}
    n = 8
    for it in range(1, n + 1):
        ck.wait_immutable_window_end(stream.cuda_stream)
        shard.update(it, stream)
        clones[it] = shard.clone_all(stream)
        ck.snapshot_async(it, stream.cuda_stream)
    ck.flush()
    ck.wait_second_tier()
    stream.synchronize()
    states = {it: ck.stats(it)["tier2_state"] for it in range(1, n + 1)}
    assert states[n] == B.CKPT_TIER2_DONE, states
    assert set(states.values()) <= {B.CKPT_TIER2_DONE, B.CKPT_TIER2_SKIPPED}, states
    if mode == B.CKPT_TIER2_EVERY:
        assert set(states.values()) == {B.CKPT_TIER2_DONE}, states
    done = [it for it, s in states.items() if s == B.CKPT_TIER2_DONE]
    present = sorted(f for f in os.listdir(slow))
    assert present == [os.path.basename(ck.second_tier_file_name(it)) for it in done[-2:]], (present, states)   # second-tier retention: 2
    for it in done[-2:]:
        host = [gu.download(c) for c in clones[it]]
        assert oracle.compare_file(shard.oracle_tensors(host), it, ck.second_tier_file_name(it)) is None, f"iteration {it}"
        assert ck.stats(it)["host_tier2_ms"] > 0
    for it in range(1, n + 1):
        if states[it] == B.CKPT_TIER2_SKIPPED:
            with pytest.raises(B.CkptError) as e:
                ck.wait_second_tier(it)
            assert e.value.code == B.CKPT_ESTATE
        else:
            ck.wait_second_tier(it)
    # the fast tier's own retention is untouched by the second tier
    names = sorted(f for f in os.listdir(fast) if not f.startswith("."))
    keep = range(n - keep_last + 1, n + 1) if keep_last else range(1, n + 1)
    assert names == [os.path.basename(ck.file_name(it)) for it in keep]
    # restore from the slower tier
    want = [gu.download(c) for c in clones[n]]
    shard.poison(0xA5)
    assert ck.restore(ck.second_tier_file_name(n), stream.cuda_stream) == n
    stream.synchronize()
    assert all(np.array_equal(g, w) for g, w in zip(gu.readback_all(shard), want))
    ck.destroy()


def test_second_tier_error_is_latched(tmp_path):
    """The slower directory disappears: the snapshot still commits in the fast tier, the failure of the
    copy is reported by ckpt_wait_second_tier, apart from the snapshot path's own errors."""
    _say("second tier error path")
    fast, slow = tmp_path / "fast", tmp_path / "slow"
    fast.mkdir()
    slow.mkdir()
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(fast), **SMALL))
    ck.register_tensors(shard.descs())
    ck.enable_second_tier(str(slow))
    with pytest.raises(B.CkptError):
        ck.enable_second_tier(str(slow))
    os.rmdir(slow)
    ck.snapshot_async(1, stream.cuda_stream)
    ck.flush(1)                                   # the fast tier is fine and does not report the other tier's trouble
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    assert open(ck.file_name(1), "rb").read() == oracle.serialize_bytes(shard.oracle_tensors(host), 1)
    with pytest.raises(B.CkptError) as e:
        ck.wait_second_tier(1)
    assert e.value.code == B.CKPT_EIO and "second tier" in e.value.text
    assert ck.stats(1)["tier2_state"] == B.CKPT_TIER2_FAILED
    ck.wait_second_tier()                         # reported once
    ck.snapshot_async(2, stream.cuda_stream)      # the snapshot path goes on
    ck.flush(2)
    with pytest.raises(B.CkptError):
        ck.destroy()                              # the second failure comes back from destroy


def test_restart_from_the_newest_whole_file(tmp_path):
    """A restart: the context that wrote the checkpoints is gone, a new one registers the same tensors,
    finds the newest whole file (a torn newer file is passed over) and restores it."""
    _say("restart via find_latest")
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    ck = B.Checkpointer(B.make_config(out_dir=str(tmp_path), **SMALL))
    ck.register_tensors(shard.descs())
    states = {}
    for it in (10, 20, 30):
        ck.wait_immutable_window_end(stream.cuda_stream)
        shard.update(it, stream)
        ck.snapshot_async(it, stream.cuda_stream)
        ck.wait_immutable_window_end(stream.cuda_stream, host_block=True)
        states[it] = gu.readback_all(shard)
    ck.flush()
    newest = ck.file_name(30)
    ck.destroy()
    assert B.find_latest(str(tmp_path)) == (30, newest)
    with open(newest, "r+b") as f:            # the newest file is torn (as after a crash in mid-write without the rename protocol)
        f.truncate(os.path.getsize(newest) // 2)
    it, path = B.find_latest(str(tmp_path))
    assert it == 20
    shard.poison(0xA5)
    ck2 = B.Checkpointer(B.make_config(out_dir=str(tmp_path), **SMALL))
    ck2.register_tensors(shard.descs())
    assert ck2.restore(path, stream.cuda_stream) == 20
    stream.synchronize()
    assert all(np.array_equal(g, w) for g, w in zip(gu.readback_all(shard), states[20]))
    with pytest.raises(B.CkptError) as e:
        ck2.restore(newest, stream.cuda_stream)
    assert e.value.code == B.CKPT_EFORMAT
    ck2.destroy()
