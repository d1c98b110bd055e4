"""The pack step on its own (ckpt_pack_image) against the oracle: the image it leaves in device memory
must be, byte for byte, the data region of the file the oracle writes for the same tensors."""
import numpy as np
import pytest

from oracle import oracle, readback
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness, shards
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def oracle_data_region(shard, host):
    ots = shard.oracle_tensors(host)
    return np.frombuffer(oracle.serialize_bytes(ots, 0), dtype=np.uint8)[oracle.header_bytes(ots):]


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_image_equals_the_oracles_data_region(config):
    print(f"pack image config {config}", flush=True)
    spec = shards.make_shard(config, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    want = oracle_data_region(shard, [shards.host_values(spec, k) for k in range(len(spec.tensors))])
    guard = 4096
    dst = harness.DevBuf(want.nbytes + 2 * guard)
    B.proxy_device_fill_async(dst.ptr, 0xEE, dst.nbytes, stream.handle)
    B.pack_image(shard.descs(), dst.ptr + guard, want.nbytes, stream.cuda_stream)
    got = gu.download(dst)
    assert np.array_equal(got[guard:-guard], want)
    assert np.all(got[:guard] == 0xEE) and np.all(got[-guard:] == 0xEE)         # nothing written outside the image
    dst.free()
    shard.free()


def test_image_of_edge_sizes_and_every_misalignment():
    """Sizes around every internal boundary (16 B word, 4 KiB unit, 32 KiB tile: whole tiles take the kernel's rolling
    pipeline, shorter ones its group cascade and the masked tail word), each at every byte misalignment 0..15 of the
    source, several tiles and a ragged tail each, more tensors than one descriptor batch holds."""
    sizes = [1, 2, 15, 16, 17, 4095, 4096, 4097, 32767, 32768, 32769, 65535, 65536, 100000, 3 * 32768 + 5, 32768 + 16 * 64 * 15 + 16 * 37 + 3]
    tensors, off = [], 0
    for i, n in enumerate(sizes):
        for m in range(16):
            off = (off + 15) // 16 * 16 + m
            tensors.append(shards.TensorSpec(f"e{i}_{m}", shards.U8, (n,), buffer=0, offset=off, role="raw"))
            off += n
    assert len(tensors) > 96 and all(t.offset % 16 == k % 16 for k, t in enumerate(tensors))
    spec = shards.ShardSpec("edges", 5, tensors, flat_buffers=[(off + 255) // 256 * 256])
    shard = harness.DeviceShard(spec)
    stream = harness.Stream()
    shard.fill_device(stream)
    host = gu.readback_all(shard)
    want = oracle_data_region(shard, host)
    dst = harness.DevBuf(want.nbytes)
    B.pack_image(shard.descs(), dst.ptr, want.nbytes, stream.cuda_stream)
    assert np.array_equal(gu.download(dst), want)
    dst.free()
    shard.free()


def test_bad_arguments_launch_nothing():
    spec = shards.make_shard(1, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    need = sum(-(-t.nbytes // 4096) * 4096 for t in spec.tensors)
    dst = harness.DevBuf(need)
    B.proxy_device_fill_async(dst.ptr, 0x11, need, 0)
    host_arr = np.zeros(64, dtype=np.uint8)
    cases = [(shard.descs(), dst.ptr, need - 4096),                                        # destination too small
             (shard.descs(), dst.ptr + 8, need - 8),                                       # not 16-byte aligned
             ([("h", B.CKPT_U8, (64,), host_arr.ctypes.data, 64)], dst.ptr, need),         # a host pointer
             ([("z", B.CKPT_U8, (0,), dst.ptr, 0)], dst.ptr, need),                        # zero bytes
             ([], dst.ptr, need)]
    for descs, p, nbytes in cases:
        with pytest.raises(B.CkptError) as e:
            B.pack_image(descs, p, nbytes, 0)
        assert e.value.code == B.CKPT_EINVAL
    readback.device_synchronize()
    assert np.all(gu.download(dst) == 0x11)
    dst.free()
    shard.free()
