"""ckpt_pack_image_noalloc (the entry point for callers that cannot allocate) against ckpt_pack_image, the
entry point it is a variant of: same image, bit for bit, on two calls in a row on one stream with no
synchronisation in between, the second with a smaller input (the static table still holds the first call's
entries behind the second call's); also against the oracle's data region, and the size limit."""
import numpy as np
import pytest

from oracle import oracle, readback
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness, shards
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _need(descs):
    return sum(-(-d[4] // 4096) * 4096 for d in descs)


def test_two_calls_in_a_row_equal_the_allocating_entry_point():
    print("no-alloc pack image, two calls in a row", flush=True)
    spec = shards.make_shard(5, tiny=True)
    shard = harness.DeviceShard(spec)
    shard.upload_host_values()
    stream = harness.Stream()
    big = shard.descs()                       # 302 fragments at odd offsets: four descriptor batches, hundreds of tiles
    small = big[17:60]                        # the second, smaller input: fewer tiles than the table still holds
    guard = 4096
    out = {}
    for name, descs in (("big", big), ("small", small)):
        n = _need(descs)
        out[name] = (harness.DevBuf(n + 2 * guard), harness.DevBuf(n), n)
        B.proxy_device_fill_async(out[name][0].ptr, 0xEE, n + 2 * guard, stream.handle)
    stream.synchronize()
    # the two calls under test, back to back on one stream, nothing waited for in between
    B.pack_image_noalloc(big, out["big"][0].ptr + guard, out["big"][2], stream.cuda_stream)
    B.pack_image_noalloc(small, out["small"][0].ptr + guard, out["small"][2], stream.cuda_stream)
    stream.synchronize()
    # the existing entry point on the same inputs
    B.pack_image(big, out["big"][1].ptr, out["big"][2], stream.cuda_stream)
    B.pack_image(small, out["small"][1].ptr, out["small"][2], stream.cuda_stream)
    host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
    for name, descs, lo, hi in (("big", big, 0, len(big)), ("small", small, 17, 60)):
        got, ref, n = gu.download(out[name][0]), gu.download(out[name][1]), out[name][2]
        assert np.array_equal(got[guard:guard + n], ref), name
        assert np.all(got[:guard] == 0xEE) and np.all(got[guard + n:] == 0xEE), name     # nothing outside the image
        ots = [(t.name, t.dtype, t.shape, host[k]) for k, t in enumerate(spec.tensors)][lo:hi]
        want = np.frombuffer(oracle.serialize_bytes(ots, 0), dtype=np.uint8)[oracle.header_bytes(ots):]
        assert np.array_equal(ref, want), name                                             # and both equal the oracle's data region
    # a third call after the smaller one, larger again
    B.proxy_device_fill_async(out["big"][0].ptr, 0x33, out["big"][0].nbytes, stream.handle)
    B.pack_image_noalloc(big, out["big"][0].ptr + guard, out["big"][2], stream.cuda_stream)
    stream.synchronize()
    assert np.array_equal(gu.download(out["big"][0])[guard:guard + out["big"][2]], gu.download(out["big"][1]))
    for a, b, _ in out.values():
        a.free(); b.free()
    shard.free()


def test_limit_and_bad_arguments_launch_nothing():
    print("no-alloc pack image, limit", flush=True)
    src = harness.DevBuf(4096)
    n = 131072 + 1                            # one tile more than the static table holds
    dst = harness.DevBuf(n * 4096)
    B.proxy_device_fill_async(dst.ptr, 0x11, 64 << 10, 0)
    descs = [("t", B.CKPT_U8, (1,), src.ptr, 1)] * n
    with pytest.raises(B.CkptError) as e:
        B.pack_image_noalloc(descs, dst.ptr, n * 4096, 0)
    assert e.value.code == B.CKPT_EINVAL and "131072" in e.value.text
    with pytest.raises(B.CkptError) as e:
        B.pack_image_noalloc(descs[:10], dst.ptr, 4096, 0)            # destination too small
    assert e.value.code == B.CKPT_EINVAL
    readback.device_synchronize()
    assert np.all(gu.download(dst, 0, 64 << 10) == 0x11)
    # exactly at the limit it runs (the sources overlap, which is allowed; every tensor is the same byte)
    B.proxy_device_fill_async(src.ptr, 0x7C, 4096, 0)
    B.pack_image_noalloc(descs[:131072], dst.ptr, 131072 * 4096, 0)
    readback.device_synchronize()
    got = gu.download(dst, 0, 131072 * 4096).reshape(131072, 4096)
    assert np.all(got[:, 0] == 0x7C) and not got[:, 1:].any()
    src.free(); dst.free()
