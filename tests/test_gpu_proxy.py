"""Parity of the proxy kernels (GEMM on the matrix cores, Adam step, seeded fills, copy) with the
numpy/float64 oracle, through the C ABI. Integer work is compared bit for bit; float32 results
within bounds derived from the arithmetic (stated at each check)."""
import numpy as np
import pytest

from oracle import proxy_oracle as po
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import harness
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _dl(buf, dtype):
    return gu.download(buf).view(dtype)


@pytest.mark.parametrize("numel", [1, 3, 1000, 65537, (1 << 20) + 5])
def test_fill_state_matches_generator(numel):
    print(f"fill_state numel {numel}", flush=True)
    p, w, m, v = harness.DevBuf(2 * numel), harness.DevBuf(4 * numel), harness.DevBuf(4 * numel), harness.DevBuf(4 * numel)
    B.proxy_fill_state(p.ptr, w.ptr, m.ptr, v.ptr, numel, 77, 5, 0)
    harness.synchronize()
    gw, gm, gv, gp = _dl(w, np.float32), _dl(m, np.float32), _dl(v, np.float32), _dl(p, np.uint16)
    ow, om, ov = po.fill_state(numel, 77, 5)
    # float32 log/sqrt/cos and float32 uniforms against float64: a few ulp of the result plus the
    # cancellation of cos near its zeros, bounded by 1e-5 relative to the scale 0.02
    assert np.max(np.abs(gw - ow)) < 0.02 * 2e-5 * 6 and np.max(np.abs(gm - om)) < 0.02 * 2e-5 * 6
    assert np.max(np.abs(gv - ov)) < 1e-6 * 36 * 1e-4
    assert np.array_equal(gp, po.bf16_bits(gw))          # the bf16 copy is exactly the rounding of the device's master


@pytest.mark.parametrize("numel", [1, 2, 7, 4096, 100003])
def test_adam_step_matches_float64(numel):
    print(f"adam numel {numel}", flush=True)
    p, w, m, v = harness.DevBuf(2 * numel + 8), harness.DevBuf(4 * numel), harness.DevBuf(4 * numel), harness.DevBuf(4 * numel)
    B.proxy_fill_state(p.ptr, w.ptr, m.ptr, v.ptr, numel, 3, 1, 0)
    harness.synchronize()
    w0, m0, v0 = (_dl(x, np.float32).astype(np.float64) for x in (w, m, v))
    for step in (1, 2, 50):
        B.proxy_adam_step(p.ptr, w.ptr, m.ptr, v.ptr, numel, 3, 1, step, 0)
        harness.synchronize()
        gw, gm, gv = (_dl(x, np.float32) for x in (w, m, v))
        ow, om, ov, g = po.adam_step(w0, m0, v0, 3, 1, step)
        # about ten float32 operations per element: 1e-5 relative to each quantity's own scale
        assert np.max(np.abs(gm - om)) <= 1e-5 * np.max(np.abs(om)) + 1e-12
        assert np.max(np.abs(gv - ov)) <= 1e-5 * np.max(np.abs(ov)) + 1e-18
        # the step lr * m^/(sqrt(v^)+eps) can be large where v is tiny, so the bound is relative to |w| + |step|, per element
        assert np.all(np.abs(gw - ow) <= 1e-5 * (np.abs(w0) + np.abs(ow - w0)) + 1e-12)
        assert np.array_equal(_dl(p, np.uint16)[:numel], po.bf16_bits(gw))
        w0, m0, v0 = gw.astype(np.float64), gm.astype(np.float64), gv.astype(np.float64)   # continue from the device's state


def test_words_fill_and_mutate_bit_exact():
    n = (1 << 18) + 3
    b = harness.DevBuf(4 * n)
    B.proxy_fill_words(b.ptr, n, 42, 0)
    harness.synchronize()
    w = _dl(b, np.uint32)
    assert np.array_equal(w, po.fill_words(n, 42))
    for step in (1, 2, 0xFFFFFFFF):
        B.proxy_mutate_words(b.ptr, n, step, 0)
        harness.synchronize()
        w = po.mutate_words(w, step)
        assert np.array_equal(_dl(b, np.uint32), w)


def test_devcopy_exact_with_ragged_size():
    n = (5 << 20) + 48
    rng = np.random.default_rng(1)
    src = rng.integers(0, 256, n, dtype=np.uint8)
    a, b = harness.DevBuf(n), harness.DevBuf(n + 64)
    a.upload(src)
    B.proxy_device_fill_async(b.ptr, 0xEE, n + 64, 0)
    B.proxy_devcopy(b.ptr, a.ptr, n, 0)
    harness.synchronize()
    out = gu.download(b)
    assert np.array_equal(out[:n], src) and np.all(out[n:] == 0xEE)


@pytest.mark.parametrize("m,n,k", [(128, 128, 64), (256, 384, 192), (1024, 640, 512),
                                   (4096, 4096, 64), (4096, 4352, 192), (8192, 4096, 320)])     # the last three take the 256 x 256 block tile
def test_gemm_bf16_against_float64(m, n, k):
    print(f"gemm {m}x{n}x{k}", flush=True)
    rng = np.random.default_rng(m + n + k)
    a = po.bf16_bits(rng.standard_normal((m, k)).astype(np.float32))
    b = po.bf16_bits(rng.standard_normal((n, k)).astype(np.float32))
    da, db, dc = harness.DevBuf(2 * m * k), harness.DevBuf(2 * n * k), harness.DevBuf(2 * m * n)
    da.upload(a); db.upload(b)
    B.proxy_gemm_bf16(da.ptr, db.ptr, dc.ptr, m, n, k, 0)
    harness.synchronize()
    got = po.bf16_to_f64(_dl(dc, np.uint16).reshape(m, n))
    ref, ref_abs = po.gemm_bf16(a, b)
    # float32 accumulation of K products (any order): K * 2^-24 * sum|a||b|; then one bf16 rounding: 2^-9 * |c| (+ the same on the error)
    bound = k * 2.0 ** -23 * ref_abs + 2.0 ** -8 * np.abs(ref) + 1e-30
    assert np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / bound))
    # and it is not trivially loose: a transposed B or a dropped K-tile would violate it
    assert not np.all(np.abs(got - po.gemm_bf16(a, np.roll(b, 1, axis=0))[0]) <= bound)
