"""Pins for the proxy oracle (no GPU): published splitmix64 outputs, bf16 rounding cases, textbook
properties of Adam's first step, moments of the normal generator, brute-force GEMM on a tiny case."""
import numpy as np

from oracle import proxy_oracle as po


def test_mix_is_the_splitmix64_output_function():
    # splitmix64 seeded with 0 yields these first three outputs (reference values of the published generator)
    g = 0x9E3779B97F4A7C15
    got = [int(po.mix(np.uint64((k * g) & 0xFFFFFFFFFFFFFFFF))) for k in range(3)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_bf16_rounding_cases():
    f = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0, -0.0, np.inf], dtype=np.float32)
    bits = po.bf16_bits(f)
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80); 1 + 3*2^-8 ties between 0x3F81 and 0x3F82 -> 0x3F82
    assert list(bits) == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000, 0x8000, 0x7F80]
    nan = po.bf16_bits(np.array([np.nan], dtype=np.float32))
    assert (nan[0] & 0x7F80) == 0x7F80 and (nan[0] & 0x7F) != 0
    assert np.array_equal(po.bf16_to_f64(np.array([0x3F80, 0xC020], dtype=np.uint16)), [1.0, -2.5])


def test_normal_generator_moments_and_independence_of_streams():
    z = po.normal(5, 3, 0, 1 << 20)
    assert abs(z.mean()) < 4e-3 and abs(z.var() - 1.0) < 6e-3
    assert abs(np.mean(z ** 4) - 3.0) < 0.05                      # kurtosis of a normal
    z2 = po.normal(5, 3, 1, 1 << 20)
    assert abs(np.corrcoef(z, z2)[0, 1]) < 5e-3
    assert np.array_equal(po.normal(5, 3, 0, 100), z[:100])        # counter based: prefix property
    # Box-Muller closed form at chosen uniforms: r with hi = 2^23-ish gives known values
    r = np.uint64((8388607 << 40) | 0)                              # u_hi = (8388607.5)/2^24, u_lo = 0.5/2^24
    u_hi, u_lo = 8388607.5 / 16777216.0, 0.5 / 16777216.0
    want = np.sqrt(-2 * np.log(u_hi)) * np.cos(2 * np.pi * u_lo)
    hi = ((r >> np.uint64(40)).astype(np.float64) + 0.5) / 16777216.0
    assert hi == u_hi and abs(want - 1.17741002) < 1e-6             # sqrt(2 ln 2) = 1.1774100226


def test_adam_first_step_is_lr_times_sign_of_gradient():
    n = 1000
    master = np.linspace(-1, 1, n)
    w, m, v, g = po.adam_step(master, np.zeros(n), np.zeros(n), seed=1, tensor=2, step=1, lr=1e-3, eps=0.0)
    assert np.allclose(master - w, 1e-3 * np.sign(g), rtol=1e-12)   # bias-corrected first step: m^ = g, v^ = g^2
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    assert np.all(np.abs(g) <= 1e-3) and abs(g.mean()) < 1e-4
    # zero gradient contribution: with beta1 = beta2 = 1 nothing moves the moments
    w2, m2, v2, _ = po.adam_step(master, np.full(n, 0.5), np.full(n, 0.25), 1, 2, 3, beta1=1.0 - 1e-16, beta2=1.0 - 1e-16)
    assert np.allclose(m2, 0.5) and np.allclose(v2, 0.25)


def test_words_and_gemm_small_cases():
    w = po.fill_words(8, 9)
    assert w.dtype == np.uint32 and len(set(w.tolist())) == 8
    m = po.mutate_words(np.array([0, 1, 0xFFFFFFFF], dtype=np.uint32), 7)
    assert list(m) == [(1013904223 + 7) & 0xFFFFFFFF, (1664525 + 1013904223 + 7) & 0xFFFFFFFF,
                       (0xFFFFFFFF * 1664525 + 1013904223 + 7) & 0xFFFFFFFF]
    rng = np.random.default_rng(0)
    a = po.bf16_bits(rng.standard_normal((3, 5)).astype(np.float32))
    b = po.bf16_bits(rng.standard_normal((4, 5)).astype(np.float32))
    c, cabs = po.gemm_bf16(a, b)
    af, bf = po.bf16_to_f64(a), po.bf16_to_f64(b)
    for i in range(3):
        for j in range(4):
            assert abs(c[i, j] - sum(af[i, k] * bf[j, k] for k in range(5))) < 1e-12     # C = A . B^T, not A . B
    eye = po.bf16_bits(np.eye(5, dtype=np.float32))
    assert np.array_equal(po.gemm_bf16(a, eye)[0], af)


# ---- the generator's structure, worked out here with plain Python integers and the math module
# (definition: include/ckpt_proxy.h); a second implementation, not a call into the oracle

_M = (1 << 64) - 1


def _mix(x):
    z = (x + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def _r(seed, tensor, tag, i):
    return _mix(_mix(seed ^ _mix((4 * tensor + tag) & _M)) ^ _mix(i))


def _normal(r):
    import math
    u_hi, u_lo = ((r >> 40) + 0.5) / 2 ** 24, ((r & 0xFFFFFF) + 0.5) / 2 ** 24
    return math.sqrt(-2.0 * math.log(u_hi)) * math.cos(2.0 * math.pi * u_lo)


def test_stream_key_and_raw_against_integer_arithmetic():
    """One (seed, tensor, tag, i) per tag with its value as a literal: a permuted tag, tensor + 4*tag
    instead of 4*tensor + tag, a dropped mix or a swapped xor operand changes every one of them."""
    want = {0: 0x59E6584482B23B58, 1: 0xB06138AC67950DF5, 2: 0x3E7E5D5C5AEE8AA1, 3: 0x839E38B7AC70B48B}
    for tag, value in want.items():
        assert _r(240610708, 3, tag, 5) == value
        assert int(po.raw(240610708, 3, tag, 6)[5]) == value
        assert int(po.stream_key(240610708, 3, tag)) == _mix(240610708 ^ _mix(12 + tag))
    assert int(po.stream_key(240610708, 3, 2)) == 0x5E4715B59C131836
    # tensor and tag are not interchangeable: (tensor 1, tag 0) and (tensor 0, tag 1) differ, and differ from 4*tag + tensor
    assert int(po.raw(7, 1, 0, 1)[0]) == 0xE1A01477873B45AA and int(po.raw(7, 0, 1, 1)[0]) == 0xD76FDF18A84B410D
    assert int(po.raw(7, 0, 0, 1)[0]) == 0x3EC50D771D8EDE0D
    assert _r(7, 1, 0, 0) == 0xE1A01477873B45AA and _mix(7 ^ _mix(1 + 4 * 0)) != _mix(7 ^ _mix(4 * 1 + 0))   # tensor + 4*tag is another key


def test_fill_state_tags_and_scale_factors():
    """master = 0.02 normal(tag 0), m = 0.02 normal(tag 1), v = (0.001 normal(tag 2))^2, element by element
    against the integer generator and math.sqrt/log/cos, plus the three scales from sample moments."""
    seed, tensor, n = 240610708, 3, 1 << 18
    master, m, v = po.fill_state(n, seed, tensor)
    for i in (0, 5, 4097, n - 1):
        assert abs(master[i] - 0.02 * _normal(_r(seed, tensor, 0, i))) < 1e-15
        assert abs(m[i] - 0.02 * _normal(_r(seed, tensor, 1, i))) < 1e-15
        assert abs(v[i] - (0.001 * _normal(_r(seed, tensor, 2, i))) ** 2) < 1e-18
    assert abs(master.std() / 0.02 - 1) < 0.01 and abs(m.std() / 0.02 - 1) < 0.01
    assert abs(v.mean() / 1e-6 - 1) < 0.02 and v.min() >= 0.0
    assert abs(np.corrcoef(master, m)[0, 1]) < 0.01                 # two streams, not one
    # the gradient of the Adam step uses tag 3 of seed + step: g = 0.001 (2 (r >> 40) / 2^24 - 1)
    _, _, _, g = po.adam_step(master[:8], m[:8], v[:8], seed, tensor, step=4)
    for i in range(8):
        assert abs(g[i] - 0.001 * (2.0 * (_r(seed + 4, tensor, 3, i) >> 40) / 2 ** 24 - 1.0)) < 1e-18


def test_fill_words_is_the_low_half_of_stream_zero():
    w = po.fill_words(6, 240610712)
    assert w.dtype == np.uint32
    assert [int(x) for x in w] == [_r(240610712, 0, 0, i) & 0xFFFFFFFF for i in range(6)]
    assert int(po.fill_words(1, 7)[0]) == 0x1D8EDE0D                # low 32 bits of r(7, 0, 0, 0) = 0x3EC50D771D8EDE0D
