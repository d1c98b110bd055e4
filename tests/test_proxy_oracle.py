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
