"""CPU oracle for the synthetic training proxy (numpy, float64). TEST INFRASTRUCTURE ONLY.

The proxy stands in for the phases of a training iteration the paper's immutability section
distinguishes: forward/backward, which only read parameters and optimizer state (here a bf16 GEMM),
and the update, which mutates all of them in bulk (here an Adam step). The paper prescribes neither;
the definitions are the ones written in include/ckpt_proxy.h, taken here step by step in float64:

  mix(x):  z = x + 0x9E3779B97F4A7C15; z = (z ^ z>>30) * 0xBF58476D1CE4E5B9;
           z = (z ^ z>>27) * 0x94D049BB133111EB; z ^ z>>31          (the splitmix64 output function)
  r(seed, tensor, tag, i) = mix( mix(seed ^ mix(4*tensor + tag)) ^ mix(i) )
  normal = sqrt(-2 ln u_hi) cos(2 pi u_lo),  u_hi = ((r>>40)+0.5)/2^24,  u_lo = ((r & 0xFFFFFF)+0.5)/2^24
"""
import numpy as np

M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def mix(x):
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def stream_key(seed, tensor, tag):
    return mix(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) ^ mix(np.uint64((tensor * 4 + tag) & 0xFFFFFFFFFFFFFFFF)))


def raw(seed, tensor, tag, n):
    i = np.arange(n, dtype=np.uint64)
    return mix(stream_key(seed, tensor, tag) ^ mix(i))


def normal(seed, tensor, tag, n):
    r = raw(seed, tensor, tag, n)
    u_hi = ((r >> np.uint64(40)).astype(np.float64) + 0.5) / 16777216.0
    u_lo = ((r & np.uint64(0xFFFFFF)).astype(np.float64) + 0.5) / 16777216.0
    return np.sqrt(-2.0 * np.log(u_hi)) * np.cos(2.0 * np.pi * u_lo)


def bf16_bits(x32):
    """float32 -> bf16 bit pattern, round to nearest, ties to even (NaN stays a quiet NaN)."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    out = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)).astype(np.uint16)
    nan = (u & np.uint64(0x7FFFFFFF)) > np.uint64(0x7F800000)
    out[nan] = ((u[nan] >> np.uint64(16)) | np.uint64(0x40)).astype(np.uint16)
    return out


def bf16_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def fill_state(numel, seed, tensor):
    """(master, m, v) in float64. p_bf16 is bf16(master) of whatever float32 master the device produced."""
    master = 0.02 * normal(seed, tensor, 0, numel)
    m = 0.02 * normal(seed, tensor, 1, numel)
    s = 0.001 * normal(seed, tensor, 2, numel)
    return master, m, s * s


def adam_step(master, m, v, seed, tensor, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step in float64 on float64 copies of the inputs; returns (master, m, v, g)."""
    master, m, v = (np.asarray(a, dtype=np.float64) for a in (master, m, v))
    n = master.size
    r = raw(seed + step, tensor, 3, n)
    g = 0.001 * (2.0 * ((r >> np.uint64(40)).astype(np.float64) / 16777216.0) - 1.0)
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - beta1 ** step)
    vhat = v1 / (1.0 - beta2 ** step)
    return master - lr * mhat / (np.sqrt(vhat) + eps), m1, v1, g


def fill_words(n_words, seed):
    return (raw(seed, 0, 0, n_words) & np.uint64(0xFFFFFFFF)).astype(np.uint32)


def mutate_words(words, step):
    w = np.asarray(words, dtype=np.uint32).astype(np.uint64)
    return ((w * np.uint64(1664525) + np.uint64(1013904223) + np.uint64(step & 0xFFFFFFFF)) & np.uint64(0xFFFFFFFF)).astype(np.uint32)


def gemm_bf16(a_bits, b_bits):
    """C = A . B^T in float64 from bf16 bit patterns A[M,K], B[N,K] (the definition, via numpy's matmul)."""
    a, b = bf16_to_f64(a_bits), bf16_to_f64(b_bits)
    return a @ b.T, np.abs(a) @ np.abs(b).T
