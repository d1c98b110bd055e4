"""Seeded synthetic shards: the tensor lists (names, dtypes, shapes, placement) and host-side values
of the five workload configurations, plus tiny variants for fast tests.

This module only describes inputs. It holds none of the checkpoint method's arithmetic (no file
offsets, no header, no alignment): both the HIP library's tests and the CPU oracle's tests take
their inputs from here. The shapes follow the model table of the paper's evaluation section
(layer counts and hidden sizes of the 7B/13B/70B rows) with tensor/pipeline-parallel splits applied
as Megatron-style column/row/vocab splits; the paper's training data and weights are not needed by
a byte mover and are replaced by seeded random state.

Every parameter tensor contributes four state tensors: `<name>.p_bf16` (bf16 working copy),
`<name>.master` (f32), `<name>.m` and `<name>.v` (f32 Adam moments): 14 bytes per parameter.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BF16, F32, F16, U8, I32, I64 = 1, 2, 3, 4, 5, 6
ELSIZE = {BF16: 2, F32: 4, F16: 2, U8: 1, I32: 4, I64: 8}
BASE_SEED = 240610707


@dataclass
class TensorSpec:
    name: str
    dtype: int
    shape: Tuple[int, ...]
    buffer: int = -1      # index into ShardSpec.flat_buffers, or -1: allocation of its own
    offset: int = 0       # byte offset inside that flat buffer
    role: str = ""        # "p_bf16" | "master" | "m" | "v" | "raw"

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= int(s)
        return n

    @property
    def nbytes(self) -> int:
        return self.numel * ELSIZE[self.dtype]


@dataclass
class ShardSpec:
    name: str
    seed: int
    tensors: List[TensorSpec]
    flat_buffers: List[int] = field(default_factory=list)  # byte size of each flat buffer
    compute_ms: float = 1000.0    # length of the synthetic forward+backward phase
    ckpt_every: int = 1
    n_params: int = 0

    @property
    def payload_bytes(self) -> int:
        return sum(t.nbytes for t in self.tensors)


def _state_of(params) -> List[TensorSpec]:
    out = []
    for name, shape in params:
        out.append(TensorSpec(name + ".p_bf16", BF16, tuple(shape), role="p_bf16"))
        out.append(TensorSpec(name + ".master", F32, tuple(shape), role="master"))
        out.append(TensorSpec(name + ".m", F32, tuple(shape), role="m"))
        out.append(TensorSpec(name + ".v", F32, tuple(shape), role="v"))
    return out


def _numel(params) -> int:
    return sum(int(np.prod(s, dtype=np.int64)) for _, s in params)


def gpt2_params(vocab=50257, hidden=768, layers=12, npos=1024):
    """GPT-2 layout with tied input/output embedding, biases and two LayerNorms per layer."""
    p = [("wte", (vocab, hidden)), ("wpe", (npos, hidden))]
    for l in range(layers):
        b = f"h.{l}."
        p += [(b + "ln_1.weight", (hidden,)), (b + "ln_1.bias", (hidden,)),
              (b + "attn.c_attn.weight", (hidden, 3 * hidden)), (b + "attn.c_attn.bias", (3 * hidden,)),
              (b + "attn.c_proj.weight", (hidden, hidden)), (b + "attn.c_proj.bias", (hidden,)),
              (b + "ln_2.weight", (hidden,)), (b + "ln_2.bias", (hidden,)),
              (b + "mlp.c_fc.weight", (hidden, 4 * hidden)), (b + "mlp.c_fc.bias", (4 * hidden,)),
              (b + "mlp.c_proj.weight", (4 * hidden, hidden)), (b + "mlp.c_proj.bias", (hidden,))]
    p += [("ln_f.weight", (hidden,)), ("ln_f.bias", (hidden,))]
    return p


def llama_params(layers, hidden, ffn, vocab, heads, kv_heads, tp=1, first_stage=True, last_stage=True,
                 layer0=0):
    """Llama layout (RMSNorm, SwiGLU, no biases) as one tensor-parallel rank of degree `tp` holds it:
    q/k/v/gate/up split by output rows, o/down split by input columns, embedding and lm_head split by
    vocabulary, norms replicated."""
    hd = hidden // heads
    q_rows = heads * hd // tp
    kv_rows = kv_heads * hd // tp
    p = []
    if first_stage:
        p.append(("embed_tokens.weight", (vocab // tp, hidden)))
    for l in range(layer0, layer0 + layers):
        b = f"layers.{l}."
        p += [(b + "input_layernorm.weight", (hidden,)),
              (b + "self_attn.q_proj.weight", (q_rows, hidden)),
              (b + "self_attn.k_proj.weight", (kv_rows, hidden)),
              (b + "self_attn.v_proj.weight", (kv_rows, hidden)),
              (b + "self_attn.o_proj.weight", (hidden, q_rows)),
              (b + "post_attention_layernorm.weight", (hidden,)),
              (b + "mlp.gate_proj.weight", (ffn // tp, hidden)),
              (b + "mlp.up_proj.weight", (ffn // tp, hidden)),
              (b + "mlp.down_proj.weight", (hidden, ffn // tp))]
    if last_stage:
        p += [("norm.weight", (hidden,)), ("lm_head.weight", (vocab // tp, hidden))]
    return p


class _SplitMix64:
    """Small documented host PRNG so that layouts are reproducible without numpy's bit generators."""

    def __init__(self, seed: int):
        self.s = seed & 0xFFFFFFFFFFFFFFFF

    def next(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        return z ^ (z >> 31)

    def uniform(self) -> float:
        return (self.next() >> 11) * (1.0 / (1 << 53))

    def below(self, n: int) -> int:
        return self.next() % n


def fragmentation_tensors(seed, n_tensors, min_bytes, max_bytes, n_buffers, n_huge=0, huge_bytes=0):
    """ZeRO-style flattened buffers: tensors are sub-ranges of a few flat device buffers, starting at
    multiples of their element size only (so most starts are not 16-byte aligned), with sizes drawn
    log-uniformly in [min_bytes, max_bytes] and rounded to the element size, not to 16 bytes.
    Tensors are carved from the buffers in a shuffled order, so registration order jumps around."""
    rng = _SplitMix64(seed)
    sizes = []
    lo, hi = np.log(min_bytes), np.log(max_bytes)
    for i in range(n_tensors):
        dtype = BF16 if rng.next() & 1 else F32
        es = ELSIZE[dtype]
        nb = int(np.exp(lo + (hi - lo) * rng.uniform()))
        nb = max(es, nb // es * es)
        sizes.append((dtype, nb))
    for i in range(n_huge):
        dtype = BF16 if i & 1 else F32
        sizes.append((dtype, huge_bytes))
    n = len(sizes)
    # shuffled carving order (Fisher-Yates)
    order = list(range(n))
    for i in range(n - 1, 0, -1):
        j = rng.below(i + 1)
        order[i], order[j] = order[j], order[i]
    cursor = [0] * n_buffers
    place = [None] * n
    for idx in order:
        dtype, nb = sizes[idx]
        es = ELSIZE[dtype]
        b = rng.below(n_buffers)
        gap = rng.below(16) * 2          # 0..30 bytes
        start = cursor[b] + gap
        start = (start + es - 1) // es * es
        place[idx] = (b, start)
        cursor[b] = start + nb
    tensors = []
    for i, (dtype, nb) in enumerate(sizes):
        b, start = place[i]
        tensors.append(TensorSpec(f"flat{b}.frag{i:05d}", dtype, (nb // ELSIZE[dtype],), buffer=b, offset=start,
                                  role="raw"))
    flat = [(c + 255) // 256 * 256 + 256 for c in cursor]
    return tensors, flat


def make_shard(config: int, tiny: bool = False) -> ShardSpec:
    """config 1..5 as named by the benchmark definition; tiny=True gives a structurally identical
    shard small enough for CPU tests (same tensor roles and raggedness, far fewer bytes)."""
    seed = BASE_SEED + config
    if config == 1:
        params = gpt2_params(vocab=503, hidden=24, layers=2, npos=32) if tiny else gpt2_params()
        s = ShardSpec("gpt2-small-124M" + ("-tiny" if tiny else ""), seed, _state_of(params), compute_ms=100.0,
                      ckpt_every=1)
    elif config == 2:
        params = (llama_params(2, 128, 344, 1000, 4, 4) if tiny
                  else llama_params(32, 4096, 11008, 32000, 32, 32))
        s = ShardSpec("llama-7B-whole" + ("-tiny" if tiny else ""), seed, _state_of(params), compute_ms=1000.0,
                      ckpt_every=10)
    elif config == 3:
        params = (llama_params(2, 160, 432, 1000, 4, 4, tp=2) if tiny
                  else llama_params(40, 5120, 13824, 32000, 40, 40, tp=2))
        s = ShardSpec("llama-13B-tp2-share" + ("-tiny" if tiny else ""), seed, _state_of(params), compute_ms=2000.0,
                      ckpt_every=1)
    elif config == 4:
        params = (llama_params(2, 256, 896, 1000, 8, 4, tp=4, last_stage=False) if tiny
                  else llama_params(20, 8192, 28672, 32000, 64, 8, tp=4, last_stage=False))
        s = ShardSpec("llama-70B-tp4pp4-stage0" + ("-tiny" if tiny else ""), seed, _state_of(params), compute_ms=300.0,
                      ckpt_every=1)
    elif config == 5:
        if tiny:
            tensors, flat = fragmentation_tensors(seed, 300, 2, 192 * 1024, 3, n_huge=2, huge_bytes=1 << 20)
        else:
            # 20,000 tensors, log-uniform 4 KiB..16 MiB (mean about 2 MB, about 40 GB in all) plus
            # eight 64 MiB tensors so the stated maximum size is exercised.
            tensors, flat = fragmentation_tensors(seed, 20000 - 8, 4096, 16 << 20, 8, n_huge=8, huge_bytes=64 << 20)
        s = ShardSpec("fragmentation-stress" + ("-tiny" if tiny else ""), seed, tensors, flat_buffers=flat,
                      compute_ms=1000.0, ckpt_every=1)
        return s
    else:
        raise ValueError("config must be 1..5")
    s.n_params = _numel(params)
    return s


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even; NaN kept quiet."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = ((u + (0x7FFF + ((u >> 16) & 1))) >> 16).astype(np.uint16)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    rounded[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return rounded


def host_values(spec: ShardSpec, k: int) -> np.ndarray:
    """Bytes (uint8 array) of tensor k of the shard, from its seed: master and m ~ N(0, 0.02),
    p_bf16 = bf16(master), v = N(0, 1e-3)^2. Raw fragments get normal values with a sprinkling of
    special bit patterns (NaN payloads, -0, denormals, all-ones) because a byte mover must not care."""
    t = spec.tensors[k]
    n = t.numel
    if t.role in ("p_bf16", "master"):
        base = k - (0 if t.role == "p_bf16" else 1)           # both derive from one stream
        g = np.random.Generator(np.random.Philox(key=spec.seed, counter=[0, 0, 0, base]))
        master = (g.standard_normal(n, dtype=np.float32) * np.float32(0.02))
        if t.role == "master":
            return master.view(np.uint8)
        return f32_to_bf16_rne(master).view(np.uint8)
    g = np.random.Generator(np.random.Philox(key=spec.seed, counter=[0, 0, 0, k]))
    if t.role == "m":
        return (g.standard_normal(n, dtype=np.float32) * np.float32(0.02)).view(np.uint8)
    if t.role == "v":
        z = g.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
        return (z * z).view(np.uint8)
    # raw fragment
    z = g.standard_normal(n, dtype=np.float32) * np.float32(0.02)
    if t.dtype == F32:
        u = z.view(np.uint32).copy()
        special = np.array([0x7FC00001, 0xFFC12345, 0x80000000, 0x00000001, 0x807FFFFF, 0xFFFFFFFF, 0x7F800000],
                           dtype=np.uint32)
    else:
        u = f32_to_bf16_rne(z).copy()
        special = np.array([0x7FC1, 0xFFFF, 0x8000, 0x0001, 0x807F, 0x7F80, 0xFF80], dtype=np.uint16)
    if n >= 8:
        pos = g.integers(0, n, size=max(1, n // 64))
        u[pos] = special[g.integers(0, len(special), size=len(pos))]
    return u.view(np.uint8)
