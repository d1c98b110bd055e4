"""Pins for the oracle's format version 2 (derived tensors; no GPU). The rounding is pinned by bit patterns
worked out by hand from IEEE 754 and by PyTorch's CPU conversion on a million random patterns; the file by an
independent struct writer; the version decision, sizes, restore and the piecewise comparison by planted changes."""
import struct

import numpy as np
import pytest

from oracle import oracle
from paper_2406_10707_amd import shards
from tests import format_reader as fr

# f32 pattern -> bf16 pattern, each worked out by hand: keep the top 16 bits, look at the 16 dropped ones
# (0x8000 is the half-way point; a tie goes to the even neighbour), NaN keeps sign and top payload and is made quiet
RNE_CASES = [
    (0x3F800000, 0x3F80),   # 1.0, nothing dropped
    (0x3F807FFF, 0x3F80),   # just below half-way: down
    (0x3F808000, 0x3F80),   # tie, 0x3F80 is even: stays
    (0x3F808001, 0x3F81),   # just above half-way: up
    (0x3F818000, 0x3F82),   # tie, 0x3F81 is odd: up to the even 0x3F82
    (0x3F817FFF, 0x3F81),
    (0xC0200000, 0xC020),   # -2.5
    (0x7F7FFFFF, 0x7F80),   # largest finite f32 rounds up to infinity
    (0x7F7F7FFF, 0x7F7F),   # ... the last one that does not
    (0x7F800000, 0x7F80), (0xFF800000, 0xFF80),       # infinities
    (0x7FC00001, 0x7FC0),   # quiet NaN, low payload dropped
    (0x7F800001, 0x7FC0),   # signalling NaN whose payload sits in the dropped bits: must not become infinity
    (0x7F80FFFF, 0x7FC0),
    (0xFFFFFFFF, 0xFFFF),
    (0x7FA12345, 0x7FE1),   # NaN payload in the kept bits survives, quiet bit set
    (0x80000000, 0x8000),   # -0
    (0x00000001, 0x0000),   # smallest denormal: down to +0
    (0x00008000, 0x0000),   # tie between 0x0000 and 0x0001: even
    (0x00008001, 0x0001),
    (0x00018000, 0x0002),   # tie, odd: up
    (0x807FFFFF, 0x8080),   # largest negative denormal rounds up in magnitude, into the normal range
]


def test_rounding_cases_worked_out_by_hand():
    for u, want in RNE_CASES:
        assert oracle.bf16_rne(u) == want, hex(u)
        assert fr.bf16_rne(u) == want, hex(u)


def test_rounding_equals_pytorch_on_random_patterns():
    """The special case that reduces to a library routine: PyTorch's CPU float32 -> bfloat16 conversion rounds to
    nearest even. A million random finite patterns (all exponents, both signs, denormals) plus every hand case
    that is not a NaN, through oracle.pairs_hold: it must accept PyTorch's result and reject it with one bit changed."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2406)
    u = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    u = np.concatenate([u, np.array([c for c, _ in RNE_CASES], dtype=np.uint32)])
    u = u[(u & 0x7FFFFFFF) <= 0x7F800000]                          # NaN policy is the format's own, pinned above
    f = torch.from_numpy(u.view(np.float32).copy())
    b = f.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    n = len(u)
    ts = [("p", shards.BF16, (n,), b.view(np.uint8)), ("w", shards.F32, (n,), u.view(np.uint8))]
    assert oracle.pairs_hold(ts, [(0, 1)])
    for pos in (0, n // 2, n - 1):
        bad = b.copy()
        bad[pos] ^= 1
        assert not oracle.pairs_hold([("p", shards.BF16, (n,), bad.view(np.uint8)), ts[1]], [(0, 1)])
    # plausible wrong roundings differ from it somewhere in this sample
    trunc = (u >> 16).astype(np.uint16)
    away = ((u.astype(np.uint64) + 0x8000) >> 16).astype(np.uint16)
    assert np.any(trunc != b) and np.any(away != b)


def _state(n_params=3, seed=5):
    """A small mixed-precision shard: per parameter p_bf16 (= rounding of master), master, m, v, and one odd-sized extra."""
    rng = np.random.default_rng(seed)
    ts, pairs = [], []
    for k, n in enumerate([5, 2049, 1500][:n_params]):
        master = (rng.standard_normal(n) * 0.02).astype(np.float32)
        master.view(np.uint32)[0] = 0x3F808000                      # a tie among the values
        p = np.array([fr.bf16_rne(int(x)) for x in master.view(np.uint32)], dtype=np.uint16)
        pairs.append((len(ts), len(ts) + 1))
        ts += [(f"w{k}.p_bf16", shards.BF16, (n,), p.view(np.uint8).copy()), (f"w{k}.master", shards.F32, (n,), master.view(np.uint8).copy()),
               (f"w{k}.m", shards.F32, (n,), rng.integers(0, 256, 4 * n, dtype=np.uint8)),
               (f"w{k}.v", shards.F32, (n,), rng.integers(0, 256, 4 * n, dtype=np.uint8))]
    ts.append(("rng_state", shards.U8, (37,), rng.integers(0, 256, 37, dtype=np.uint8)))
    return ts, pairs


def test_version_2_file_against_independent_writer():
    ts, pairs = _state()
    got, version = oracle.serialize_bytes_v2(ts, 77, pairs)
    assert version == 2
    want = fr.expected_file_v2([(n, d, s, x.tobytes()) for n, d, s, x in ts], 77, pairs)
    assert got == want
    hb, db = oracle.v2_sizes(ts, pairs)
    assert (hb, db) == struct.unpack_from("<QQ", got, 32) and len(got) == hb + db
    # sizes by hand: stored tensors are master, m, v of 5, 2049 and 1500 elements (one, three and two 4 KiB units each) and 37 bytes
    assert db == 3 * 4096 + 3 * 3 * 4096 + 3 * 2 * 4096 + 4096
    v1 = oracle.serialize_bytes(ts, 77)
    assert len(v1) - len(got) == 4096 + 2 * 4096 + 4096           # the three bf16 copies (10, 4098, 3000 bytes) and no header growth
    assert struct.unpack_from("<I", got, 8)[0] == 2 and struct.unpack_from("<I", v1, 8)[0] == 1


def test_one_wrong_element_falls_back_to_version_1():
    ts, pairs = _state()
    for k, byte in ((0, 0), (4, 4097), (8, 2999)):                  # first, middle and last derived tensor; first, inner, last byte
        bad = list(ts)
        x = ts[k][3].copy()
        x[byte] ^= 0x10
        bad[k] = (ts[k][0], ts[k][1], ts[k][2], x)
        assert not oracle.pairs_hold(bad, pairs)
        got, version = oracle.serialize_bytes_v2(bad, 3, pairs)
        assert version == 1 and got == oracle.serialize_bytes(bad, 3)
    assert oracle.serialize_bytes_v2(ts, 3, []) == (oracle.serialize_bytes(ts, 3), 1)     # nothing declared: version 1


def test_restore_regenerates_derived_tensors(tmp_path):
    ts, pairs = _state()
    blob, version = oracle.serialize_bytes_v2(ts, 9, pairs)
    p = str(tmp_path / "v2.dsl")
    open(p, "wb").write(blob)
    blank = [(n, d, s, np.full(x.nbytes, 0xA5, dtype=np.uint8)) for n, d, s, x in ts]
    assert oracle.restore_file_v2(p, blank, pairs) == (9, 2)
    assert all(np.array_equal(b[3], t[3]) for b, t in zip(blank, ts))
    assert oracle.serialize_bytes_v2(blank, 9, pairs) == (blob, 2)              # restore then serialize is the identity
    # a version-1 file of the same registration restores through the same call
    open(p, "wb").write(oracle.serialize_bytes(ts, 9))
    blank = [(n, d, s, np.zeros(x.nbytes, dtype=np.uint8)) for n, d, s, x in ts]
    assert oracle.restore_file_v2(p, blank, pairs) == (9, 1)
    assert all(np.array_equal(b[3], t[3]) for b, t in zip(blank, ts))
    # the file's pairs must be the declared ones; a damaged enc byte is a bad file; the v1 reader refuses version 2
    open(p, "wb").write(blob)
    for wrong in ([], pairs[:2], [(0, 1), (4, 5), (8, 5)]):
        with pytest.raises(oracle.OracleError) as e:
            oracle.restore_file_v2(p, blank, wrong)
        assert e.value.code in (oracle.MISMATCH, oracle.BAD_ARG)
    first_entry_end = 64 + 2 + len("w0.p_bf16") + 2 + 8 + 16
    bad = bytearray(blob); bad[first_entry_end] = 7
    open(p, "wb").write(bad)
    with pytest.raises(oracle.OracleError) as e:
        oracle.restore_file_v2(p, blank, pairs)
    assert e.value.code == oracle.BAD_FILE
    open(p, "wb").write(blob)
    with pytest.raises(oracle.OracleError):
        oracle.restore_file(p, blank)


def test_malformed_pairs_are_rejected():
    ts, pairs = _state()
    for wrong in ([(1, 0)], [(0, 2), (0, 1)], [(0, 0)], [(0, 99)], [(0, 5)], [(12, 1)]):   # f32 derived from bf16; twice; self; range; shape; u8
        with pytest.raises(oracle.OracleError):
            oracle.pairs_hold(ts, wrong)


def test_piecewise_comparison_of_a_version_2_file(tmp_path):
    ts, pairs = _state()
    blob, _ = oracle.serialize_bytes_v2(ts, 4, pairs)
    whole = bytearray(fr.expected_file_v2([(n, d, s, x.tobytes()) for n, d, s, x in ts], 4, pairs))
    p = str(tmp_path / "f.dsl")
    cmp = oracle.SpanComparer(ts, pairs)
    pieces = [(0, 4), (4, 5), (5, 12), (12, 13)]

    def run():
        return [cmp.compare(4, a, [None if (k, k + 1) in pairs else ts[k][3] for k in range(a, b)], p, version=2) for a, b in pieces]

    open(p, "wb").write(whole)
    assert run() == [None] * 4
    hb = struct.unpack_from("<Q", whole, 32)[0]
    # stored tensors in order: w0.master at hb, ...; piece (4,5) owns only a derived tensor, i.e. no byte of the file
    owners = {20: 0, hb: 0, hb + 3 * 4096: 2, hb + 3 * 4096 + 2: 2, len(whole) - 1: 3, len(whole) - 4096 + 37: 3}
    for off, owner in owners.items():
        bad = bytearray(whole); bad[off] ^= 0x04
        open(p, "wb").write(bad)
        assert run() == [off if i == owner else None for i in range(4)], off
    open(p, "wb").write(oracle.serialize_bytes(ts, 4))              # a version-1 file where version 2 is expected: wrong size
    assert all(r is not None for r in run())


@pytest.mark.parametrize("config,v1_data,v2_data", [(1, 1_742_157_312 + 600_576, 1_493_277_696 + 340_992),
                                                     (2, 94_337_818_624, 80_860_987_392),
                                                     (3, 91_113_953_280 + 165_888, 78_097_674_240),
                                                     (4, 60_816_752_640, 52_128_645_120)])
def test_closed_form_sizes_of_the_workloads(config, v1_data, v2_data):
    """12 of 14 bytes per parameter remain (payload x 6/7), plus the padding of the stored tensors alone, worked out by
    hand: workload 1 pads its f32 tensors by 3 x (1024 for wte + 12 layers x (4 norms x 1024 + 3072 + 1024 + 1024 for the
    biases) + 2 x 1024 for the final norm) = 340,992 bytes (the other 259,584 of version 1's 600,576 belong to the bf16
    copies); workload 3's whole padding (81 norm weights x 2048) belongs to bf16 copies; 2 and 4 have none."""
    spec = shards.make_shard(config)
    ts = [(t.name, t.dtype, t.shape, None) for t in spec.tensors]
    pairs = [(k, k + 1) for k, t in enumerate(spec.tensors) if t.role == "p_bf16"]
    assert len(pairs) * 4 == len(ts)
    assert oracle.data_bytes(ts) == v1_data
    hb, db = oracle.v2_sizes(ts, pairs)
    assert db == v2_data
    assert spec.payload_bytes * 6 // 7 == sum(t.nbytes for t in spec.tensors if t.role != "p_bf16")
    assert hb == -(-(64 + sum(2 + len(t.name) + 2 + 8 * len(t.shape) + 16 + 5 for t in spec.tensors)) // 4096) * 4096
