"""Pins for the CPU oracle (no GPU). Nothing in the paper prints a byte of a checkpoint file, so the
oracle is pinned by: a file built byte by byte from the format page by independent code, closed-form
sizes of the five workloads, structural invariants, the special case that reduces to numpy's
tobytes(), round trips, and planted mistakes that each pin must catch."""
import os
import struct

import numpy as np
import pytest

from oracle import oracle
from paper_2406_10707_amd import shards
from tests import format_reader as fr


def _tiny3():
    rng = np.random.default_rng(7)
    a = rng.integers(0, 256, 2, dtype=np.uint8)
    b = rng.integers(0, 256, 4097, dtype=np.uint8)
    c = rng.integers(0, 256, 8192, dtype=np.uint8)
    return [("a", shards.BF16, (1,), a), ("b.bytes", shards.U8, (4097,), b), ("c", shards.F32, (2, 1024), c)]


def test_brute_force_three_tensor_file():
    ts = _tiny3()
    want = fr.expected_file([(n, d, s, x.tobytes()) for n, d, s, x in ts], 42)
    got = oracle.serialize_bytes(ts, 42)
    assert got == want
    # sizes worked out by hand: entries 21+1+... ; header fits one unit; data 4096 + 8192 + 8192
    assert len(got) == 4096 + 4096 + 8192 + 8192
    assert oracle.tensor_offsets(ts) == [4096, 8192, 16384]


def test_file_and_memory_serializers_agree(tmp_path):
    ts = _tiny3()
    p = tmp_path / "t.dsl"
    oracle.serialize_file(ts, 5, str(p))
    assert p.read_bytes() == oracle.serialize_bytes(ts, 5)
    assert oracle.compare_file(ts, 5, str(p)) is None


def test_only_iter_differs_between_snapshots():
    ts = _tiny3()
    a, b = oracle.serialize_bytes(ts, 1), oracle.serialize_bytes(ts, 0x0102030405060708)
    diff = [i for i in range(len(a)) if a[i] != b[i]]
    assert diff and min(diff) >= 16 and max(diff) < 24
    assert struct.unpack_from("<Q", b, 16)[0] == 0x0102030405060708


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_tiny_shards_against_independent_writer_and_reader(config, tmp_path):
    spec = shards.make_shard(config, tiny=True)
    ts = [(t.name, t.dtype, t.shape, shards.host_values(spec, k)) for k, t in enumerate(spec.tensors)]
    got = oracle.serialize_bytes(ts, 3)
    assert got == fr.expected_file([(n, d, s, x.tobytes()) for n, d, s, x in ts], 3)
    it, table = fr.parse(got)
    assert it == 3 and [e["name"] for e in table] == [t.name for t in spec.tensors]
    # invariants: first offset = header_bytes, strictly increasing, aligned, disjoint, inside file
    hb = oracle.header_bytes(ts)
    assert table[0]["offset"] == hb
    for e, f in zip(table, table[1:]):
        assert e["offset"] % 4096 == 0 and e["offset"] + e["nbytes"] <= f["offset"]
    assert table[-1]["offset"] + table[-1]["nbytes"] <= len(got)
    # special case reducing to a library routine: data region = concatenation of tobytes() + zero pad
    cat = b"".join(x.tobytes() + b"\0" * (-x.nbytes % 4096) for _, _, _, x in ts)
    assert got[hb:] == cat
    # closed form of the file size
    assert len(got) == hb + sum(-(-x.nbytes // 4096) * 4096 for _, _, _, x in ts)


# closed forms worked out from the model shapes with 14 bytes per parameter
PAYLOAD = {1: 1_742_157_312, 2: 94_337_818_624, 3: 91_113_953_280, 4: 60_816_752_640}
PARAMS = {1: 124_439_808, 2: 6_738_415_616, 3: 6_508_139_520, 4: 4_344_053_760}
PAD = {1: 600_576, 2: 0, 3: 165_888, 4: 0}
NTENS = {1: 592, 2: 1164, 3: 1452, 4: 724, 5: 20000}


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_full_size_headers_and_closed_form_sizes(config):
    spec = shards.make_shard(config)
    ts = [(t.name, t.dtype, t.shape, None) for t in spec.tensors]
    assert len(ts) == NTENS[config]
    if config in PAYLOAD:
        assert spec.n_params == PARAMS[config]
        assert spec.payload_bytes == PAYLOAD[config] == 14 * PARAMS[config]
        assert oracle.data_bytes(ts) == PAYLOAD[config] + PAD[config]
    else:
        assert 38e9 < spec.payload_bytes < 42e9
        assert oracle.data_bytes(ts) - spec.payload_bytes <= 20000 * 4095
        assert max(t.nbytes for t in spec.tensors) == 64 << 20 and min(t.nbytes for t in spec.tensors) >= 4096
    hdr = oracle.build_header(ts, 9)
    hb = oracle.header_bytes(ts)
    assert len(hdr) == hb and hb % 4096 == 0
    # independent parse of the table only (no data present): append nothing, check fields by hand
    version, align, it, n, hb2, db, fb, res = struct.unpack_from("<IIQQQQQQ", hdr, 8)
    assert (version, align, it, n, hb2, res) == (1, 4096, 9, len(ts), hb, 0)
    assert db == oracle.data_bytes(ts) and fb == hb + db
    pos, expect = 64, hb
    for t in spec.tensors:
        (ln,) = struct.unpack_from("<H", hdr, pos); pos += 2
        assert hdr[pos:pos + ln].decode() == t.name; pos += ln
        dtype, ndim = struct.unpack_from("<BB", hdr, pos); pos += 2
        shape = struct.unpack_from("<%dq" % ndim, hdr, pos); pos += 8 * ndim
        off, nb = struct.unpack_from("<QQ", hdr, pos); pos += 16
        assert (dtype, tuple(shape), off, nb) == (t.dtype, tuple(t.shape), expect, t.nbytes)
        expect += -(-nb // 4096) * 4096
    assert expect == fb and not any(hdr[pos:])


@pytest.mark.parametrize("config", [1, 5])
def test_restore_then_reserialize_is_identity(config, tmp_path):
    spec = shards.make_shard(config, tiny=True)
    ts = [(t.name, t.dtype, t.shape, shards.host_values(spec, k).copy()) for k, t in enumerate(spec.tensors)]
    p = str(tmp_path / "a.dsl")
    oracle.serialize_file(ts, 11, p)
    blank = [(n, d, s, np.full(x.nbytes, 0xA5, dtype=np.uint8)) for n, d, s, x in ts]
    assert oracle.restore_file(p, blank) == 11
    for (_, _, _, x), (_, _, _, y) in zip(ts, blank):
        assert np.array_equal(x, y)
    q = str(tmp_path / "b.dsl")
    oracle.serialize_file(blank, 11, q)
    assert open(p, "rb").read() == open(q, "rb").read()


def test_restore_rejects_truncated_corrupt_and_mismatched(tmp_path):
    ts = _tiny3()
    p = str(tmp_path / "a.dsl")
    oracle.serialize_file(ts, 1, p)
    whole = open(p, "rb").read()
    blank = [(n, d, s, np.zeros(x.nbytes, dtype=np.uint8)) for n, d, s, x in ts]
    open(p, "wb").write(whole[:-1])
    with pytest.raises(oracle.OracleError) as e:
        oracle.restore_file(p, blank)
    assert e.value.code == oracle.BAD_FILE
    open(p, "wb").write(b"X" + whole[1:])
    with pytest.raises(oracle.OracleError) as e:
        oracle.restore_file(p, blank)
    assert e.value.code == oracle.BAD_FILE
    open(p, "wb").write(whole)
    other = [("a", shards.BF16, (1,), blank[0][3]), ("b.bytes", shards.U8, (4097,), blank[1][3]),
             ("c", shards.F32, (1024, 2), blank[2][3])]
    with pytest.raises(oracle.OracleError) as e:
        oracle.restore_file(p, other)
    assert e.value.code == oracle.MISMATCH


def test_compare_reports_first_differing_offset(tmp_path):
    ts = _tiny3()
    p = str(tmp_path / "a.dsl")
    oracle.serialize_file(ts, 1, p)
    whole = bytearray(open(p, "rb").read())
    for off in (17, 4096 + 1, 4096 + 2, 8192 + 4096, 8192 + 4097, len(whole) - 1):
        bad = bytearray(whole)
        bad[off] ^= 0x40
        open(p, "wb").write(bad)
        assert oracle.compare_file(ts, 1, p) == off
    open(p, "wb").write(whole + b"\0")
    assert oracle.compare_file(ts, 1, p) == len(whole)


@pytest.mark.parametrize("config", [1, 5])
def test_span_comparison_covers_the_file_piece_by_piece(config, tmp_path):
    """The piecewise comparison used on shards too large to hold twice: every single-byte change anywhere in
    the file (header, payload, padding) is reported by exactly the piece that owns the byte, at its offset,
    and by no other piece; pieces fed only their own tensors' bytes accept the independent writer's file."""
    spec = shards.make_shard(config, tiny=True)
    ts = [(t.name, t.dtype, t.shape, shards.host_values(spec, k)) for k, t in enumerate(spec.tensors)]
    whole = bytearray(fr.expected_file([(n, d, s, x.tobytes()) for n, d, s, x in ts], 9))    # not the oracle's own writer
    p = str(tmp_path / "f.dsl")
    open(p, "wb").write(whole)
    cmp = oracle.SpanComparer(ts)
    n = len(ts)
    cuts = [0, 1, 2, n // 3, n // 2, n - 1, n]
    pieces = [(a, b) for a, b in zip(cuts, cuts[1:]) if b > a]

    def run():
        return [cmp.compare(9, a, [ts[k][3] for k in range(a, b)], p) for a, b in pieces]

    assert run() == [None] * len(pieces)
    _, table = fr.parse(bytes(whole))
    hb = table[0]["offset"]
    rng = np.random.default_rng(config)
    picks = [0, 20, hb - 1, hb, len(whole) - 1]                                    # header, first data byte, last pad byte
    for e in (table[1], table[n // 2], table[-1]):
        picks += [e["offset"], e["offset"] + e["nbytes"] - 1]                      # first and last payload byte of a tensor
        if e["nbytes"] % 4096:
            picks.append(e["offset"] + e["nbytes"])                                # first padding byte behind it
    picks += [int(x) for x in rng.integers(0, len(whole), 12)]
    starts = [table[a]["offset"] if a < n else len(whole) for a, _ in pieces]
    for off in picks:
        bad = bytearray(whole)
        bad[off] ^= 0x21
        open(p, "wb").write(bad)
        owner = 0 if off < hb else max(i for i, s in enumerate(starts) if s <= off)
        assert run() == [off if i == owner else None for i in range(len(pieces))], off
    open(p, "wb").write(whole[:-4096])                                             # wrong size: every piece says so
    assert all(r == len(whole) - 4096 for r in run())
    open(p, "wb").write(whole)
    assert cmp.compare(10, 0, [ts[0][3]], p) == 16                                  # the iteration field belongs to piece 0
    with pytest.raises(ValueError):
        cmp.compare(9, 0, [ts[0][3][:-1]], p)


def test_rejects_bad_descriptions():
    good = np.zeros(8, dtype=np.uint8)
    with pytest.raises(oracle.OracleError):
        oracle.build_header([("x", 9, (2,), None)], 0)            # unknown dtype
    with pytest.raises(oracle.OracleError):
        oracle.build_header([("x", shards.F32, (0,), None)], 0)   # zero bytes
    with pytest.raises(ValueError):
        oracle.serialize_bytes([("x", shards.F32, (3,), good)], 0)  # bytes disagree with shape


def test_planted_mistakes_are_caught():
    """Each pin above must have teeth: mutate the independent expectation the way a plausible bug
    would (unpadded offsets, big-endian field, table order, nonzero pad) and see the oracle differ."""
    ts = _tiny3()
    got = oracle.serialize_bytes(ts, 42)
    flat = [(n, d, s, x.tobytes()) for n, d, s, x in ts]
    want = bytearray(fr.expected_file(flat, 42))
    swapped = fr.expected_file([flat[1], flat[0], flat[2]], 42)
    assert got != swapped
    be = bytearray(want); be[16:24] = struct.pack(">Q", 42)
    assert got != bytes(be)
    pad = bytearray(want); pad[4096 + 2] = 1
    assert got != bytes(pad)
    # offsets without padding (a dropped align_up) would put tensor b at 4098
    assert oracle.tensor_offsets(ts)[1] != 4096 + 2
