"""Host logic of the HIP library, no GPU needed: the shared library loads and exports every symbol
its headers declare; the plan (header bytes, file offsets, tile table) agrees with the CPU oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import oracle
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import shards

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_BASE = 0x7000_0000_0000


def _declared_symbols():
    names = []
    for h in ("ckpt.h", "ckpt_proxy.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b((?:ckpt|proxy)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    declared = _declared_symbols()
    assert len(declared) >= 20
    raw = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name
    assert set(declared) == set(B.EXPORTED)


def _fake_descs(spec):
    """Device addresses are never dereferenced by the planner: lay tensors out in a fake address space."""
    addr = FAKE_BASE
    flat_base = []
    for n in spec.flat_buffers:
        flat_base.append(addr)
        addr += n + 4096
    descs = []
    for t in spec.tensors:
        if t.buffer >= 0:
            p = flat_base[t.buffer] + t.offset
        else:
            p = addr
            addr += (t.nbytes + 511) // 512 * 512
        descs.append((t.name, t.dtype, t.shape, p, t.nbytes))
    return descs, addr - FAKE_BASE


@pytest.mark.parametrize("tiny", [True, False])
@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_header_and_offsets_match_oracle(config, tiny):
    spec = shards.make_shard(config, tiny=tiny)
    descs, _ = _fake_descs(spec)
    plan = B.Plan(descs)
    ots = [(t.name, t.dtype, t.shape, None) for t in spec.tensors]
    assert plan.header(77) == oracle.build_header(ots, 77)
    lay = plan.layout()
    assert lay["header_bytes"] == oracle.header_bytes(ots)
    assert lay["data_bytes"] == oracle.data_bytes(ots)
    assert lay["file_bytes"] == lay["header_bytes"] + lay["data_bytes"]
    assert lay["payload_bytes"] == spec.payload_bytes
    if tiny:
        assert plan.offsets() == oracle.tensor_offsets(ots)
    plan.close()


@pytest.mark.parametrize("config", [1, 5])
@pytest.mark.parametrize("chunk,superchunk", [(64 << 10, 128 << 10), (128 << 10, 1 << 20)])
def test_tile_table_reproduces_the_data_region(config, chunk, superchunk):
    """Walk the tile table on the host over a fake address space and compare the bytes it would
    produce with the oracle's data region: pins tile sources, destinations, zero padding and that
    no tile crosses a super-chunk."""
    spec = shards.make_shard(config, tiny=True)
    descs, span = _fake_descs(spec)
    mem = np.full(span + 64, 0xEE, dtype=np.uint8)
    host = []
    for k, (name, dtype, shape, p, nb) in enumerate(descs):
        v = shards.host_values(spec, k)
        mem[p - FAKE_BASE:p - FAKE_BASE + nb] = v
        host.append(v)
    cfg = B.make_config(dma_chunk_bytes=chunk, pack_superchunk_bytes=superchunk)
    plan = B.Plan(descs, cfg)
    lay = plan.layout()
    tiles = plan.tiles()
    out = np.full(lay["data_bytes"], 0xCC, dtype=np.uint8)
    pos = 0
    for t in tiles:
        assert t.dst_off == pos and t.dst_off % 16 == 0 and t.total_bytes % 16 == 0 and 0 < t.total_bytes <= lay["tile_bytes"]
        assert t.dst_off // superchunk == (t.dst_off + t.total_bytes - 1) // superchunk
        s = t.src - FAKE_BASE
        out[pos:pos + t.copy_bytes] = mem[s:s + t.copy_bytes]
        out[pos + t.copy_bytes:pos + t.total_bytes] = 0
        pos += t.total_bytes
    assert pos == lay["data_bytes"]
    ots = [(t.name, t.dtype, t.shape, h) for t, h in zip(spec.tensors, host)]
    want = oracle.serialize_bytes(ots, 0)
    assert out.tobytes() == want[lay["header_bytes"]:]
    first = plan.superchunk_tiles()
    assert first[0] == 0 and first[-1] == len(tiles) and lay["n_superchunks"] == -(-lay["data_bytes"] // superchunk)
    for s in range(lay["n_superchunks"]):
        for i in range(first[s], first[s + 1]):
            assert tiles[i].dst_off // superchunk == s
    assert lay["n_chunks"] == -(-lay["data_bytes"] // chunk)
    plan.close()


@pytest.mark.parametrize("config", [1, 5])
@pytest.mark.parametrize("direct_min", [0, 4096, 20000, 1 << 20])
def test_segments_reproduce_the_data_region(config, direct_min):
    """The hybrid plan on the host: tiles fill a staging image (holes where large tensors are copied
    directly), then every chunk is put together from its segments the way the copy engine would:
    STAGED out of staging, DIRECT out of the tensor's own memory, ZERO by the host. The result must
    be the oracle's data region, and no segment may cross a chunk."""
    chunk, superchunk = 64 << 10, 256 << 10
    spec = shards.make_shard(config, tiny=True)
    descs, span = _fake_descs(spec)
    mem = np.full(span + 64, 0xEE, dtype=np.uint8)
    host = []
    for k, (name, dtype, shape, p, nb) in enumerate(descs):
        v = shards.host_values(spec, k)
        mem[p - FAKE_BASE:p - FAKE_BASE + nb] = v
        host.append(v)
    plan = B.Plan(descs, B.make_config(dma_chunk_bytes=chunk, pack_superchunk_bytes=superchunk, direct_min_bytes=direct_min))
    lay = plan.layout()
    big = [k for k, d in enumerate(descs) if direct_min and d[4] >= direct_min]
    assert lay["n_direct_tensors"] == len(big) and lay["direct_bytes"] == sum(descs[k][4] for k in big)
    staging = np.full(lay["data_bytes"], 0xCC, dtype=np.uint8)       # 0xCC: never written by a pack kernel
    packed = np.zeros(lay["data_bytes"], dtype=bool)
    for t in plan.tiles():
        s = t.src - FAKE_BASE
        staging[t.dst_off:t.dst_off + t.copy_bytes] = mem[s:s + t.copy_bytes]
        staging[t.dst_off + t.copy_bytes:t.dst_off + t.total_bytes] = 0
        assert not packed[t.dst_off:t.dst_off + t.total_bytes].any()
        packed[t.dst_off:t.dst_off + t.total_bytes] = True
    segs, first = plan.segments(), plan.chunk_segments()
    assert first[0] == 0 and first[-1] == len(segs) == lay["n_segments"] and len(first) == lay["n_chunks"] + 1
    out = np.full(lay["data_bytes"], 0x77, dtype=np.uint8)
    pos = 0
    kinds = set()
    for ch in range(lay["n_chunks"]):
        assert first[ch] < first[ch + 1]
        for j in range(first[ch], first[ch + 1]):
            sg = segs[j]
            assert sg.data_off == pos and sg.nbytes > 0 and sg.data_off // chunk == ch == (sg.data_off + sg.nbytes - 1) // chunk
            a, b = sg.data_off, sg.data_off + sg.nbytes
            kinds.add(sg.kind)
            if sg.kind == B.CKPT_SEG_STAGED:
                assert packed[a:b].all()
                out[a:b] = staging[a:b]
            elif sg.kind == B.CKPT_SEG_DIRECT:
                assert not packed[a:b].any() and sg.tensor in big
                assert descs[sg.tensor][3] <= sg.src and sg.src + sg.nbytes <= descs[sg.tensor][3] + descs[sg.tensor][4]
                out[a:b] = mem[sg.src - FAKE_BASE:sg.src - FAKE_BASE + sg.nbytes]
            else:
                assert sg.kind == B.CKPT_SEG_ZERO and not packed[a:b].any() and sg.nbytes < 4096
                out[a:b] = 0
            pos = b
    assert pos == lay["data_bytes"]
    if direct_min == 0:
        assert kinds == {B.CKPT_SEG_STAGED} and len(segs) == lay["n_chunks"]
    elif direct_min == 4096:
        assert B.CKPT_SEG_DIRECT in kinds and lay["n_direct_tensors"] > 0
    ots = [(t.name, t.dtype, t.shape, h) for t, h in zip(spec.tensors, host)]
    assert out.tobytes() == oracle.serialize_bytes(ots, 0)[lay["header_bytes"]:]
    plan.close()


def test_host_resident_objects_in_the_plan():
    """Objects flagged CKPT_PLACE_HOST: same header and offsets as if they lived on the device (the
    file does not record placement), no tiles, HOST segments that point into the objects, ZERO
    segments for their padding; any address alignment is accepted for them."""
    chunk = 64 << 10
    spec = shards.make_shard(1, tiny=True)
    descs, span = _fake_descs(spec)
    host_base = 0x5000_0000_0001                 # odd on purpose
    extra = [("rng_state", B.CKPT_U8 | B.CKPT_PLACE_HOST, (5056,), host_base, 5056),
             ("offloaded.exp_avg", B.CKPT_F32 | B.CKPT_PLACE_HOST, (300, 77), host_base + 8192, 300 * 77 * 4),
             ("args", B.CKPT_U8 | B.CKPT_PLACE_HOST, (137,), host_base + 200000, 137)]
    mixed = descs[:5] + extra[:2] + descs[5:] + extra[2:]
    plan = B.Plan(mixed, B.make_config(dma_chunk_bytes=chunk, pack_superchunk_bytes=4 * chunk))
    lay = plan.layout()
    assert lay["n_host_objects"] == 3 and lay["host_bytes"] == 5056 + 92400 + 137
    assert lay["host_data_bytes"] == 8192 + 94208 + 4096
    plain = [(n, d & 0xFF, s, None) for n, d, s, p_, nb in mixed]
    assert plan.header(5) == oracle.build_header(plain, 5)
    assert plan.offsets() == oracle.tensor_offsets(plain)
    offs = plan.offsets()
    host_idx = {k for k, d in enumerate(mixed) if d[1] & B.CKPT_PLACE_HOST}
    covered = {k: 0 for k in host_idx}
    for sg in plan.segments():
        if sg.kind == B.CKPT_SEG_HOST:
            d = mixed[sg.tensor]
            assert sg.tensor in host_idx and d[3] <= sg.src and sg.src + sg.nbytes <= d[3] + d[4]
            assert sg.data_off + lay["header_bytes"] == offs[sg.tensor] + (sg.src - d[3])
            covered[sg.tensor] += sg.nbytes
        elif sg.kind == B.CKPT_SEG_ZERO:
            assert sg.tensor in host_idx
    assert all(covered[k] == mixed[k][4] for k in host_idx)
    for t in plan.tiles():        # no tile reads a host address
        assert t.copy_bytes == 0 or FAKE_BASE <= t.src < FAKE_BASE + span
    plan.close()


def test_full_size_hybrid_plan_counts():
    """Llama-7B with everything of 1 MiB and more copied directly: only the norm weights are packed."""
    spec = shards.make_shard(2)
    descs, _ = _fake_descs(spec)
    plan = B.Plan(descs, B.make_config(direct_min_bytes=1 << 20))
    lay = plan.layout()
    small = [d for d in descs if d[4] < (1 << 20)]
    assert lay["n_direct_tensors"] == len(descs) - len(small) and 0 < len(small) < len(descs)
    assert len(small) <= lay["n_tiles"] <= 2 * len(small)      # 8 and 16 KiB norm weights: one or two tiles each
    assert lay["direct_bytes"] == sum(d[4] for d in descs) - sum(d[4] for d in small)
    assert lay["n_segments"] <= lay["n_chunks"] + 3 * len(descs)
    plan.close()


def test_full_size_tile_counts():
    spec = shards.make_shard(2)
    descs, _ = _fake_descs(spec)
    plan = B.Plan(descs)
    lay = plan.layout()
    assert lay["n_superchunks"] == -(-lay["data_bytes"] // (1 << 30)) and lay["n_chunks"] == -(-lay["data_bytes"] // (256 << 20))   # the defaults: 1 GiB per pack launch, 256 MiB per copy
    assert lay["data_bytes"] // lay["tile_bytes"] <= lay["n_tiles"] <= lay["data_bytes"] // lay["tile_bytes"] + 2 * lay["n_tensors"]
    plan.close()


def _expect(code, descs, **cfg):
    with pytest.raises(B.CkptError) as e:
        B.Plan(descs, B.make_config(**cfg))
    assert e.value.code == code and e.value.text


def test_bad_descriptions_and_configs_are_rejected():
    ok = ("t", B.CKPT_F32, (4,), FAKE_BASE, 16)
    B.Plan([ok]).close()
    _expect(B.CKPT_EINVAL, [ok], direct_min_bytes=100)                        # below one alignment unit
    _expect(B.CKPT_EINVAL, [ok], direct_min_bytes=4096, window_policy=B.CKPT_WINDOW_PACK)
    _expect(B.CKPT_EINVAL, [("t", 9, (4,), FAKE_BASE, 16)])                   # unknown dtype
    _expect(B.CKPT_EINVAL, [("t", B.CKPT_F32, (4,), FAKE_BASE, 12)])          # nbytes != dtype x shape
    _expect(B.CKPT_EINVAL, [("t", B.CKPT_F32, (0,), FAKE_BASE, 0)])           # empty tensor
    _expect(B.CKPT_EINVAL, [("", B.CKPT_F32, (4,), FAKE_BASE, 16)])           # empty name
    _expect(B.CKPT_EINVAL, [("t", B.CKPT_F32, (4,), FAKE_BASE + 2, 16)])      # address not element aligned
    _expect(B.CKPT_EINVAL, [("t", B.CKPT_F32, (-4,), FAKE_BASE, 16)])         # negative dimension
    _expect(B.CKPT_EINVAL, [])                                                # nothing to register
    _expect(B.CKPT_EINVAL, [ok], dma_chunk_bytes=4096)                        # not a multiple of the tile size
    _expect(B.CKPT_EINVAL, [ok], dma_chunk_bytes=1 << 20, pack_superchunk_bytes=(1 << 20) + (64 << 10))
    _expect(B.CKPT_EINVAL, [ok], n_dma_streams=9)
    _expect(B.CKPT_EINVAL, [ok], window_policy=7)
    # scalars are allowed: empty shape, one element
    p = B.Plan([("s", B.CKPT_I64, (), FAKE_BASE, 8)])
    assert p.layout()["data_bytes"] == 4096
    p.close()


def test_find_latest_picks_the_newest_whole_file(tmp_path):
    """Restart helper on a directory of oracle-written files: passes over truncated files, files whose
    header names another iteration, temporary names and foreign files; no device involved."""
    g = np.random.default_rng(5)
    ts = [("a", B.CKPT_F32, (1000,), g.standard_normal(1000).astype(np.float32).view(np.uint8)),
          ("b", B.CKPT_U8, (77,), g.integers(0, 256, 77, dtype=np.uint8))]
    name = lambda it: os.path.join(tmp_path, "ckpt_iter%020d.dsl" % it)
    with pytest.raises(B.CkptError) as e:
        B.find_latest(str(tmp_path))
    assert e.value.code == B.CKPT_EINVAL
    for it in (3, 12, 40, 41, 50):
        oracle.serialize_file(ts, it, name(it))
    assert B.find_latest(str(tmp_path)) == (50, name(50))
    with open(name(50), "r+b") as f:                     # truncated: size disagrees with the header
        f.truncate(os.path.getsize(name(50)) - 4096)
    assert B.find_latest(str(tmp_path)) == (41, name(41))
    os.rename(name(41), name(60))                        # header says 41, name says 60
    assert B.find_latest(str(tmp_path)) == (40, name(40))
    oracle.serialize_file(ts, 70, name(70) + ".tmp")     # never committed
    open(os.path.join(tmp_path, "ckpt_iter00000000000000000099.dsl"), "wb").write(b"not a checkpoint" * 512)
    open(os.path.join(tmp_path, "notes.txt"), "w").write("x")
    assert B.find_latest(str(tmp_path)) == (40, name(40))
    with open(name(40), "r+b") as f:                     # damaged magic
        f.write(b"X")
    assert B.find_latest(str(tmp_path)) == (12, name(12))
    with pytest.raises(B.CkptError) as e:
        B.find_latest(str(tmp_path / "missing"))
    assert e.value.code == B.CKPT_EIO


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr) and "{" not in r.stdout


def test_bench_finds_the_measured_traffic_ratio_of_every_workload():
    """bench.py's `roofline.traffic` is the algorithmic bytes per launch times the HBM traffic ratio that the counter
    runs measured on the same workload; the summaries under profiles/ must hold one for each of the five workloads."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for config in (1, 2, 3, 4, 5):
        ratio = bench.traffic_ratio(config)
        assert ratio is not None and 0.99 < ratio < 1.02, (config, ratio)


def test_headers_compile_as_plain_c(tmp_path):
    """The boundary is a C ABI: both headers must be valid C99 on their own."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "hdr.c"
    src.write_text('#include "ckpt.h"\n#include "ckpt_proxy.h"\nint main(void) { ckpt_config c = {0}; (void)c; return 0; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"), "-fsyntax-only", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_describe_file_agrees_with_the_independent_reader(tmp_path):
    """The library's own reading of a file's tensor table against the test suite's struct-based reader, on
    an oracle-written file of the tiny fragmentation workload; damaged files are refused."""
    from tests import format_reader as fr
    spec = shards.make_shard(5, tiny=True)
    ts = [(t.name, t.dtype, t.shape, shards.host_values(spec, k)) for k, t in enumerate(spec.tensors)]
    ts.append(("scalar", B.CKPT_I64, (), np.arange(1, dtype=np.int64).view(np.uint8)))
    path = os.path.join(tmp_path, "ckpt_iter%020d.dsl" % 123)
    oracle.serialize_file(ts, 123, path)
    text = B.describe_file(path)
    lines = text.rstrip("\n").split("\n")
    it, table = fr.parse(open(path, "rb").read())
    head = lines[0].split()
    assert head[:4] == ["iter", str(it), "tensors", str(len(table))] and it == 123 and len(lines) == len(table) + 1
    names = {B.CKPT_BF16: "bf16", B.CKPT_F32: "f32", B.CKPT_F16: "f16", B.CKPT_U8: "u8", B.CKPT_I32: "i32", B.CKPT_I64: "i64"}
    for line, e in zip(lines[1:], table):
        name, dtype, shape, off, nb = line.split("\t")
        assert name == e["name"] and dtype == names[e["dtype"]] and int(off) == e["offset"] and int(nb) == e["nbytes"]
        assert shape == ("x".join(str(d) for d in e["shape"]) if e["shape"] else "-")
    with open(path, "r+b") as f:
        f.truncate(os.path.getsize(path) - 4096)
    with pytest.raises(B.CkptError) as e:
        B.describe_file(path)
    assert e.value.code == B.CKPT_EFORMAT
    with pytest.raises(B.CkptError) as e:
        B.describe_file(os.path.join(tmp_path, "missing.dsl"))
    assert e.value.code == B.CKPT_EIO


@pytest.mark.parametrize("tiny", [True, False])
@pytest.mark.parametrize("config", [1, 2, 3, 4])
def test_version_2_plan_matches_the_oracle(config, tiny):
    """The planner's version-2 header, offsets and sizes (derived tensors described, not stored) against the
    oracle's: byte-identical header on the tiny shards (taken from the oracle's whole version-2 file), sizes at
    full size; the tile table covers exactly the stored tensors."""
    spec = shards.make_shard(config, tiny=tiny)
    descs, span = _fake_descs(spec)
    pairs = [(k, k + 1) for k, t in enumerate(spec.tensors) if t.role == "p_bf16"]
    plan = B.Plan(descs, derived=pairs)
    lay = plan.layout()
    ots = [(t.name, t.dtype, t.shape, None) for t in spec.tensors]
    hb, db = oracle.v2_sizes(ots, pairs)
    assert (lay["version"], lay["header_bytes"], lay["data_bytes"]) == (2, hb, db)
    assert lay["n_derived_tensors"] == len(pairs) and lay["derived_bytes"] == sum(spec.tensors[d].nbytes for d, _ in pairs)
    assert lay["payload_bytes"] == spec.payload_bytes
    if tiny:
        host = [shards.host_values(spec, k) for k in range(len(spec.tensors))]
        blob, version = oracle.serialize_bytes_v2([(t.name, t.dtype, t.shape, h) for t, h in zip(spec.tensors, host)], 41, pairs)
        assert version == 2 and plan.header(41) == blob[:hb]
        # the tile table over a fake address space reproduces the oracle's version-2 data region
        mem = np.full(span + 64, 0xEE, dtype=np.uint8)
        for (name, dtype, shape, p, nb), v in zip(descs, host):
            mem[p - FAKE_BASE:p - FAKE_BASE + nb] = v
        out = np.full(db, 0xCC, dtype=np.uint8)
        pos = 0
        for t in plan.tiles():
            assert t.dst_off == pos
            s = t.src - FAKE_BASE
            out[pos:pos + t.copy_bytes] = mem[s:s + t.copy_bytes]
            out[pos + t.copy_bytes:pos + t.total_bytes] = 0
            pos += t.total_bytes
        assert pos == db and out.tobytes() == blob[hb:]
        offs = plan.offsets()
        assert all(offs[d] == 0 for d, _ in pairs) and offs[1] == hb
    plan.close()
    # malformed declarations are refused by the planner
    for wrong in ([(1, 0)], [(0, 1), (0, 1)], [(0, len(descs) + 5)]):
        with pytest.raises(B.CkptError) as e:
            B.Plan(descs, derived=wrong)
        assert e.value.code == B.CKPT_EINVAL
