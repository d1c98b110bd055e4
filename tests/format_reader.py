"""A second, independent implementation of docs/FORMAT.md in pure Python `struct`: a writer that
builds the expected file byte by byte and a reader that parses and checks one. Written from the
format page only; it calls neither the oracle nor the HIP library, so it can pin both."""
import struct

A = 4096
ELSIZE = {1: 2, 2: 4, 3: 2, 4: 1, 5: 4, 6: 8}
MAGIC = b"DSLLMCK\x01"


def up(x):
    return -(-x // A) * A


def expected_file(tensors, it):
    """tensors: list of (name, dtype, shape, bytes). Returns the whole file as bytes."""
    entries = []
    for name, dtype, shape, data in tensors:
        nm = name.encode("utf-8")
        entries.append(2 + len(nm) + 1 + 1 + 8 * len(shape) + 8 + 8)
    header_bytes = up(64 + sum(entries))
    data_bytes = sum(up(len(d)) for _, _, _, d in tensors)
    out = bytearray()
    out += MAGIC
    out += struct.pack("<IIQQQQQQ", 1, A, it, len(tensors), header_bytes, data_bytes, header_bytes + data_bytes, 0)
    off = header_bytes
    for name, dtype, shape, data in tensors:
        nm = name.encode("utf-8")
        out += struct.pack("<H", len(nm)) + nm + struct.pack("<BB", dtype, len(shape))
        for s in shape:
            out += struct.pack("<q", s)
        out += struct.pack("<QQ", off, len(data))
        off += up(len(data))
    out += b"\x00" * (header_bytes - len(out))
    for name, dtype, shape, data in tensors:
        out += bytes(data)
        out += b"\x00" * (up(len(data)) - len(data))
    assert len(out) == header_bytes + data_bytes
    return bytes(out)


def bf16_rne(u):
    """FORMAT.md, version 2: bf16 rounding of an f32 bit pattern, on Python integers."""
    if (u & 0x7FFFFFFF) > 0x7F800000:
        return ((u >> 16) | 0x0040) & 0xFFFF
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF


def expected_file_v2(tensors, it, pairs):
    """Version 2: tensors as above, pairs = list of (derived index, source index); derived tensors are described, not stored."""
    ref = {d: s for d, s in pairs}
    entries = [2 + len(name.encode("utf-8")) + 1 + 1 + 8 * len(shape) + 8 + 8 + 1 + 4 for name, dtype, shape, data in tensors]
    header_bytes = up(64 + sum(entries))
    data_bytes = sum(up(len(d)) for k, (_, _, _, d) in enumerate(tensors) if k not in ref)
    out = bytearray()
    out += MAGIC
    out += struct.pack("<IIQQQQQQ", 2, A, it, len(tensors), header_bytes, data_bytes, header_bytes + data_bytes, 0)
    off = header_bytes
    for k, (name, dtype, shape, data) in enumerate(tensors):
        nm = name.encode("utf-8")
        out += struct.pack("<H", len(nm)) + nm + struct.pack("<BB", dtype, len(shape))
        for s in shape:
            out += struct.pack("<q", s)
        if k in ref:
            out += struct.pack("<QQBI", 0, len(data), 1, ref[k])
        else:
            out += struct.pack("<QQBI", off, len(data), 0, 0)
            off += up(len(data))
    out += b"\x00" * (header_bytes - len(out))
    for k, (name, dtype, shape, data) in enumerate(tensors):
        if k not in ref:
            out += bytes(data) + b"\x00" * (up(len(data)) - len(data))
    assert len(out) == header_bytes + data_bytes
    return bytes(out)


class FormatError(Exception):
    pass


def parse(buf):
    """Parse and check a whole file held in memory. Returns (iter, [dict(name,dtype,shape,offset,nbytes)])."""
    if len(buf) < 64 or buf[:8] != MAGIC:
        raise FormatError("magic")
    version, align, it, n, hb, db, fb, reserved = struct.unpack_from("<IIQQQQQQ", buf, 8)
    if version != 1 or align != A or reserved != 0:
        raise FormatError("fixed fields")
    if hb % A or fb != hb + db or fb != len(buf):
        raise FormatError("sizes")
    pos = 64
    table = []
    expect = hb
    for k in range(n):
        (ln,) = struct.unpack_from("<H", buf, pos); pos += 2
        name = buf[pos:pos + ln].decode("utf-8"); pos += ln
        dtype, ndim = struct.unpack_from("<BB", buf, pos); pos += 2
        shape = struct.unpack_from("<%dq" % ndim, buf, pos); pos += 8 * ndim
        off, nb = struct.unpack_from("<QQ", buf, pos); pos += 16
        if pos > hb:
            raise FormatError("table runs past header")
        numel = 1
        for s in shape:
            numel *= s
        if off != expect or off % A or nb == 0 or nb != numel * ELSIZE[dtype]:
            raise FormatError("entry %d" % k)
        table.append(dict(name=name, dtype=dtype, shape=tuple(shape), offset=off, nbytes=nb))
        expect += up(nb)
    if expect != fb:
        raise FormatError("data size")
    if any(buf[pos:hb]):
        raise FormatError("header padding not zero")
    for e in table:
        end = e["offset"] + e["nbytes"]
        if any(buf[end:e["offset"] + up(e["nbytes"])]):
            raise FormatError("tensor padding not zero: " + e["name"])
    return it, table
