"""Python face of the plain-C oracle (oracle_ckpt.c), plus the blocking per-tensor read-back that
feeds it. Test infrastructure only.

The oracle follows the paper's definition of a checkpoint (design principles, "lazy non-blocking
copies"; Implementation, three-phase save): the file of iteration i is the serialization of the
bytes every tensor holds after update i. It is the blocking baseline the paper calls the default
engine: stop, copy each tensor to the host, write header and tensors in order.

A tensor is described by (name, dtype_code, shape, host_bytes) where host_bytes is a contiguous
numpy uint8 array (or None for header-only calls).
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

_ELSIZE = {1: 2, 2: 4, 3: 2, 4: 1, 5: 4, 6: 8}
OK, BAD_ARG, IO, BAD_FILE, MISMATCH, NOMEM = 0, 1, 2, 3, 4, 5


class _Tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dtype", C.c_int32), ("ndim", C.c_uint32),
                ("shape", C.POINTER(C.c_int64)), ("host_bytes", C.c_void_p), ("nbytes", C.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build(force=False)
        L = C.CDLL(path)
        P = C.POINTER(_Tensor)
        L.oracle_header_bytes.restype = C.c_uint64
        L.oracle_header_bytes.argtypes = [P, C.c_size_t]
        L.oracle_data_bytes.restype = C.c_uint64
        L.oracle_data_bytes.argtypes = [P, C.c_size_t]
        L.oracle_tensor_offset.restype = C.c_uint64
        L.oracle_tensor_offset.argtypes = [P, C.c_size_t, C.c_size_t]
        L.oracle_build_header.restype = C.c_int
        L.oracle_build_header.argtypes = [P, C.c_size_t, C.c_uint64, C.c_void_p, C.c_uint64]
        L.oracle_serialize_file.restype = C.c_int
        L.oracle_serialize_file.argtypes = [P, C.c_size_t, C.c_uint64, C.c_char_p]
        L.oracle_serialize_mem.restype = C.c_int
        L.oracle_serialize_mem.argtypes = [P, C.c_size_t, C.c_uint64, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64)]
        L.oracle_compare_file.restype = C.c_int
        L.oracle_compare_file.argtypes = [P, C.c_size_t, C.c_uint64, C.c_char_p, C.POINTER(C.c_uint64)]
        L.oracle_compare_file_span.restype = C.c_int
        L.oracle_compare_file_span.argtypes = [P, C.c_size_t, C.c_uint64, C.c_size_t, C.c_size_t, C.c_char_p, C.POINTER(C.c_uint64)]
        U32P = C.POINTER(C.c_uint32)
        L.oracle_bf16_rne.restype = C.c_uint16
        L.oracle_bf16_rne.argtypes = [C.c_uint32]
        L.oracle_pairs_hold.restype = C.c_int
        L.oracle_pairs_hold.argtypes = [P, C.c_size_t, U32P, U32P, C.c_size_t]
        L.oracle_v2_sizes.restype = C.c_int
        L.oracle_v2_sizes.argtypes = [P, C.c_size_t, U32P, U32P, C.c_size_t, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.oracle_v2_serialize_mem.restype = C.c_int
        L.oracle_v2_serialize_mem.argtypes = [P, C.c_size_t, U32P, U32P, C.c_size_t, C.c_uint64, C.c_void_p, C.c_uint64,
                                              C.POINTER(C.c_uint64), U32P]
        L.oracle_v2_compare_file_span.restype = C.c_int
        L.oracle_v2_compare_file_span.argtypes = [P, C.c_size_t, U32P, U32P, C.c_size_t, C.c_uint32, C.c_uint64, C.c_size_t, C.c_size_t,
                                                  C.c_char_p, C.POINTER(C.c_uint64)]
        L.oracle_v2_restore_file.restype = C.c_int
        L.oracle_v2_restore_file.argtypes = [C.c_char_p, P, C.c_size_t, U32P, U32P, C.c_size_t, C.POINTER(C.c_uint64), U32P]
        L.oracle_restore_file.restype = C.c_int
        L.oracle_restore_file.argtypes = [C.c_char_p, P, C.c_size_t, C.POINTER(C.c_uint64)]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def _marshal(tensors):
    """tensors: list of (name, dtype_code, shape, host_bytes-or-None). Returns (array, keepalive)."""
    n = len(tensors)
    arr = (_Tensor * n)()
    keep = []
    for k, (name, dtype, shape, data) in enumerate(tensors):
        shp = (C.c_int64 * max(1, len(shape)))(*shape)
        numel = 1
        for s in shape:
            numel *= int(s)
        nbytes = numel * _ELSIZE.get(dtype, 0)
        nm = name.encode("utf-8")
        keep += [shp, nm]
        ptr = None
        if data is not None:
            a = np.ascontiguousarray(data).view(np.uint8).reshape(-1)
            if a.nbytes != nbytes:
                raise ValueError(f"tensor {name}: {a.nbytes} bytes given, dtype x shape says {nbytes}")
            keep.append(a)
            ptr = a.ctypes.data
        arr[k] = _Tensor(nm, dtype, len(shape), C.cast(shp, C.POINTER(C.c_int64)), ptr, nbytes)
    return arr, keep


def header_bytes(tensors):
    arr, keep = _marshal(tensors)
    return int(lib().oracle_header_bytes(arr, len(tensors)))


def data_bytes(tensors):
    arr, keep = _marshal(tensors)
    return int(lib().oracle_data_bytes(arr, len(tensors)))


def tensor_offsets(tensors):
    """File offset of every tensor (linear walk in C per tensor would be quadratic; done here from
    the first offset and the oracle's own data_bytes recurrence on prefixes only for small lists)."""
    arr, keep = _marshal(tensors)
    n = len(tensors)
    return [int(lib().oracle_tensor_offset(arr, n, k)) for k in range(n)]


def build_header(tensors, it):
    arr, keep = _marshal(tensors)
    hb = int(lib().oracle_header_bytes(arr, len(tensors)))
    out = np.empty(hb, dtype=np.uint8)
    rc = lib().oracle_build_header(arr, len(tensors), it, out.ctypes.data, hb)
    if rc:
        raise OracleError(rc, "build_header")
    return out.tobytes()


def serialize_file(tensors, it, path):
    arr, keep = _marshal(tensors)
    rc = lib().oracle_serialize_file(arr, len(tensors), it, os.fsencode(path))
    if rc:
        raise OracleError(rc, "serialize_file")


def serialize_bytes(tensors, it):
    arr, keep = _marshal(tensors)
    n = len(tensors)
    total = int(lib().oracle_header_bytes(arr, n)) + int(lib().oracle_data_bytes(arr, n))
    out = np.empty(total, dtype=np.uint8)
    written = C.c_uint64(0)
    rc = lib().oracle_serialize_mem(arr, n, it, out.ctypes.data, total, C.byref(written))
    if rc:
        raise OracleError(rc, "serialize_mem")
    assert written.value == total
    return out.tobytes()


def compare_file(tensors, it, path):
    """None when the file is exactly what the oracle would write, else the first differing offset."""
    arr, keep = _marshal(tensors)
    first = C.c_uint64(0)
    rc = lib().oracle_compare_file(arr, len(tensors), it, os.fsencode(path), C.byref(first))
    if rc == OK:
        return None
    if rc == MISMATCH:
        return int(first.value)
    raise OracleError(rc, "compare_file")


def _pairs(pairs):
    """pairs: list of (derived index, source index) -> two ctypes uint32 arrays and their length."""
    pairs = list(pairs or [])
    d = (C.c_uint32 * max(1, len(pairs)))(*[p[0] for p in pairs])
    s = (C.c_uint32 * max(1, len(pairs)))(*[p[1] for p in pairs])
    return d, s, len(pairs)


def bf16_rne(u):
    """The format's bf16 rounding of one f32 bit pattern (an int)."""
    return int(lib().oracle_bf16_rne(int(u) & 0xFFFFFFFF))


def pairs_hold(tensors, pairs):
    """True when every declared derived tensor is, element for element, bf16_rne of its source in the given bytes."""
    arr, keep = _marshal(tensors)
    d, s, n = _pairs(pairs)
    rc = lib().oracle_pairs_hold(arr, len(tensors), d, s, n)
    if rc < 0:
        raise OracleError(-rc, "pairs_hold")
    return bool(rc)


def v2_sizes(tensors, pairs):
    """(header_bytes, data_bytes) of the version-2 file of this tensor list and these pairs."""
    arr, keep = _marshal(tensors)
    d, s, n = _pairs(pairs)
    hb, db = C.c_uint64(0), C.c_uint64(0)
    rc = lib().oracle_v2_sizes(arr, len(tensors), d, s, n, C.byref(hb), C.byref(db))
    if rc:
        raise OracleError(rc, "v2_sizes")
    return int(hb.value), int(db.value)


def serialize_bytes_v2(tensors, it, pairs):
    """The file for a tensor list with declared (derived, source) pairs: (bytes, version). Version 2 when every
    pair holds in the given bytes, else the version-1 file."""
    arr, keep = _marshal(tensors)
    d, s, n = _pairs(pairs)
    total = int(lib().oracle_header_bytes(arr, len(tensors))) + int(lib().oracle_data_bytes(arr, len(tensors)))
    out = np.empty(total + 8 * len(tensors) + 4096, dtype=np.uint8)     # the version-2 header is a little longer, its data shorter
    written, version = C.c_uint64(0), C.c_uint32(0)
    rc = lib().oracle_v2_serialize_mem(arr, len(tensors), d, s, n, it, out.ctypes.data, out.nbytes, C.byref(written), C.byref(version))
    if rc:
        raise OracleError(rc, "v2_serialize_mem")
    return out[:written.value].tobytes(), int(version.value)


def restore_file_v2(path, tensors, pairs):
    """Restore with declared pairs; tensors carry writable host arrays. Returns (iter, version of the file)."""
    arr, keep = _marshal(tensors)
    d, s, n = _pairs(pairs)
    it, version = C.c_uint64(0), C.c_uint32(0)
    rc = lib().oracle_v2_restore_file(os.fsencode(path), arr, len(tensors), d, s, n, C.byref(it), C.byref(version))
    if rc:
        raise OracleError(rc, "v2_restore_file")
    return int(it.value), int(version.value)


class SpanComparer:
    """oracle_compare_file_span on a long tensor list, piece by piece: the list is marshalled once
    (names, dtypes, shapes), and every call supplies the host bytes of one run of tensors only.
    With pairs (format version 2) a derived tensor's bytes may be given as None when the expected version is 2."""

    def __init__(self, tensors, pairs=None):
        self._n = len(tensors)
        self._arr, self._keep = _marshal([(name, dtype, shape, None) for name, dtype, shape, _ in tensors])
        self._d, self._s, self._np = _pairs(pairs)

    def compare(self, it, first, arrays, path, version=1):
        """arrays: host bytes of tensors first, first+1, ...; returns None or the first differing file offset."""
        held = []
        for j, data in enumerate(arrays):
            if data is None:
                held.append(None)
                continue
            a = np.ascontiguousarray(data).view(np.uint8).reshape(-1)
            if a.nbytes != self._arr[first + j].nbytes:
                raise ValueError(f"tensor {first + j}: {a.nbytes} bytes given, {self._arr[first + j].nbytes} expected")
            held.append(a)
            self._arr[first + j].host_bytes = a.ctypes.data
        diff = C.c_uint64(0)
        try:
            rc = lib().oracle_v2_compare_file_span(self._arr, self._n, self._d, self._s, self._np, version, it, first, len(held),
                                                   os.fsencode(path), C.byref(diff))
        finally:
            for j in range(len(held)):
                self._arr[first + j].host_bytes = None
        if rc == OK:
            return None
        if rc == MISMATCH:
            return int(diff.value)
        raise OracleError(rc, "compare_file_span")


def restore_file(path, tensors):
    """tensors carry writable host arrays; they are overwritten with the file's bytes. Returns iter."""
    arr, keep = _marshal(tensors)
    it = C.c_uint64(0)
    rc = lib().oracle_restore_file(os.fsencode(path), arr, len(tensors), C.byref(it))
    if rc:
        raise OracleError(rc, "restore_file")
    return int(it.value)
