"""ctypes binding of libdsllm_ckpt.so: same names as the C ABI (include/ckpt.h, include/ckpt_proxy.h),
argument marshalling only. There is no fallback: if the library has not been built, importing this
module raises."""
import ctypes as C
import os

# The library must use the same HIP runtime as whoever owns the device memory and the streams it is
# handed; one process must never hold two HIP runtimes. libdsllm_ckpt.so binds to whichever
# libamdhip64 is already loaded, else to the system one (/opt/rocm). A caller that also uses PyTorch,
# which ships a runtime of its own, must import torch BEFORE this module. The harness, tests and
# benchmark of this repository do not use PyTorch at all and so run on the system runtime.

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdsllm_ckpt.so")

CKPT_OK, CKPT_EINVAL, CKPT_ENOMEM, CKPT_EIO, CKPT_EHIP, CKPT_ESTATE, CKPT_EFORMAT, CKPT_EMISMATCH = 0, -1, -2, -3, -4, -5, -6, -7
CKPT_BF16, CKPT_F32, CKPT_F16, CKPT_U8, CKPT_I32, CKPT_I64 = 1, 2, 3, 4, 5, 6
CKPT_WINDOW_D2H, CKPT_WINDOW_PACK = 0, 1
CKPT_IO_AUTO, CKPT_IO_PWRITE, CKPT_IO_MMAP = 0, 1, 2
CKPT_ITER_ALL = 0xFFFFFFFFFFFFFFFF
_STATUS_NAMES = {0: "CKPT_OK", -1: "CKPT_EINVAL", -2: "CKPT_ENOMEM", -3: "CKPT_EIO", -4: "CKPT_EHIP", -5: "CKPT_ESTATE",
                 -6: "CKPT_EFORMAT", -7: "CKPT_EMISMATCH"}


class ckpt_tensor_desc(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dtype", C.c_int32), ("ndim", C.c_uint32), ("shape", C.POINTER(C.c_int64)),
                ("dev_ptr", C.c_void_p), ("nbytes", C.c_uint64)]


class ckpt_config(C.Structure):
    _fields_ = [("device", C.c_int32), ("out_dir", C.c_char_p), ("host_ring_bytes", C.c_uint64),
                ("dma_chunk_bytes", C.c_uint64), ("pack_superchunk_bytes", C.c_uint64), ("dev_staging_bytes", C.c_uint64),
                ("n_dma_streams", C.c_int32), ("n_io_threads", C.c_int32), ("window_policy", C.c_int32),
                ("o_direct", C.c_int32), ("fsync_on_commit", C.c_int32), ("io_mode", C.c_int32), ("keep_last", C.c_int32),
                ("prealloc_files", C.c_int32), ("direct_min_bytes", C.c_uint64), ("reserved", C.c_int32 * 2)]


class ckpt_layout(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("n_tensors", "header_bytes", "data_bytes", "file_bytes", "payload_bytes", "n_tiles",
                                          "n_chunks", "n_superchunks", "dma_chunk_bytes", "pack_superchunk_bytes", "tile_bytes",
                                          "n_segments", "n_direct_tensors", "direct_bytes", "direct_data_bytes",
                                          "n_host_objects", "host_bytes", "host_data_bytes", "version", "n_derived_tensors",
                                          "derived_bytes", "reduced_header_bytes", "reduced_data_bytes")]


class ckpt_tile(C.Structure):
    _fields_ = [("src", C.c_uint64), ("dst_off", C.c_uint64), ("copy_bytes", C.c_uint32), ("total_bytes", C.c_uint32),
                ("reserved", C.c_uint64)]


CKPT_SEG_STAGED, CKPT_SEG_DIRECT, CKPT_SEG_ZERO, CKPT_SEG_HOST = 0, 1, 2, 3
CKPT_PLACE_HOST = 0x100


class ckpt_segment(C.Structure):
    _fields_ = [("data_off", C.c_uint64), ("nbytes", C.c_uint64), ("src", C.c_uint64), ("kind", C.c_uint32), ("tensor", C.c_uint32)]


class ckpt_stats(C.Structure):
    _fields_ = [("iter", C.c_uint64), ("payload_bytes", C.c_uint64), ("data_bytes", C.c_uint64), ("file_bytes", C.c_uint64),
                ("d2h_done", C.c_int32), ("committed", C.c_int32), ("pack_launches", C.c_int32), ("tier2_state", C.c_int32),
                ("pack_ms_sum", C.c_double), ("request_to_d2h_end_ms", C.c_double), ("d2h_span_ms", C.c_double),
                ("request_to_pack_end_ms", C.c_double), ("host_submit_ms", C.c_double), ("host_request_to_commit_ms", C.c_double),
                ("host_backpressure_ms", C.c_double), ("host_snapshot_call_ms", C.c_double),
                ("host_flush_span_ms", C.c_double), ("host_io_wait_ms_sum", C.c_double), ("host_io_copy_ms_sum", C.c_double),
                ("host_tier2_ms", C.c_double), ("format_version", C.c_int32), ("reserved0", C.c_int32), ("verify_ms", C.c_double),
                ("host_window_wait_ms", C.c_double), ("init_d2h_gbps", C.c_double)]

CKPT_TIER2_NEWEST, CKPT_TIER2_EVERY = 0, 1
CKPT_TIER2_NONE, CKPT_TIER2_QUEUED, CKPT_TIER2_COPYING, CKPT_TIER2_DONE, CKPT_TIER2_SKIPPED, CKPT_TIER2_FAILED = range(6)


class CkptError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"{_STATUS_NAMES.get(code, code)}: {text}")
        self.code = code
        self.text = text


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python paper_2406_10707_amd/build.py) first. There is no fallback path.")

lib = C.CDLL(LIB_PATH)

_vp, _u64, _i32 = C.c_void_p, C.c_uint64, C.c_int32
_SIGS = {
    "ckpt_plan_create": (C.c_int, [C.POINTER(ckpt_tensor_desc), C.c_size_t, C.POINTER(ckpt_config), C.POINTER(_vp)]),
    "ckpt_plan_create_derived": (C.c_int, [C.POINTER(ckpt_tensor_desc), C.c_size_t, C.POINTER(ckpt_config), C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_uint32), C.c_size_t, C.POINTER(_vp)]),
    "ckpt_plan_layout": (C.c_int, [_vp, C.POINTER(ckpt_layout)]),
    "ckpt_plan_header": (C.c_int, [_vp, _u64, _vp, _u64]),
    "ckpt_plan_offsets": (C.c_int, [_vp, C.POINTER(_u64), C.c_size_t]),
    "ckpt_plan_tiles": (C.c_int, [_vp, _u64, _u64, C.POINTER(ckpt_tile)]),
    "ckpt_plan_superchunk_tiles": (C.c_int, [_vp, C.POINTER(_u64), C.c_size_t]),
    "ckpt_plan_segments": (C.c_int, [_vp, _u64, _u64, C.POINTER(ckpt_segment)]),
    "ckpt_plan_chunk_segments": (C.c_int, [_vp, C.POINTER(_u64), C.c_size_t]),
    "ckpt_plan_destroy": (None, [_vp]),
    "ckpt_init": (C.c_int, [C.POINTER(ckpt_config), C.POINTER(_vp)]),
    "ckpt_declare_derived": (C.c_int, [_vp, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.c_size_t]),
    "ckpt_register_tensors": (C.c_int, [_vp, C.POINTER(ckpt_tensor_desc), C.c_size_t]),
    "ckpt_snapshot_async": (C.c_int, [_vp, _u64, _vp]),
    "ckpt_wait_immutable_window_end": (C.c_int, [_vp, _vp, _i32]),
    "ckpt_set_window_policy": (C.c_int, [_vp, _i32]),
    "ckpt_flush": (C.c_int, [_vp, _u64]),
    "ckpt_restore": (C.c_int, [_vp, C.c_char_p, _vp, C.POINTER(_u64)]),
    "ckpt_enable_second_tier": (C.c_int, [_vp, C.c_char_p, _i32, _i32, _i32, _i32]),
    "ckpt_wait_second_tier": (C.c_int, [_vp, _u64]),
    "ckpt_second_tier_file_name": (C.c_int, [_vp, _u64, C.c_char_p, C.c_size_t]),
    "ckpt_describe_file": (C.c_int, [C.c_char_p, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]),
    "ckpt_find_latest": (C.c_int, [C.c_char_p, C.POINTER(_u64), C.c_char_p, C.c_size_t]),
    "ckpt_pack_image": (C.c_int, [C.POINTER(ckpt_tensor_desc), C.c_size_t, _vp, _u64, _vp]),
    "ckpt_pack_image_noalloc": (C.c_int, [C.POINTER(ckpt_tensor_desc), C.c_size_t, _vp, _u64, _vp]),
    "ckpt_get_layout": (C.c_int, [_vp, C.POINTER(ckpt_layout)]),
    "ckpt_get_init_probe": (C.c_int, [_vp, C.POINTER(C.c_double)]),
    "ckpt_get_stats": (C.c_int, [_vp, _u64, C.POINTER(ckpt_stats)]),
    "ckpt_file_name": (C.c_int, [_vp, _u64, C.c_char_p, C.c_size_t]),
    "ckpt_last_error": (C.c_char_p, []),
    "ckpt_destroy": (C.c_int, [_vp]),
    "proxy_gemm_bf16": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _i32, _vp]),
    "proxy_fill_state": (C.c_int, [_vp, _vp, _vp, _vp, _u64, _u64, _u64, _vp]),
    "proxy_adam_step": (C.c_int, [_vp, _vp, _vp, _vp, _u64, _u64, _u64, _u64, C.c_float, C.c_float, C.c_float, C.c_float, _vp]),
    "proxy_fill_words": (C.c_int, [_vp, _u64, _u64, _vp]),
    "proxy_mutate_words": (C.c_int, [_vp, _u64, _u64, _vp]),
    "proxy_devcopy": (C.c_int, [_vp, _vp, _u64, _vp]),
    "proxy_device_alloc": (C.c_int, [_u64, C.POINTER(_vp)]),
    "proxy_device_free": (C.c_int, [_vp]),
    "proxy_host_alloc_pinned": (C.c_int, [_u64, C.POINTER(_vp)]),
    "proxy_host_free_pinned": (C.c_int, [_vp]),
    "proxy_copy_h2d": (C.c_int, [_vp, _vp, _u64]),
    "proxy_copy_d2h": (C.c_int, [_vp, _vp, _u64]),
    "proxy_copy_d2d_async": (C.c_int, [_vp, _vp, _u64, _vp]),
    "proxy_copy_pinned_async": (C.c_int, [_vp, _vp, _u64, _i32, _vp]),
    "proxy_device_fill_async": (C.c_int, [_vp, _i32, _u64, _vp]),
    "proxy_stream_synchronize": (C.c_int, [_vp]),
    "proxy_device_synchronize": (C.c_int, []),
    "proxy_event_create": (C.c_int, [C.POINTER(_vp)]),
    "proxy_event_destroy": (C.c_int, [_vp]),
    "proxy_event_record": (C.c_int, [_vp, _vp]),
    "proxy_event_synchronize": (C.c_int, [_vp]),
    "proxy_event_elapsed_ms": (C.c_int, [_vp, _vp, C.POINTER(C.c_float)]),
    "proxy_device_info": (C.c_int, [C.c_char_p, _u64, C.POINTER(_i32), C.POINTER(_u64), C.POINTER(_u64), C.POINTER(_i32)]),
    "proxy_stream_create": (C.c_int, [C.POINTER(_vp)]),
    "proxy_stream_destroy": (C.c_int, [_vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)      # raises if the library does not export the symbol
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED = tuple(_SIGS)


def _check(rc):
    if rc != 0:
        raise CkptError(rc, (lib.ckpt_last_error() or b"").decode("utf-8", "replace"))


def _struct_dict(s):
    return {n: getattr(s, n) for n, _ in s._fields_ if not n.startswith("reserved")}


def make_config(out_dir="", device=0, host_ring_bytes=0, dma_chunk_bytes=0, pack_superchunk_bytes=0, dev_staging_bytes=0,
                n_dma_streams=0, n_io_threads=0, window_policy=CKPT_WINDOW_D2H, o_direct=0, fsync_on_commit=0,
                io_mode=CKPT_IO_AUTO, keep_last=0, prealloc_files=0, direct_min_bytes=0):
    cfg = ckpt_config()
    cfg.device = device
    cfg.out_dir = os.fsencode(out_dir) if out_dir else None
    cfg.host_ring_bytes = host_ring_bytes
    cfg.dma_chunk_bytes = dma_chunk_bytes
    cfg.pack_superchunk_bytes = pack_superchunk_bytes
    cfg.dev_staging_bytes = dev_staging_bytes
    cfg.n_dma_streams = n_dma_streams
    cfg.n_io_threads = n_io_threads
    cfg.window_policy = window_policy
    cfg.o_direct = o_direct
    cfg.fsync_on_commit = fsync_on_commit
    cfg.io_mode = io_mode
    cfg.keep_last = keep_last
    cfg.prealloc_files = prealloc_files
    cfg.direct_min_bytes = direct_min_bytes
    return cfg


def make_descs(tensors):
    """tensors: iterable of (name, dtype_code, shape, dev_ptr, nbytes). Returns (ctypes array, keepalive list)."""
    tensors = list(tensors)
    arr = (ckpt_tensor_desc * max(1, len(tensors)))()
    keep = []
    for k, (name, dtype, shape, ptr, nbytes) in enumerate(tensors):
        shp = (C.c_int64 * max(1, len(shape)))(*[int(s) for s in shape])
        nm = name.encode("utf-8") if isinstance(name, str) else name
        keep += [shp, nm]
        arr[k] = ckpt_tensor_desc(nm, dtype, len(shape), C.cast(shp, C.POINTER(C.c_int64)), ptr, nbytes)
    return arr, keep


def describe_file(path):
    """ckpt_describe_file: the tensor table of a checkpoint file as text."""
    need = C.c_size_t(0)
    rc = lib.ckpt_describe_file(os.fsencode(path), None, 0, C.byref(need))
    if need.value == 0:
        _check(rc)
    buf = C.create_string_buffer(need.value)
    _check(lib.ckpt_describe_file(os.fsencode(path), buf, need.value, None))
    return buf.value.decode("utf-8", "replace")


def find_latest(directory):
    """ckpt_find_latest: (iteration, path) of the newest whole checkpoint file in `directory`."""
    it = _u64()
    buf = C.create_string_buffer(4096)
    _check(lib.ckpt_find_latest(os.fsencode(directory), C.byref(it), buf, 4096))
    return it.value, os.fsdecode(buf.value)


def pack_image(tensors, dev_dst, dst_bytes, stream):
    """ckpt_pack_image: tensors as for register_tensors; the data-region image lands at device address dev_dst."""
    tensors = list(tensors)
    arr, keep = make_descs(tensors)
    _check(lib.ckpt_pack_image(arr, len(tensors), dev_dst, dst_bytes, stream))


def pack_image_noalloc(tensors, dev_dst, dst_bytes, stream):
    """ckpt_pack_image_noalloc: as pack_image, no allocation, returns without waiting for the stream."""
    tensors = list(tensors)
    arr, keep = make_descs(tensors)
    _check(lib.ckpt_pack_image_noalloc(arr, len(tensors), dev_dst, dst_bytes, stream))


def _pair_arrays(pairs):
    pairs = list(pairs)
    d = (C.c_uint32 * max(1, len(pairs)))(*[p[0] for p in pairs])
    s = (C.c_uint32 * max(1, len(pairs)))(*[p[1] for p in pairs])
    return d, s


class Plan:
    """ckpt_plan_*: layout, header, offsets and tile table of a tensor list, no device needed."""

    def __init__(self, tensors, cfg=None, derived=None):
        """derived: list of (derived index, source index): the version-2 plan (ckpt_plan_create_derived)."""
        cfg = cfg or make_config()
        tensors = list(tensors)
        arr, keep = make_descs(tensors)
        self._h = _vp()
        if derived is None:
            _check(lib.ckpt_plan_create(arr, len(tensors), C.byref(cfg), C.byref(self._h)))
        else:
            d, s = _pair_arrays(derived)
            _check(lib.ckpt_plan_create_derived(arr, len(tensors), C.byref(cfg), d, s, len(derived), C.byref(self._h)))

    def layout(self):
        out = ckpt_layout()
        _check(lib.ckpt_plan_layout(self._h, C.byref(out)))
        return _struct_dict(out)

    def header(self, it):
        n = self.layout()["header_bytes"]
        buf = C.create_string_buffer(n)
        _check(lib.ckpt_plan_header(self._h, it, buf, n))
        return buf.raw

    def offsets(self):
        n = self.layout()["n_tensors"]
        out = (_u64 * n)()
        _check(lib.ckpt_plan_offsets(self._h, out, n))
        return list(out)

    def tiles(self):
        n = self.layout()["n_tiles"]
        out = (ckpt_tile * n)()
        _check(lib.ckpt_plan_tiles(self._h, 0, n, out))
        return out

    def superchunk_tiles(self):
        n = self.layout()["n_superchunks"] + 1
        out = (_u64 * n)()
        _check(lib.ckpt_plan_superchunk_tiles(self._h, out, n))
        return list(out)

    def segments(self):
        n = self.layout()["n_segments"]
        out = (ckpt_segment * max(1, n))()
        _check(lib.ckpt_plan_segments(self._h, 0, n, out))
        return out[:n]

    def chunk_segments(self):
        n = self.layout()["n_chunks"] + 1
        out = (_u64 * n)()
        _check(lib.ckpt_plan_chunk_segments(self._h, out, n))
        return list(out)

    def close(self):
        if self._h:
            lib.ckpt_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


class Checkpointer:
    """One ckpt_ctx. Method names are the C entry points without the prefix."""

    def __init__(self, cfg):
        self._h = _vp()
        self._cfg = cfg
        _check(lib.ckpt_init(C.byref(cfg), C.byref(self._h)))

    def declare_derived(self, pairs):
        """ckpt_declare_derived: pairs = list of (derived index, source index), before register_tensors."""
        pairs = list(pairs)
        d, s = _pair_arrays(pairs)
        _check(lib.ckpt_declare_derived(self._h, d, s, len(pairs)))

    def register_tensors(self, tensors):
        tensors = list(tensors)
        arr, keep = make_descs(tensors)
        _check(lib.ckpt_register_tensors(self._h, arr, len(tensors)))

    def snapshot_async(self, it, stream):
        _check(lib.ckpt_snapshot_async(self._h, it, stream))

    def wait_immutable_window_end(self, stream, host_block=False):
        _check(lib.ckpt_wait_immutable_window_end(self._h, stream, 1 if host_block else 0))

    def set_window_policy(self, policy):
        _check(lib.ckpt_set_window_policy(self._h, policy))

    def flush(self, it=CKPT_ITER_ALL):
        _check(lib.ckpt_flush(self._h, it))

    def restore(self, path, stream):
        it = _u64(0)
        _check(lib.ckpt_restore(self._h, os.fsencode(path), stream, C.byref(it)))
        return it.value

    def layout(self):
        out = ckpt_layout()
        _check(lib.ckpt_get_layout(self._h, C.byref(out)))
        return _struct_dict(out)

    def init_probe(self):
        """ckpt_get_init_probe: GB/s of the timed device-to-host copy made by ckpt_init."""
        out = C.c_double(0)
        _check(lib.ckpt_get_init_probe(self._h, C.byref(out)))
        return out.value

    def stats(self, it):
        out = ckpt_stats()
        _check(lib.ckpt_get_stats(self._h, it, C.byref(out)))
        return _struct_dict(out)

    def enable_second_tier(self, directory, n_threads=0, o_direct=0, keep_last=1, mode=CKPT_TIER2_NEWEST):
        _check(lib.ckpt_enable_second_tier(self._h, os.fsencode(directory), n_threads, o_direct, keep_last, mode))

    def wait_second_tier(self, it=CKPT_ITER_ALL):
        _check(lib.ckpt_wait_second_tier(self._h, it))

    def second_tier_file_name(self, it):
        buf = C.create_string_buffer(4096)
        _check(lib.ckpt_second_tier_file_name(self._h, it, buf, 4096))
        return os.fsdecode(buf.value)

    def file_name(self, it):
        buf = C.create_string_buffer(4096)
        _check(lib.ckpt_file_name(self._h, it, buf, 4096))
        return os.fsdecode(buf.value)

    def destroy(self):
        if self._h:
            h, self._h = self._h, None
            _check(lib.ckpt_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _proxy(rc, what):
    if rc != 0:
        raise CkptError(rc, what + " failed")


def proxy_gemm_bf16(a, b, c, m, n, k, stream):
    _proxy(lib.proxy_gemm_bf16(a, b, c, m, n, k, stream), "proxy_gemm_bf16")


def proxy_fill_state(p, master, m, v, numel, seed, tensor, stream):
    _proxy(lib.proxy_fill_state(p, master, m, v, numel, seed, tensor, stream), "proxy_fill_state")


def proxy_adam_step(p, master, m, v, numel, seed, tensor, step, stream, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    _proxy(lib.proxy_adam_step(p, master, m, v, numel, seed, tensor, step, lr, beta1, beta2, eps, stream), "proxy_adam_step")


def proxy_fill_words(w, n_words, seed, stream):
    _proxy(lib.proxy_fill_words(w, n_words, seed, stream), "proxy_fill_words")


def proxy_mutate_words(w, n_words, step, stream):
    _proxy(lib.proxy_mutate_words(w, n_words, step, stream), "proxy_mutate_words")


def proxy_devcopy(dst, src, nbytes, stream):
    _proxy(lib.proxy_devcopy(dst, src, nbytes, stream), "proxy_devcopy")


def proxy_stream_create():
    out = _vp()
    _proxy(lib.proxy_stream_create(C.byref(out)), "proxy_stream_create")
    return out.value


def proxy_stream_destroy(stream):
    _proxy(lib.proxy_stream_destroy(stream), "proxy_stream_destroy")


def proxy_device_alloc(nbytes):
    out = _vp()
    _proxy(lib.proxy_device_alloc(nbytes, C.byref(out)), "proxy_device_alloc(%d)" % nbytes)
    return out.value


def proxy_device_free(ptr):
    _proxy(lib.proxy_device_free(ptr), "proxy_device_free")


def proxy_host_alloc_pinned(nbytes):
    out = _vp()
    _proxy(lib.proxy_host_alloc_pinned(nbytes, C.byref(out)), "proxy_host_alloc_pinned(%d)" % nbytes)
    return out.value


def proxy_host_free_pinned(ptr):
    _proxy(lib.proxy_host_free_pinned(ptr), "proxy_host_free_pinned")


def proxy_copy_h2d(dev, host, nbytes):
    _proxy(lib.proxy_copy_h2d(dev, host, nbytes), "proxy_copy_h2d")


def proxy_copy_d2h(host, dev, nbytes):
    _proxy(lib.proxy_copy_d2h(host, dev, nbytes), "proxy_copy_d2h")


def proxy_copy_d2d_async(dst, src, nbytes, stream):
    _proxy(lib.proxy_copy_d2d_async(dst, src, nbytes, stream), "proxy_copy_d2d_async")


def proxy_copy_pinned_async(dst, src, nbytes, to_host, stream):
    _proxy(lib.proxy_copy_pinned_async(dst, src, nbytes, 1 if to_host else 0, stream), "proxy_copy_pinned_async")


def proxy_device_fill_async(dev, byte, nbytes, stream):
    _proxy(lib.proxy_device_fill_async(dev, byte, nbytes, stream), "proxy_device_fill_async")


def proxy_stream_synchronize(stream):
    _proxy(lib.proxy_stream_synchronize(stream), "proxy_stream_synchronize")


def proxy_device_synchronize():
    _proxy(lib.proxy_device_synchronize(), "proxy_device_synchronize")


def proxy_event_create():
    out = _vp()
    _proxy(lib.proxy_event_create(C.byref(out)), "proxy_event_create")
    return out.value


def proxy_event_destroy(ev):
    _proxy(lib.proxy_event_destroy(ev), "proxy_event_destroy")


def proxy_event_record(ev, stream):
    _proxy(lib.proxy_event_record(ev, stream), "proxy_event_record")


def proxy_event_synchronize(ev):
    _proxy(lib.proxy_event_synchronize(ev), "proxy_event_synchronize")


def proxy_event_elapsed_ms(start, stop):
    ms = C.c_float(0)
    _proxy(lib.proxy_event_elapsed_ms(start, stop, C.byref(ms)), "proxy_event_elapsed_ms")
    return ms.value


def proxy_device_info():
    name = C.create_string_buffer(256)
    cus, ver = _i32(0), _i32(0)
    total, free = _u64(0), _u64(0)
    _proxy(lib.proxy_device_info(name, 256, C.byref(cus), C.byref(total), C.byref(free), C.byref(ver)), "proxy_device_info")
    return {"name": name.value.decode(), "compute_units": cus.value, "total_mem": total.value, "free_mem": free.value,
            "hip_runtime_version": ver.value}
