/*
 * libdsllm_ckpt — lazy asynchronous snapshot of one GPU's training-state shard (MI355X / gfx950).
 *
 * The operations follow the paper's system design: a pre-allocated, pre-pinned host cache that all
 * checkpoints reuse ("coalescing of shards to host memory"); device-to-host copies that overlap the
 * forward and backward passes, in which parameters and optimizer state are immutable, and that
 * must be over before the update mutates them ("lazy non-blocking copies"); flushing of every piece
 * to storage as soon as it is on the host, with back-pressure when the host cache is full
 * ("streamlined multi-level flushing"); and the three-phase save of the Implementation section
 * (tensor list -> header with a file offset per tensor -> asynchronous transfers and writes).
 * Here phases one and two run once, at registration.
 *
 * Plain C ABI: plain pointers and sizes only. "dev" pointers are device (HBM) addresses valid on
 * the context's GPU; every other pointer is a host pointer. A stream argument is a hipStream_t
 * passed as void*. All calls return a ckpt_status (0 = ok, negative = error) and never throw or
 * abort; ckpt_last_error() gives the text of the last error of the calling thread.
 *
 * File layout: docs/FORMAT.md (fixed 64-byte header, tensor table, 4 KiB-aligned data).
 */
#ifndef DSLLM_CKPT_H
#define DSLLM_CKPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ckpt_ctx ckpt_ctx;    /* opaque, library-owned */
typedef struct ckpt_plan ckpt_plan;  /* opaque, library-owned */

typedef enum {
    CKPT_OK = 0,
    CKPT_EINVAL = -1,    /* bad argument (null, zero-size tensor, nbytes != dtype x shape, bad config) */
    CKPT_ENOMEM = -2,    /* host or device allocation failed */
    CKPT_EIO = -3,       /* open/write/read/rename failed (also latched from the flush threads) */
    CKPT_EHIP = -4,      /* a HIP runtime call failed */
    CKPT_ESTATE = -5,    /* call out of order (see each function) */
    CKPT_EFORMAT = -6,   /* restore: not a well-formed checkpoint file */
    CKPT_EMISMATCH = -7  /* restore: file's tensor table differs from the registered tensors */
} ckpt_status;

typedef enum { CKPT_BF16 = 1, CKPT_F32 = 2, CKPT_F16 = 3, CKPT_U8 = 4, CKPT_I32 = 5, CKPT_I64 = 6 } ckpt_dtype;

/* Placement flag, OR'ed into ckpt_tensor_desc.dtype: the object lives in HOST memory (the paper's
 * heterogeneous state: host-resident tensors of an offloaded optimizer, and small non-tensor objects
 * such as generator state or serialized arguments, registered as CKPT_U8 blobs of a fixed size).
 * dev_ptr is then a host address. Such an object is read inside ckpt_snapshot_async, before the call
 * returns (the caller may change it right afterwards; nothing orders host memory with the stream), and
 * written inside ckpt_restore, before that call returns. It takes its place in the file like any
 * other tensor; the file does not record where a tensor lived. */
#define CKPT_PLACE_HOST 0x100

/* One tensor of the shard. Caller-owned; the library copies name and shape at registration.
 * dev_ptr must be aligned to the element size only. The memory must stay allocated, at this
 * address, for as long as the registration lives. */
typedef struct {
    const char *name;      /* UTF-8, NUL-terminated, 1..65535 bytes */
    int32_t dtype;         /* ckpt_dtype, optionally | CKPT_PLACE_HOST */
    uint32_t ndim;         /* 0..8; 0 = scalar */
    const int64_t *shape;  /* ndim entries, each >= 0 */
    void *dev_ptr;         /* device address of the first element (ignored by ckpt_plan_create) */
    uint64_t nbytes;       /* must equal elsize(dtype) * product(shape) and be > 0 */
} ckpt_tensor_desc;

/* when the update may start: after the last device-to-host copy of the pending snapshot (the
 * paper's rule), or as soon as the last pack kernel has read the tensors (the packed bytes then
 * sit in device staging memory, which only makes a difference when staging holds the whole shard
 * or its tail) */
typedef enum { CKPT_WINDOW_D2H = 0, CKPT_WINDOW_PACK = 1 } ckpt_window_policy;

/* how the I/O threads put a ring slot into the file: pwrite (serialised per file by the kernel for
 * buffered writes, but the only way with O_DIRECT), or stores into a shared mapping of the file
 * (parallel across threads; the choice for tmpfs and page-cache sinks). AUTO = mmap unless o_direct. */
typedef enum { CKPT_IO_AUTO = 0, CKPT_IO_PWRITE = 1, CKPT_IO_MMAP = 2 } ckpt_io_mode;

/* Zero in a size/count field selects the default given in the comment. */
typedef struct {
    int32_t device;                 /* HIP device ordinal */
    const char *out_dir;            /* directory of the checkpoint files; must exist. File names carry the iteration
                                       only: one directory per context (per GPU, per rank) */
    uint64_t host_ring_bytes;       /* pinned host ring; the paper's one knob. default 8 GiB; rounded down to
                                       whole DMA chunks, at least 2 chunks */
    uint64_t dma_chunk_bytes;       /* one device-to-host copy and one ring slot. default 256 MiB; multiple of 32 KiB.
                                       Larger copies come closer to the link's rate (copies run one after the other with
                                       a fixed gap between two); smaller ones start the pipeline sooner, which a shard
                                       of only a few GB notices (64 MiB suits those) */
    uint64_t pack_superchunk_bytes; /* bytes one pack launch produces. default 1 GiB; multiple of dma_chunk_bytes */
    uint64_t dev_staging_bytes;     /* device staging; default 2 super-chunks; rounded down to whole super-chunks, at least 2
                                       (or the whole data region when that is smaller) */
    int32_t n_dma_streams;          /* default 2, at most 8 */
    int32_t n_io_threads;           /* host threads that write (and, on restore, read) ring slots. default 4, at most 64 */
    int32_t window_policy;          /* ckpt_window_policy */
    int32_t o_direct;               /* 1: open files with O_DIRECT (all offsets and sizes are 4 KiB multiples); data then
                                       passes through a 4 MiB bounce buffer per I/O thread, because the kernel does not
                                       accept the pinned ring's pages for direct I/O */
    int32_t fsync_on_commit;        /* 0 (default) or 1: the file is fsync'ed (and its mapping msync'ed) before the rename that
                                       commits it, and the directory is fsync'ed after it, so that a file ckpt_flush has
                                       reported survives a power loss. -1: no fsync at all (a memory file system as the
                                       sink, or measurements that must not include the disk's flush) */
    int32_t io_mode;                /* ckpt_io_mode */
    int32_t keep_last;              /* 0: every checkpoint file stays. K > 0: once a snapshot is committed only the K
                                       newest files keep their names; older ones are retired to hidden spare files whose
                                       pages the next snapshots overwrite in place (no page allocation on the write path,
                                       as with the host cache). K valid files plus one being written exist at a time. */
    int32_t prealloc_files;         /* spare files created, with all pages allocated, at registration (needs keep_last > 0) */
    uint64_t direct_min_bytes;      /* 0: every tensor goes through the pack kernel. N > 0: hybrid path (the paper's
                                       tensor-by-tensor copies for what is large, coalescing for what is small): a
                                       tensor of at least N bytes is copied by the DMA engines straight between its own
                                       device memory and the ring slot, without pack kernel or staging; only smaller
                                       tensors are packed. Needs window_policy CKPT_WINDOW_D2H (the copies read the
                                       tensors themselves). At least 4096 when set. */
    int32_t reserved[2];            /* must be zero */
} ckpt_config;

/* Sizes that follow from a tensor list and a configuration. */
typedef struct {
    uint64_t n_tensors;
    uint64_t header_bytes, data_bytes, file_bytes; /* docs/FORMAT.md */
    uint64_t payload_bytes;                        /* sum of nbytes, without padding */
    uint64_t n_tiles;                              /* pack work items (one wavefront each) */
    uint64_t n_chunks;                             /* DMA chunks per snapshot */
    uint64_t n_superchunks;                        /* pack launches per snapshot */
    uint64_t dma_chunk_bytes, pack_superchunk_bytes, tile_bytes;
    uint64_t n_segments;                           /* copy segments per snapshot (>= n_chunks) */
    uint64_t n_direct_tensors, direct_bytes;       /* tensors copied without the pack kernel, and their payload */
    uint64_t direct_data_bytes;                    /* the same tensors' share of the data region (payload + padding) */
    uint64_t n_host_objects, host_bytes;           /* host-resident objects (CKPT_PLACE_HOST) and their payload */
    uint64_t host_data_bytes;                      /* their share of the data region */
    uint64_t version;                              /* format version of the file this layout describes (1, or 2: derived tensors) */
    uint64_t n_derived_tensors, derived_bytes;     /* version 2: tensors described but not stored, and their payload */
    uint64_t reduced_header_bytes, reduced_data_bytes; /* of the version-2 file of the same registration (0: no pairs declared) */
} ckpt_layout;

/* One pack work item: `copy_bytes` bytes from device address `src` go to offset `dst_off` of the data
 * region (file offset minus header_bytes), followed by zero bytes up to `total_bytes`. dst_off and
 * total_bytes are multiples of 16; a tile never crosses a super-chunk boundary or a tensor boundary. */
typedef struct {
    uint64_t src;
    uint64_t dst_off;
    uint32_t copy_bytes;
    uint32_t total_bytes;
    uint64_t reserved;
} ckpt_tile;

/* One piece of a DMA chunk. The segments of a chunk partition it, in order. STAGED: the bytes come
 * from (go to, on restore) device staging, where the pack kernel put them; DIRECT: they are `nbytes`
 * bytes of a registered tensor at device address `src`; HOST: bytes of a host-resident object at host
 * address `src`, copied by the CPU; ZERO: the padding behind a DIRECT or HOST tensor, zero-filled in
 * the ring slot by the host and skipped on restore. Without direct_min_bytes and host-resident
 * objects every chunk is one STAGED segment. */
typedef enum { CKPT_SEG_STAGED = 0, CKPT_SEG_DIRECT = 1, CKPT_SEG_ZERO = 2, CKPT_SEG_HOST = 3 } ckpt_segment_kind;
typedef struct {
    uint64_t data_off;   /* offset in the data region */
    uint64_t nbytes;
    uint64_t src;        /* DIRECT: device address; HOST: host address; otherwise 0 */
    uint32_t kind;       /* ckpt_segment_kind */
    uint32_t tensor;     /* DIRECT, HOST, ZERO: registration index of the tensor; otherwise 0 */
} ckpt_segment;

/* What the second storage tier takes: the newest committed snapshot whenever it is free (a snapshot
 * still waiting when a newer one is committed is skipped; training is never held back), or every
 * snapshot (a new snapshot does not start before its predecessor is on its way to the second tier;
 * when that tier is slower than the checkpoint rate, training waits for it at the window, which is
 * the paper's behaviour for a full host cache). */
typedef enum { CKPT_TIER2_NEWEST = 0, CKPT_TIER2_EVERY = 1 } ckpt_tier2_mode;

/* Where a snapshot stands with respect to the second storage tier (ckpt_enable_second_tier). */
typedef enum {
    CKPT_TIER2_NONE = 0,     /* no second tier, or not committed to the first tier yet */
    CKPT_TIER2_QUEUED = 1,   /* committed; the newest snapshot waiting for the second tier */
    CKPT_TIER2_COPYING = 2,
    CKPT_TIER2_DONE = 3,     /* whole, fsync'ed and renamed in the second-tier directory */
    CKPT_TIER2_SKIPPED = 4,  /* a newer snapshot was committed before the second tier got to this one */
    CKPT_TIER2_FAILED = 5
} ckpt_tier2_state;

/* Per-snapshot measurements. Times in milliseconds on the device timeline (HIP events) unless
 * marked host. A field is -1 while not yet known. */
typedef struct {
    uint64_t iter;
    uint64_t payload_bytes, data_bytes, file_bytes;
    int32_t d2h_done, committed;      /* 1 once the last copy has landed / the file has its final name */
    int32_t pack_launches;
    int32_t tier2_state;              /* ckpt_tier2_state */
    double pack_ms_sum;               /* sum over pack launches of (end - start) on the pack stream */
    double request_to_d2h_end_ms;     /* boundary event on the caller's stream -> last copy done */
    double d2h_span_ms;               /* first copy start -> last copy done */
    double request_to_pack_end_ms;    /* boundary event -> last pack kernel done */
    double host_submit_ms;            /* host: request -> every pack and copy enqueued (includes ring back-pressure) */
    double host_request_to_commit_ms; /* host: request -> file renamed */
    double host_backpressure_ms;      /* host: time the submit thread spent waiting for a free ring slot */
    double host_snapshot_call_ms;     /* host: time the caller spent inside ckpt_snapshot_async */
    double host_flush_span_ms;        /* host: first chunk on the host -> file renamed (the flush proper) */
    double host_io_wait_ms_sum;       /* host: summed over I/O threads, time waiting for chunks' copy events */
    double host_io_copy_ms_sum;       /* host: summed over I/O threads, time writing ring slots to the file */
    double host_tier2_ms;             /* host: copy of the committed file to the second tier, open to rename (-1: none yet) */
    int32_t format_version;           /* 1 or 2 (docs/FORMAT.md); 0 while not yet decided */
    int32_t reserved0;                /* zero */
    double verify_ms;                 /* device time of the derived-tensor check that decides the version (-1: no pairs declared) */
    double host_window_wait_ms;       /* host: time the caller spent inside ckpt_wait_immutable_window_end for this snapshot */
    double init_d2h_gbps;             /* the context's set-up probe (ckpt_get_init_probe), repeated here */
} ckpt_stats;

#define CKPT_ITER_ALL UINT64_MAX

/* ---- planning without a device (also used internally by registration) ---- */

/* Computes header, offsets, tile table and chunk table for a tensor list; dev_ptr values are taken
 * as given and never dereferenced. CKPT_EINVAL on a bad description or configuration. */
int ckpt_plan_create(const ckpt_tensor_desc *tensors, size_t n, const ckpt_config *cfg, ckpt_plan **out);
int ckpt_plan_layout(const ckpt_plan *plan, ckpt_layout *out);
/* The same for format version 2 (docs/FORMAT.md, derived tensors): tensor derived[i] (bf16) is declared to be the
 * round-to-nearest-even of tensor source[i] (f32, same shape, both device-resident) and gets a table entry but no
 * place in the data region. CKPT_EINVAL for a malformed pair list. */
int ckpt_plan_create_derived(const ckpt_tensor_desc *tensors, size_t n, const ckpt_config *cfg, const uint32_t *derived,
                             const uint32_t *source, size_t n_pairs, ckpt_plan **out);
/* Copies the header_bytes bytes of the header for iteration `iter` into buf (cap >= header_bytes). */
int ckpt_plan_header(const ckpt_plan *plan, uint64_t iter, void *buf, uint64_t cap);
/* File offset of every tensor, in registration order (cap >= n_tensors entries). */
int ckpt_plan_offsets(const ckpt_plan *plan, uint64_t *out, size_t cap);
/* Copies tiles [first, first+count) into out; first_tile_of_superchunk (n_superchunks+1 entries) may be NULL. */
int ckpt_plan_tiles(const ckpt_plan *plan, uint64_t first, uint64_t count, ckpt_tile *out);
int ckpt_plan_superchunk_tiles(const ckpt_plan *plan, uint64_t *first_tile_of_superchunk, size_t cap);
/* Copies segments [first, first+count) into out; first_segment_of_chunk takes n_chunks+1 entries. */
int ckpt_plan_segments(const ckpt_plan *plan, uint64_t first, uint64_t count, ckpt_segment *out);
int ckpt_plan_chunk_segments(const ckpt_plan *plan, uint64_t *first_segment_of_chunk, size_t cap);
void ckpt_plan_destroy(ckpt_plan *plan);

/* ---- the snapshot path ---- */

/* Allocates and pins the host ring once, touches every page, creates streams, events and threads.
 * Hidden spare files (retention) that a process which no longer exists left in out_dir are removed.
 * The ring is reused by every later snapshot and restore (paper: pre-allocated, pre-pinned cache). */
int ckpt_init(const ckpt_config *cfg, ckpt_ctx **out);

/* The first two phases of the paper's three-phase save (Implementation section: list the tensors, compute
 * the header with a file offset for each), done once instead of at every checkpoint, plus the set-up of the
 * "coalescing of shards" design principle on the device side.
 * Registers the shard's tensors, once per context: builds header, file offsets, the tile table
 * (uploaded to the device) and the chunk and copy-segment tables, allocates device staging and
 * pre-allocates the spare files the configuration asks for. Every device range is checked to be
 * memory of this GPU (CKPT_EINVAL otherwise). CKPT_ESTATE if tensors are already registered.
 * Overlapping device ranges are allowed (serialized twice). */
int ckpt_register_tensors(ckpt_ctx *ctx, const ckpt_tensor_desc *tensors, size_t n);

/* Data reduction, the future work the paper's Conclusions name (and the limitation its Introduction states: link
 * and storage cannot keep up with the checkpoint rate), in a first lossless form (docs/FORMAT.md, version 2).
 * Declares that registered tensor derived[i] (bf16) is kept by the training loop as the round-to-nearest-even of
 * tensor source[i] (f32, same shape): the working copy and the master weights of mixed-precision training, 2 of
 * 14 bytes per parameter. To be called after ckpt_init and before ckpt_register_tensors (indices refer to the list
 * registered afterwards, where they are checked: CKPT_EINVAL there). From then on every snapshot first checks on
 * the device, on the captured state, that every declared pair holds element for element (integer arithmetic on
 * the bit patterns, 6 bytes per parameter read once); if so the file is version 2 and the derived tensors are
 * neither packed, nor copied, nor written; if any element differs the snapshot is an ordinary version-1 file.
 * Either way a restore returns exactly the captured bytes: ckpt_restore reads both versions and recomputes the
 * derived tensors on the device. Host-resident objects cannot take part. CKPT_ESTATE after registration. */
int ckpt_declare_derived(ckpt_ctx *ctx, const uint32_t *derived, const uint32_t *source, size_t n_pairs);

/* A checkpoint request as the "lazy non-blocking copies" design principle defines it: it returns at once,
 * the copies run while the next forward and backward passes leave the state untouched (the paper's section on
 * the immutability of parameters and optimizer state), and a full host cache delays the copies, not the caller.
 * Requests the snapshot of iteration `iter`: the state captured is what the tensors hold once all
 * work already enqueued on `hip_stream_compute` has run. Returns without waiting for any copy; the
 * caller goes on with the next forward/backward pass. Pack kernels, copies and file writes are
 * issued by library threads; if the ring is full they wait for flushed slots (never for the
 * caller). A library thread waits, on the host, until the device has reached this point of the stream, and issues
 * the snapshot's kernels and copies only then (work parked in other queues behind an event that has not fired
 * slows every kernel launch of the caller's stream): the stream must get there without further calls into the
 * library. CKPT_ESTATE: nothing registered, or a previous snapshot's window was never closed with
 * ckpt_wait_immutable_window_end / ckpt_flush, or `iter` is still in flight. A latched I/O error of
 * an earlier snapshot is returned here (CKPT_EIO / CKPT_EHIP) and cleared. */
int ckpt_snapshot_async(ckpt_ctx *ctx, uint64_t iter, void *hip_stream_compute);

/* The one call a conventional save/load engine does not have: to be made before the update that
 * mutates the registered tensors. Orders all later work on `hip_stream_compute` after the pending
 * snapshot's last read of the tensors (per window_policy) with a device-side wait; with
 * host_block != 0 it also blocks the calling thread until then. The host is blocked in any case
 * until the library has enqueued all of the snapshot's copies, which takes longer than a moment
 * only when the ring is smaller than the shard and the flush is behind. No-op without a pending
 * snapshot. Does not wait for file writes: those may overlap the update. */
int ckpt_wait_immutable_window_end(ckpt_ctx *ctx, void *hip_stream_compute, int32_t host_block);

/* Changes the window policy (ckpt_window_policy) for later snapshots (a snapshot keeps the policy
 * that was in force when it was requested). CKPT_ESTATE while a snapshot's window is open;
 * CKPT_EINVAL for CKPT_WINDOW_PACK on a context with direct_min_bytes set. */
int ckpt_set_window_policy(ckpt_ctx *ctx, int32_t policy);

/* The end of the "streamlined multi-level flushing" design principle (every piece goes from the host cache to
 * storage as soon as it has arrived) and the single-participant form of the paper's asynchronous distributed
 * consolidation: a checkpoint counts once all of it is on storage under its final name.
 * Blocks until the file of `iter` (or of every requested snapshot, CKPT_ITER_ALL) is written, fsync'ed
 * (unless fsync_on_commit is -1) and renamed to its final name. Returns the latched asynchronous error, if
 * any, and clears it; a snapshot that failed (its file then never gets its final name and is removed) also
 * reports its own failure whenever it is asked about by `iter`, even after another call has taken the
 * latched error. CKPT_EINVAL if `iter` was never requested. */
int ckpt_flush(ckpt_ctx *ctx, uint64_t iter);

/* The way back, which the paper names only as the purpose of a checkpoint (Background: resuming after a
 * failure); it runs the snapshot path in reverse through the same host cache.
 * Reads a checkpoint file back into the registered tensors: header checked against the
 * registration (CKPT_EFORMAT / CKPT_EMISMATCH), data read into ring slots by the I/O threads,
 * copied host-to-device into staging, scattered by a kernel (tensors that the hybrid path copies
 * directly are written by the DMA engines straight from the ring slot; host-resident objects by
 * the calling thread). Returns when everything is enqueued (the file has been read by then);
 * `hip_stream` is made to wait for the last scatter kernel and the last copy. The path may lie in
 * either storage tier. iter_out may be NULL. CKPT_ESTATE while a snapshot is in flight. */
int ckpt_restore(ckpt_ctx *ctx, const char *path, void *hip_stream, uint64_t *iter_out);

/* The paper's multi-level flush, one level further: out_dir is the fast tier (host memory file system
 * or node-local NVMe) that absorbs checkpoints at the speed of the host link; every file committed
 * there is then copied, by a thread of its own and without holding up training or later snapshots,
 * to `dir` on slower, durable storage (n_threads writers, default 4, each moving 8 MiB blocks;
 * o_direct != 0 opens the copy with O_DIRECT and writes straight out of the first tier's mapping when
 * there is one; always fsync'ed before it gets its final name, the same
 * name as in out_dir). mode (ckpt_tier2_mode) NEWEST: the slower tier takes the newest committed
 * snapshot whenever it is free; one that is still waiting when a newer one is committed is skipped
 * (CKPT_TIER2_SKIPPED), so the second tier lags by at most one copy and never delays training. EVERY:
 * no snapshot is skipped; the wait for the slower tier shows up in host_backpressure_ms. With retention in the fast tier (keep_last > 0) the file being
 * copied is exempt from recycling until the copy is over. keep_last here: second-tier files kept
 * (0: all). To be called after ckpt_init and before the first snapshot; CKPT_ESTATE otherwise. */
int ckpt_enable_second_tier(ckpt_ctx *ctx, const char *dir, int32_t n_threads, int32_t o_direct, int32_t keep_last, int32_t mode);
/* Blocks until the snapshot of `iter` is durable in the second tier (CKPT_OK), was skipped
 * (CKPT_ESTATE) or failed; with CKPT_ITER_ALL until the second tier has nothing left to do. Failures
 * of second-tier copies are kept apart from those of the snapshot path: the first one is returned
 * here (CKPT_EIO) and cleared, or by ckpt_destroy; ckpt_flush and ckpt_snapshot_async never report them. */
int ckpt_wait_second_tier(ckpt_ctx *ctx, uint64_t iter);
/* Writes "<second-tier dir>/ckpt_iter<20 digits>.dsl" into buf. */
int ckpt_second_tier_file_name(ckpt_ctx *ctx, uint64_t iter, char *buf, size_t cap);

/* Restart helper, no context and no device needed: looks through `dir` for files named like the
 * library's own ("ckpt_iter<20 digits>.dsl") and returns the one with the highest iteration number
 * that is whole: magic, version and alignment as in docs/FORMAT.md, size fields consistent with each
 * other and with the file's size, iteration field equal to the name's. Files still under their
 * temporary name, truncated or foreign files are passed over. iter_out and path_buf may be NULL.
 * CKPT_EINVAL if nothing valid is there, CKPT_EIO if the directory cannot be read. Works for either
 * storage tier. */
int ckpt_find_latest(const char *dir, uint64_t *iter_out, char *path_buf, size_t cap);

/* The file describes itself: writes the tensor table of the checkpoint file at `path` into buf as text,
 * one line "iter <n> tensors <n> header_bytes <n> data_bytes <n>" and then one line per tensor,
 * "<name>\t<dtype>\t<d0>x<d1>...\t<file offset>\t<nbytes>" (dtype as in ckpt_dtype: bf16 f32 f16 u8 i32
 * i64; a scalar's shape is "-"). No context and no device needed. *needed_out (may be NULL) receives the
 * bytes the text takes including the terminating NUL; CKPT_EINVAL if cap is smaller (nothing is
 * written then, so a first call with cap 0 sizes the buffer). CKPT_EFORMAT for a file that is not a
 * whole checkpoint, CKPT_EIO if it cannot be read. */
int ckpt_describe_file(const char *path, char *buf, size_t cap, size_t *needed_out);

/* The pack step on its own, without a context (the paper's coalescing of a shard's many tensors into one
 * contiguous region, done here on the device instead of in host memory): gathers the n tensors, in order,
 * into the image of their checkpoint data region at device address dev_dst: tensor k's bytes at
 * sum over j < k of align_up(nbytes_j, 4096), zero bytes up to the next multiple of 4096 behind each, i.e.
 * the bytes a checkpoint file of these tensors holds from header_bytes on (docs/FORMAT.md). Of a descriptor
 * only dev_ptr (any byte alignment) and nbytes (> 0) are read; name, dtype and shape are ignored. Tensors
 * and destination must be device memory of the CURRENT device (hipSetDevice), inside their allocations;
 * dev_dst 16-byte aligned, dst_bytes at least the size of the data region; source and destination must
 * not overlap. The tile table the kernel walks is built on the device by a kernel of its own, in a
 * temporary device allocation: the call allocates, enqueues on hip_stream (after whatever is already
 * there), waits for the stream, and frees. CKPT_EINVAL for a bad argument (nothing is launched then),
 * CKPT_ENOMEM, CKPT_EHIP. */
int ckpt_pack_image(const ckpt_tensor_desc *tensors, size_t n, void *dev_dst, uint64_t dst_bytes, void *hip_stream);

/* ckpt_pack_image for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation. Same arguments, same image, same checks, but the tile table lives in a
 * static device array of the library (4 MiB per GPU, held until the process ends) instead of a temporary
 * allocation: the call makes no hipMalloc, hipFree or other allocating call, enqueues its kernels on
 * hip_stream and returns WITHOUT waiting for them (the image is complete when the stream gets there).
 * Limit: 131,072 tiles, i.e. about 4 GiB of data region (a tensor takes one tile per 32 KiB boundary it
 * touches, at least one); beyond it CKPT_EINVAL, nothing launched. Every call on a GPU shares that GPU's
 * table: calls on one stream are ordered and safe, calls that overlap on one GPU (different streams, or
 * threads) race and must be serialized by the caller. The table's address on a device is looked up on the
 * first call there, or by ckpt_init for its device: make that first call (or ckpt_init) outside any region
 * in which the runtime must not load code. */
int ckpt_pack_image_noalloc(const ckpt_tensor_desc *tensors, size_t n, void *dev_dst, uint64_t dst_bytes, void *hip_stream);

int ckpt_get_layout(ckpt_ctx *ctx, ckpt_layout *out);
/* ckpt_init copies one ring slot's worth (at most 64 MiB) from device memory into the pinned ring on a copy
 * stream (once untimed, then the best of three timed): *d2h_gbps is that rate in GB/s (-1 if it could not be measured). The paper's design rests on
 * a copy engine that moves checkpoints without taking compute resources from training; whether the copies of
 * this process go that way is a property of the HIP runtime it has loaded. On MI355X the system runtime reaches
 * about 56 GB/s here; a figure far below the link's rate means the runtime executes copies with kernels on the
 * compute units, and snapshots will both run slower and slow training down. One exception seen on MI355X boxes: for
 * the first second or so after ANOTHER process has released tens of GB of pinned or file memory, every pinned copy of a
 * new process runs at about half the link's rate (30 GB/s), this probe included; copies a second later are at full rate. */
int ckpt_get_init_probe(ckpt_ctx *ctx, double *d2h_gbps);
/* Measurements of one requested snapshot; CKPT_EINVAL if unknown (records of the 1024 most recent
 * requests are kept). Device-timeline fields are filled
 * once d2h_done is set. */
int ckpt_get_stats(ckpt_ctx *ctx, uint64_t iter, ckpt_stats *out);
/* Writes "<out_dir>/ckpt_iter<20 digits>.dsl" into buf. */
int ckpt_file_name(ckpt_ctx *ctx, uint64_t iter, char *buf, size_t cap);

/* Text of the calling thread's last error; library-owned, valid until that thread's next failing call. */
const char *ckpt_last_error(void);

/* Drains every pending snapshot (as ckpt_flush(ALL)) and the second tier, stops the threads, frees ring, staging,
 * streams and events. */
int ckpt_destroy(ckpt_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
