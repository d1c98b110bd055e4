// The snapshot engine behind the C ABI of include/ckpt.h.
//
// Threads: the caller (records the boundary event, never waits for copies), one submit thread
// (enqueues pack kernels and device-to-host copies, blocks on ring back-pressure so the caller does
// not), and n I/O threads (wait for a chunk's copy event, write the ring slot to the file, free the
// slot; on restore they read file chunks into ring slots). This is the producer/consumer circular
// host cache of the paper's design, with the device-to-host copies gated by HIP events.
#include "engine_internal.hpp"

using namespace dsllm;

thread_local std::string dsllm::g_last_error;

// Returns the latched asynchronous error of the snapshot path, if any, and clears it.
int dsllm::take_async_error(ckpt_ctx *c) {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->async_code == 0) return CKPT_OK;
    int code = c->async_code;
    g_last_error = c->async_err;
    c->async_code = 0;
    c->async_err.clear();
    return code;
}

// Creates a file of `bytes` zero bytes with every page allocated, reopened (and mapped) the way the flush uses it.
bool dsllm::preallocate_file(const std::string &path, uint64_t bytes, int n_threads, bool map_it, bool o_direct, FileSlot *out, std::string *err) {
    int fd = open(path.c_str(), O_RDWR | O_CREAT | O_TRUNC, 0644);
    if (fd < 0) { *err = path + ": open: " + strerror(errno); return false; }
    const uint64_t piece = 16ull << 20;
    std::vector<uint8_t> zeros(piece, 0);
    std::atomic<uint64_t> next{0};
    std::atomic<bool> ok{true};
    std::mutex emu;
    std::vector<std::thread> th;
    for (int t = 0; t < n_threads; t++)
        th.emplace_back([&] {
            for (;;) {
                uint64_t off = next.fetch_add(piece);
                if (off >= bytes || !ok) return;
                std::string e;
                if (!pwrite_all(fd, zeros.data(), std::min(piece, bytes - off), off, &e)) { std::lock_guard<std::mutex> lk(emu); *err = path + ": " + e; ok = false; }
            }
        });
    for (auto &t : th) t.join();
    close(fd);
    if (!ok) { unlink(path.c_str()); return false; }
    // reopen the way the flush will use it; with a mapping, fault every page in now
    out->path = path;
    out->bytes = bytes;
    out->fd = open(path.c_str(), (map_it ? O_RDWR : O_WRONLY) | (o_direct ? O_DIRECT : 0));
    if (out->fd < 0) { *err = path + ": open: " + strerror(errno); unlink(path.c_str()); return false; }
    if (map_it) {
        void *m = mmap(nullptr, bytes, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_POPULATE, out->fd, 0);
        if (m == MAP_FAILED) { *err = path + ": mmap: " + strerror(errno); close(out->fd); unlink(path.c_str()); return false; }
        out->map = static_cast<uint8_t *>(m);
        out->map_bytes = bytes;
    }
    return true;
}

// Spare files carry the process id of their owner in their name. Those of processes that no longer exist
// (a run that was killed) are removed: on a memory file system each of them holds a checkpoint's worth of RAM.
static void remove_stale_spares(const std::string &dir) {
    DIR *d = opendir(dir.c_str());
    if (!d) return;
    std::vector<std::string> stale;
    while (struct dirent *e = readdir(d)) {
        unsigned long pid = 0, seq = 0;
        int used = 0;
        if (sscanf(e->d_name, ".spare_%lu_%lu.dsl%n", &pid, &seq, &used) == 2 && used == int(strlen(e->d_name)) && pid > 0 &&
            pid != (unsigned long)getpid() && kill(pid_t(pid), 0) != 0 && errno == ESRCH)
            stale.push_back(dir + "/" + e->d_name);
    }
    closedir(d);
    for (const auto &p : stale) unlink(p.c_str());
}

// ------------------------------------------------------------------ C ABI

extern "C" {

const char *ckpt_last_error(void) { return g_last_error.c_str(); }

int ckpt_plan_create(const ckpt_tensor_desc *tensors, size_t n, const ckpt_config *cfg, ckpt_plan **out) {
    if (!cfg || !out) return fail(CKPT_EINVAL, "null argument");
    ResolvedConfig rc;
    std::string err;
    int r = resolve_config(cfg, &rc, &err);
    if (r) return fail(r, err);
    std::unique_ptr<ckpt_plan> p(new ckpt_plan);
    r = build_plan(tensors, n, rc, &p->plan, &err);
    if (r) return fail(r, err);
    *out = p.release();
    return CKPT_OK;
}

int ckpt_plan_create_derived(const ckpt_tensor_desc *tensors, size_t n, const ckpt_config *cfg, const uint32_t *derived, const uint32_t *source,
                             size_t n_pairs, ckpt_plan **out) {
    if (!cfg || !out || (n_pairs && (!derived || !source))) return fail(CKPT_EINVAL, "null argument");
    ResolvedConfig rc;
    std::string err;
    int r = resolve_config(cfg, &rc, &err);
    if (r) return fail(r, err);
    DerivedPairs dp;
    dp.derived.assign(derived, derived + n_pairs);
    dp.source.assign(source, source + n_pairs);
    std::unique_ptr<ckpt_plan> p(new ckpt_plan);
    r = build_plan(tensors, n, rc, &p->plan, &err, &dp, true);
    if (r) return fail(r, err);
    *out = p.release();
    return CKPT_OK;
}

static void fill_layout(const Plan &p, ckpt_layout *o) {
    o->n_tensors = p.tensors.size();
    o->header_bytes = p.header_bytes;
    o->data_bytes = p.data_bytes;
    o->file_bytes = p.file_bytes();
    o->payload_bytes = p.payload_bytes;
    o->n_tiles = p.tiles.size();
    o->n_chunks = p.n_chunks;
    o->n_superchunks = p.n_superchunks;
    o->dma_chunk_bytes = p.cfg.dma_chunk_bytes;
    o->pack_superchunk_bytes = p.cfg.pack_superchunk_bytes;
    o->tile_bytes = kTileBytes;
    o->n_segments = p.segs.size();
    o->n_direct_tensors = p.n_direct;
    o->direct_bytes = p.direct_bytes;
    o->direct_data_bytes = p.direct_data_bytes;
    o->n_host_objects = p.n_host;
    o->host_bytes = p.host_bytes;
    o->host_data_bytes = p.host_data_bytes;
    o->version = p.version;
    o->n_derived_tensors = p.n_derived;
    o->derived_bytes = p.derived_bytes;
    o->reduced_header_bytes = p.version == 2 ? p.header_bytes : 0;
    o->reduced_data_bytes = p.version == 2 ? p.data_bytes : 0;
}

int ckpt_plan_layout(const ckpt_plan *plan, ckpt_layout *out) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    fill_layout(plan->plan, out);
    return CKPT_OK;
}

int ckpt_plan_header(const ckpt_plan *plan, uint64_t iter, void *buf, uint64_t cap) {
    if (!plan || !buf) return fail(CKPT_EINVAL, "null argument");
    const Plan &p = plan->plan;
    if (cap < p.header_bytes) return fail(CKPT_EINVAL, "buffer smaller than header_bytes");
    memcpy(buf, p.header.data(), p.header_bytes);
    for (int i = 0; i < 8; i++) static_cast<uint8_t *>(buf)[16 + i] = uint8_t(iter >> (8 * i));
    return CKPT_OK;
}

int ckpt_plan_offsets(const ckpt_plan *plan, uint64_t *out, size_t cap) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    if (cap < plan->plan.tensors.size()) return fail(CKPT_EINVAL, "buffer smaller than n_tensors");
    for (size_t k = 0; k < plan->plan.tensors.size(); k++) out[k] = plan->plan.tensors[k].file_off;
    return CKPT_OK;
}

int ckpt_plan_tiles(const ckpt_plan *plan, uint64_t first, uint64_t count, ckpt_tile *out) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    const auto &t = plan->plan.tiles;
    if (first > t.size() || count > t.size() - first) return fail(CKPT_EINVAL, "tile range out of bounds");
    memcpy(out, t.data() + first, count * sizeof(ckpt_tile));
    return CKPT_OK;
}

int ckpt_plan_superchunk_tiles(const ckpt_plan *plan, uint64_t *out, size_t cap) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    const auto &v = plan->plan.sc_first_tile;
    if (cap < v.size()) return fail(CKPT_EINVAL, "buffer smaller than n_superchunks + 1");
    memcpy(out, v.data(), v.size() * sizeof(uint64_t));
    return CKPT_OK;
}

int ckpt_plan_segments(const ckpt_plan *plan, uint64_t first, uint64_t count, ckpt_segment *out) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    const auto &v = plan->plan.segs;
    if (first > v.size() || count > v.size() - first) return fail(CKPT_EINVAL, "segment range out of bounds");
    memcpy(out, v.data() + first, count * sizeof(ckpt_segment));
    return CKPT_OK;
}

int ckpt_plan_chunk_segments(const ckpt_plan *plan, uint64_t *out, size_t cap) {
    if (!plan || !out) return fail(CKPT_EINVAL, "null argument");
    const auto &v = plan->plan.chunk_first_seg;
    if (cap < v.size()) return fail(CKPT_EINVAL, "buffer smaller than n_chunks + 1");
    memcpy(out, v.data(), v.size() * sizeof(uint64_t));
    return CKPT_OK;
}

void ckpt_plan_destroy(ckpt_plan *plan) { delete plan; }

int ckpt_init(const ckpt_config *cfg, ckpt_ctx **out) {
    if (!cfg || !out) return fail(CKPT_EINVAL, "null argument");
    if (!cfg->out_dir || !*cfg->out_dir) return fail(CKPT_EINVAL, "config: out_dir is required");
    struct stat st;
    if (stat(cfg->out_dir, &st) != 0 || !S_ISDIR(st.st_mode)) return fail(CKPT_EIO, std::string(cfg->out_dir) + ": not a directory");
    ResolvedConfig rc;
    std::string err;
    int r = resolve_config(cfg, &rc, &err);
    if (r) return fail(r, err);
    int ndev = 0;
    HIP_TRY(nullptr, hipGetDeviceCount(&ndev));
    if (cfg->device < 0 || cfg->device >= ndev) return fail(CKPT_EINVAL, "config: no such device");
    HIP_TRY(nullptr, hipSetDevice(cfg->device));
    if ((r = pack_scratch_setup()) != CKPT_OK) return r;   // the static table of ckpt_pack_image_noalloc on this device

    std::unique_ptr<ckpt_ctx> c(new ckpt_ctx);
    c->cfg = rc;
    c->device = cfg->device;
    c->out_dir = cfg->out_dir;
    c->n_slots = rc.host_ring_bytes / rc.dma_chunk_bytes;
    remove_stale_spares(c->out_dir);
    trace("init: creating streams and events");
    c->slot_state.assign(c->n_slots, SLOT_FREE);
    c->slot_reads_left.assign(c->n_slots, 0);
    hipError_t e = hipSuccess;
    auto cleanup_fail = [&](int code, const std::string &m) { trace(("init: failed: " + m).c_str()); ckpt_destroy(c.release()); return fail(code, m); };
    if ((e = hipStreamCreateWithFlags(&c->pack_stream, hipStreamNonBlocking)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
    for (int k = 0; k < rc.n_dma_streams; k++) {
        hipStream_t s;
        if ((e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
        c->dma.push_back(s);
    }
    trace("init: streams created");
    for (uint64_t i = 0; i < c->n_slots; i++) {
        hipEvent_t ev;
        if ((e = hipEventCreateWithFlags(&ev, hipEventBlockingSync)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
        c->ev_slot.push_back(ev);
    }
    trace("init: slot events created");
    for (int k = 0; k < rc.n_dma_streams; k++) {
        hipEvent_t ev;
        if ((e = hipEventCreateWithFlags(&ev, hipEventBlockingSync)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
        c->ev_job_tail.push_back(ev);
    }
    for (int k = 0; k < kBoundaryEvents; k++) {   // one per snapshot in flight; none is created on the per-iteration path
        hipEvent_t ev;
        // blocking: the submit thread sleeps on a boundary until the device reaches it
        if ((e = hipEventCreateWithFlags(&ev, hipEventBlockingSync)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
        c->ev_boundary_free.push_back(ev);
    }
    if ((e = hipEventCreate(&c->ev_first_copy)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
    if ((e = hipEventCreate(&c->ev_user)) != hipSuccess) return cleanup_fail(CKPT_EHIP, hipGetErrorString(e));
    void *ring = nullptr;
    trace("init: allocating the pinned ring");
    e = hipHostMalloc(&ring, rc.host_ring_bytes, hipHostMallocDefault);
    trace("init: ring allocated, touching pages");
    if (e != hipSuccess) return cleanup_fail(CKPT_ENOMEM, std::string("hipHostMalloc(ring): ") + hipGetErrorString(e));
    c->ring = static_cast<uint8_t *>(ring);
    {   // touch every page now, in parallel, so no snapshot pays for first-touch page faults
        int nt = std::max(1, std::min(rc.n_io_threads, 16));
        std::vector<std::thread> th;
        uint64_t per = (rc.host_ring_bytes / 4096 + nt - 1) / nt * 4096;
        for (int i = 0; i < nt; i++)
            th.emplace_back([&, i] {
                uint64_t b = uint64_t(i) * per, e2 = std::min<uint64_t>(rc.host_ring_bytes, b + per);
                for (uint64_t o = b; o < e2; o += 4096) c->ring[o] = 0;
            });
        for (auto &t : th) t.join();
    }
    trace("init: pages touched");
    {   // One ring slot's worth of device-to-host copy, timed on a copy stream: tells the caller at what rate the HIP
        // runtime of this process moves pinned copies (the copy engines reach the link's rate; a runtime that
        // executes copies with kernels on the compute units does not, and takes the units from training).
        const size_t nb = size_t(std::min<uint64_t>(rc.dma_chunk_bytes, 64ull << 20));
        void *d = nullptr;
        hipEvent_t t0 = nullptr, t1 = nullptr;
        if (hipMalloc(&d, nb) == hipSuccess && hipEventCreate(&t0) == hipSuccess && hipEventCreate(&t1) == hipSuccess) {
            // one untimed copy (first use of the path), then the best of three timed ones: right after another process
            // has released tens of GB of pinned memory a single copy has been seen at half the link's rate
            bool ok = hipMemcpyAsync(c->ring, d, nb, hipMemcpyDeviceToHost, c->dma[0]) == hipSuccess;
            for (int rep = 0; ok && rep < 3; rep++) {
                float ms = 0;
                ok = hipEventRecord(t0, c->dma[0]) == hipSuccess;
                ok = ok && hipMemcpyAsync(c->ring, d, nb, hipMemcpyDeviceToHost, c->dma[0]) == hipSuccess;
                ok = ok && hipEventRecord(t1, c->dma[0]) == hipSuccess && hipEventSynchronize(t1) == hipSuccess;
                if (ok && hipEventElapsedTime(&ms, t0, t1) == hipSuccess && ms > 0)
                    c->init_d2h_gbps = std::max(c->init_d2h_gbps, double(nb) / (double(ms) * 1e6));
            }
        }
        (void)hipGetLastError();
        if (t0) (void)hipEventDestroy(t0);
        if (t1) (void)hipEventDestroy(t1);
        if (d) (void)hipFree(d);
    }
    trace("init: starting threads");
    c->submit_thread = std::thread(submit_thread_main, c.get());
    for (int i = 0; i < rc.n_io_threads; i++) c->io_threads.emplace_back(io_thread_main, c.get());
    *out = c.release();
    trace("init: done");
    return CKPT_OK;
}


int ckpt_register_tensors(ckpt_ctx *c, const ckpt_tensor_desc *tensors, size_t n) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    if (c->registered) return fail(CKPT_ESTATE, "tensors already registered in this context");
    HIP_TRY(c, hipSetDevice(c->device));
    for (size_t k = 0; tensors && k < n; k++)
        if (!tensors[k].dev_ptr) return fail(CKPT_EINVAL, "tensor " + std::to_string(k) + ": null device pointer");
    std::string err;
    Plan p, rp;
    const bool reduce = c->pairs.size() > 0;
    int r = build_plan(tensors, n, c->cfg, &p, &err, reduce ? &c->pairs : nullptr, false);
    if (r) return fail(r, err);
    if (reduce && (r = build_plan(tensors, n, c->cfg, &rp, &err, &c->pairs, true)) != CKPT_OK) return fail(r, err);
    // every source range must be device memory of this GPU: checked here, once, before any launch
    for (const auto &t : p.tensors) {
        if (t.host) continue;   // host-resident object: the caller vouches for the range
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, reinterpret_cast<void *>(t.dev_addr));
        if (e != hipSuccess || attr.type != hipMemoryTypeDevice || attr.device != c->device) {
            (void)hipGetLastError();
            return fail(CKPT_EINVAL, "tensor " + t.name + ": not device memory of this GPU");
        }
        void *base = nullptr; size_t span = 0;
        e = hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t *>(&base), &span, reinterpret_cast<hipDeviceptr_t>(t.dev_addr));
        if (e == hipSuccess && t.dev_addr + t.nbytes > uint64_t(base) + span)
            return fail(CKPT_EINVAL, "tensor " + t.name + ": range runs past its allocation");
        if (e != hipSuccess) (void)hipGetLastError();
    }
    // staging: whole super-chunks; no more than the data region needs
    uint64_t SC = c->cfg.pack_superchunk_bytes;
    uint64_t want = c->cfg.dev_staging_bytes / SC;
    if (want > p.n_superchunks) want = std::max<uint64_t>(p.n_superchunks, 1);
    c->n_stage = want;
    uint64_t stage_bytes = p.n_superchunks <= 1 ? std::max<uint64_t>(p.data_bytes, kAlign) : c->n_stage * SC;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&c->staging), stage_bytes);
    if (e != hipSuccess) return fail(CKPT_ENOMEM, std::string("hipMalloc(staging): ") + hipGetErrorString(e));
    e = hipMalloc(reinterpret_cast<void **>(&c->dev_tiles), p.tiles.size() * sizeof(ckpt_tile));
    if (e != hipSuccess) return fail(CKPT_ENOMEM, std::string("hipMalloc(tile table): ") + hipGetErrorString(e));
    HIP_TRY(c, hipMemcpy(c->dev_tiles, p.tiles.data(), p.tiles.size() * sizeof(ckpt_tile), hipMemcpyHostToDevice));
    if (reduce) {
        // the version-2 plan's tile table, the work items of the check, and the word its verdict lands in
        e = hipMalloc(reinterpret_cast<void **>(&c->dev_rtiles), std::max<size_t>(rp.tiles.size(), 1) * sizeof(ckpt_tile));
        if (e != hipSuccess) return fail(CKPT_ENOMEM, std::string("hipMalloc(tile table): ") + hipGetErrorString(e));
        HIP_TRY(c, hipMemcpy(c->dev_rtiles, rp.tiles.data(), rp.tiles.size() * sizeof(ckpt_tile), hipMemcpyHostToDevice));
        e = hipMalloc(reinterpret_cast<void **>(&c->dev_pairs), std::max<size_t>(p.pair_tiles.size(), 1) * sizeof(PairTile));
        if (e != hipSuccess) return fail(CKPT_ENOMEM, std::string("hipMalloc(pair table): ") + hipGetErrorString(e));
        HIP_TRY(c, hipMemcpy(c->dev_pairs, p.pair_tiles.data(), p.pair_tiles.size() * sizeof(PairTile), hipMemcpyHostToDevice));
        HIP_TRY(c, hipMalloc(reinterpret_cast<void **>(&c->dev_flag), 256));
        HIP_TRY(c, hipHostMalloc(reinterpret_cast<void **>(&c->host_flag), 4096, hipHostMallocDefault));
        *c->host_flag = 1;
        HIP_TRY(c, hipEventCreate(&c->ev_verify_start));
        HIP_TRY(c, hipEventCreate(&c->ev_verify_done));
        HIP_TRY(c, hipEventCreate(&c->ev_derived));
    }
    for (uint64_t s = 0; s < p.n_superchunks; s++) {
        hipEvent_t a, b, d;
        HIP_TRY(c, hipEventCreate(&a));
        HIP_TRY(c, hipEventCreate(&b));
        HIP_TRY(c, hipEventCreate(&d));
        c->ev_pack_start.push_back(a);
        c->ev_packed.push_back(b);
        c->ev_pack_end.push_back(d);
    }
    c->ev_stage_done.resize(c->n_stage);
    for (uint64_t s = 0; s < c->n_stage; s++)
        for (size_t k = 0; k < c->dma.size(); k++) {
            hipEvent_t ev;
            HIP_TRY(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming | hipEventBlockingSync));   // the submit thread sleeps on these
            c->ev_stage_done[s].push_back(ev);
        }
    if (posix_memalign(reinterpret_cast<void **>(&c->hdr_buf), 4096, std::max(p.header_bytes, reduce ? rp.header_bytes : 0)) != 0) return fail(CKPT_ENOMEM, "header buffer");
    c->plan = std::move(p);
    if (reduce) { c->rplan = std::move(rp); c->have_rplan = true; }
    c->registered = true;
    // spare files side by side: page allocation is serialized per file, not across files
    // with a second tier the file under copy there is exempt from recycling: one more file is in rotation
    const int n_spare = c->cfg.prealloc_files + (c->tier2_on && c->cfg.prealloc_files > 0 ? 1 : 0);
    std::vector<FileSlot> made(n_spare);
    std::vector<std::string> errs(n_spare);
    std::vector<char> ok(n_spare, 0);
    std::vector<std::thread> workers;
    for (int i = 0; i < n_spare; i++) {
        std::string spare = c->out_dir + "/.spare_" + std::to_string(getpid()) + "_" + std::to_string(c->spare_seq++) + ".dsl";
        workers.emplace_back([&, i, spare] {
            // sized for the file a snapshot is expected to be: version 2 when pairs are declared
            ok[i] = preallocate_file(spare, expected_file_bytes(c), std::min(c->cfg.n_io_threads, 8), c->cfg.io_mode == CKPT_IO_MMAP, c->cfg.o_direct,
                                     &made[i], &errs[i]);
        });
    }
    for (auto &w : workers) w.join();
    for (int i = 0; i < n_spare; i++)
        if (ok[i]) c->spares.push_back(made[i]);
    for (int i = 0; i < n_spare; i++)
        if (!ok[i]) return fail(CKPT_EIO, errs[i]);   // the spares that were made are removed by ckpt_destroy
    return CKPT_OK;
}

int ckpt_snapshot_async(ckpt_ctx *c, uint64_t iter, void *stream) {
    auto t0 = Clock::now();
    if (!c) return fail(CKPT_EINVAL, "null context");
    if (!c->registered) return fail(CKPT_ESTATE, "no tensors registered");
    if (iter == CKPT_ITER_ALL) return fail(CKPT_EINVAL, "iteration number reserved");
    int r = take_async_error(c);
    if (r) return r;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (c->restoring) return fail(CKPT_ESTATE, "restore in progress");
        if (c->tier2_enabling) return fail(CKPT_ESTATE, "the second tier is still being set up");
        if (c->last_snap && !c->last_snap->window_closed)
            return fail(CKPT_ESTATE, "previous snapshot's window was not closed (call ckpt_wait_immutable_window_end before the update)");
        auto it = c->snaps.find(iter);
        if (it != c->snaps.end() && !it->second->committed) return fail(CKPT_ESTATE, "this iteration's snapshot is still in flight");
    }
    HIP_TRY(c, hipSetDevice(c->device));
    auto sp = std::make_shared<Snap>();
    sp->iter = iter;
    sp->final_path = file_name_for(c->out_dir, iter);
    sp->tmp_path = sp->final_path + ".tmp";
    sp->t_request = t0;
    if (c->plan.n_host) {   // host memory is not ordered with the stream: read it now, the caller may change it after this call
        sp->host_capture.resize(c->plan.host_bytes);
        for (const auto &t : c->plan.tensors)
            if (t.host) memcpy(sp->host_capture.data() + t.capture_off, reinterpret_cast<const void *>(t.dev_addr), t.nbytes);
    }
    {   // a boundary event from the pool made at set-up (it comes back when the snapshot's last copy has landed)
        std::lock_guard<std::mutex> lk(c->mu);
        if (!c->ev_boundary_free.empty()) { sp->ev_boundary = c->ev_boundary_free.back(); c->ev_boundary_free.pop_back(); }
    }
    if (!sp->ev_boundary) HIP_TRY(c, hipEventCreate(&sp->ev_boundary));   // more snapshots in flight than the pool foresaw
    hipError_t e = hipEventRecord(sp->ev_boundary, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        std::lock_guard<std::mutex> lk(c->mu);
        c->ev_boundary_free.push_back(sp->ev_boundary);
        return fail(CKPT_EHIP, std::string("record boundary: ") + hipGetErrorString(e));
    }
    {
        std::lock_guard<std::mutex> lk(c->mu);
        sp->policy = c->cfg.window_policy;
        // records of long-finished snapshots are dropped, lowest iteration first (a long run takes thousands)
        while (c->snaps.size() >= kMaxSnapRecords) {
            auto oldest = c->snaps.begin();
            const Snap &o = *oldest->second;
            if (!o.committed || o.tier2_state == CKPT_TIER2_QUEUED || o.tier2_state == CKPT_TIER2_COPYING || oldest->second == c->last_snap) break;
            c->snaps.erase(oldest);
        }
        c->snaps[iter] = sp;
        c->last_snap = sp;
        c->submit_q.push_back(sp);
        sp->call_ms = ms_between(t0, Clock::now());
    }
    c->cv_submit.notify_one();
    return CKPT_OK;
}

int ckpt_wait_immutable_window_end(ckpt_ctx *c, void *stream, int32_t host_block) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    const auto t_enter = Clock::now();
    std::shared_ptr<Snap> sp;
    {
        std::unique_lock<std::mutex> lk(c->mu);
        sp = c->last_snap;
        if (!sp || sp->window_closed) return CKPT_OK;
        // a device-side wait means something only for events that have been recorded: every copy of the
        // pending snapshot must have been enqueued (policy D2H), or every pack launch (policy PACK)
        const bool pack_only = sp->policy == CKPT_WINDOW_PACK;
        c->cv_state.wait(lk, [&] { return sp->submitted || (pack_only && sp->packs_submitted); });
    }
    HIP_TRY(c, hipSetDevice(c->device));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (sp->policy == CKPT_WINDOW_PACK) {
        hipEvent_t ev = c->ev_packed[sp->plan->n_superchunks - 1];
        HIP_TRY(c, hipStreamWaitEvent(st, ev, 0));
        if (host_block) HIP_TRY(c, hipEventSynchronize(ev));
    } else {
        for (size_t k = 0; k < c->dma.size(); k++) HIP_TRY(c, hipStreamWaitEvent(st, c->ev_job_tail[k], 0));
        if (host_block)
            for (size_t k = 0; k < c->dma.size(); k++) HIP_TRY(c, hipEventSynchronize(c->ev_job_tail[k]));
    }
    std::lock_guard<std::mutex> lk(c->mu);
    sp->window_closed = true;
    sp->window_wait_ms = ms_between(t_enter, Clock::now());
    return CKPT_OK;
}

int ckpt_set_window_policy(ckpt_ctx *c, int32_t policy) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    if (policy != CKPT_WINDOW_D2H && policy != CKPT_WINDOW_PACK) return fail(CKPT_EINVAL, "unknown window_policy");
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->last_snap && !c->last_snap->window_closed) return fail(CKPT_ESTATE, "a snapshot's window is still open");
    if (policy == CKPT_WINDOW_PACK && c->cfg.direct_min_bytes) return fail(CKPT_EINVAL, "direct_min_bytes needs window_policy CKPT_WINDOW_D2H");
    c->cfg.window_policy = policy;
    return CKPT_OK;
}

int ckpt_flush(ckpt_ctx *c, uint64_t iter) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    std::shared_ptr<Snap> failed;
    {
        std::unique_lock<std::mutex> lk(c->mu);
        if (iter == CKPT_ITER_ALL) {
            c->cv_state.wait(lk, [&] {
                for (auto &kv : c->snaps) if (!kv.second->committed) return false;
                return true;
            });
            for (auto &kv : c->snaps) kv.second->window_closed = true;
        } else {
            auto it = c->snaps.find(iter);
            if (it == c->snaps.end()) return fail(CKPT_EINVAL, "no snapshot was requested for this iteration");
            auto sp = it->second;
            c->cv_state.wait(lk, [&] { return sp->committed; });
            sp->window_closed = true;   // its copies are over, so its window is closed too
            failed = sp;
        }
    }
    int r = take_async_error(c);
    if (r) return r;
    // the latch may have been taken by an earlier call; a snapshot that failed still says so when asked about
    if (failed) {
        std::lock_guard<std::mutex> lk(c->mu);
        if (failed->failed) return fail(failed->fail_code, failed->fail_msg);
    }
    return CKPT_OK;
}

int ckpt_get_layout(ckpt_ctx *c, ckpt_layout *out) {
    if (!c || !out) return fail(CKPT_EINVAL, "null argument");
    if (!c->registered) return fail(CKPT_ESTATE, "no tensors registered");
    fill_layout(c->plan, out);
    if (c->have_rplan) {
        out->n_derived_tensors = c->rplan.n_derived;
        out->derived_bytes = c->rplan.derived_bytes;
        out->reduced_header_bytes = c->rplan.header_bytes;
        out->reduced_data_bytes = c->rplan.data_bytes;
    }
    return CKPT_OK;
}

int ckpt_declare_derived(ckpt_ctx *c, const uint32_t *derived, const uint32_t *source, size_t n_pairs) {
    if (!c || (n_pairs && (!derived || !source))) return fail(CKPT_EINVAL, "null argument");
    if (c->registered) return fail(CKPT_ESTATE, "derived tensors must be declared before ckpt_register_tensors");
    c->pairs.derived.assign(derived, derived + n_pairs);
    c->pairs.source.assign(source, source + n_pairs);
    return CKPT_OK;
}

int ckpt_get_init_probe(ckpt_ctx *c, double *d2h_gbps) {
    if (!c || !d2h_gbps) return fail(CKPT_EINVAL, "null argument");
    *d2h_gbps = c->init_d2h_gbps;
    return CKPT_OK;
}

int ckpt_get_stats(ckpt_ctx *c, uint64_t iter, ckpt_stats *o) {
    if (!c || !o) return fail(CKPT_EINVAL, "null argument");
    std::lock_guard<std::mutex> lk(c->mu);
    auto it = c->snaps.find(iter);
    if (it == c->snaps.end()) return fail(CKPT_EINVAL, "no snapshot was requested for this iteration");
    const Snap &s = *it->second;
    memset(o, 0, sizeof *o);
    o->iter = s.iter;
    const Plan &sp = s.plan ? *s.plan : c->plan;
    o->payload_bytes = sp.payload_bytes - sp.derived_bytes;   // what this snapshot stores
    o->data_bytes = sp.data_bytes;
    o->file_bytes = sp.file_bytes();
    o->format_version = s.plan ? int32_t(s.plan->version) : 0;
    o->verify_ms = s.verify_ms;
    o->host_window_wait_ms = s.window_wait_ms;
    o->init_d2h_gbps = c->init_d2h_gbps;
    o->d2h_done = s.d2h_done;
    o->committed = s.committed;
    o->pack_launches = int32_t(sp.n_superchunks);
    o->tier2_state = s.tier2_state;
    o->host_tier2_ms = s.tier2_ms;
    o->pack_ms_sum = s.pack_ms_sum;
    o->request_to_d2h_end_ms = s.req_to_d2h_end_ms;
    o->d2h_span_ms = s.d2h_span_ms;
    o->request_to_pack_end_ms = s.req_to_pack_end_ms;
    o->host_submit_ms = s.submitted ? ms_between(s.t_request, s.t_submitted) : -1;
    o->host_request_to_commit_ms = s.committed ? ms_between(s.t_request, s.t_committed) : -1;
    o->host_backpressure_ms = s.submitted ? s.backpressure_ms : -1;
    o->host_snapshot_call_ms = s.call_ms;
    o->host_io_wait_ms_sum = s.io_wait_us.load() / 1000.0;
    o->host_io_copy_ms_sum = s.io_copy_us.load() / 1000.0;
    o->host_flush_span_ms = (s.committed && s.have_first_chunk) ? ms_between(s.t_first_chunk, s.t_committed) : -1;
    return CKPT_OK;
}

int ckpt_file_name(ckpt_ctx *c, uint64_t iter, char *buf, size_t cap) {
    if (!c || !buf) return fail(CKPT_EINVAL, "null argument");
    std::string n = file_name_for(c->out_dir, iter);
    if (cap < n.size() + 1) return fail(CKPT_EINVAL, "buffer too small");
    memcpy(buf, n.c_str(), n.size() + 1);
    return CKPT_OK;
}

int ckpt_destroy(ckpt_ctx *c) {
    if (!c) return CKPT_OK;
    int rc = CKPT_OK;
    if (c->submit_thread.joinable()) {
        {   // drain
            std::unique_lock<std::mutex> lk(c->mu);
            c->cv_state.wait(lk, [&] {
                for (auto &kv : c->snaps) if (!kv.second->committed) return false;
                return true;
            });
            c->stopping = true;
            for (size_t i = 0; i < c->io_threads.size(); i++) c->io_q.push_back(IoJob{});
        }
        c->cv_submit.notify_all();
        c->cv_io.notify_all();
        c->submit_thread.join();
        for (auto &t : c->io_threads) t.join();
        if (c->tier2_thread.joinable()) {   // the second tier finishes what it has been offered
            {
                std::unique_lock<std::mutex> lk(c->mu);
                c->cv_state.wait(lk, [&] { return !c->tier2_waiting && !c->tier2_active; });
                c->tier2_stop = true;
            }
            c->cv_tier2.notify_all();
            c->tier2_thread.join();
            if (c->tier2_unlinker.joinable()) c->tier2_unlinker.join();
        }
        rc = take_async_error(c);
        if (rc == CKPT_OK && c->tier2_code) { rc = c->tier2_code; g_last_error = c->tier2_err; }
    }
    (void)hipSetDevice(c->device);
    if (c->pack_stream) (void)hipStreamSynchronize(c->pack_stream);
    for (auto s : c->dma) (void)hipStreamSynchronize(s);
    for (auto &kv : c->snaps) if (kv.second->ev_boundary) (void)hipEventDestroy(kv.second->ev_boundary);
    for (auto ev : c->ev_boundary_free) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_slot) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_pack_start) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_packed) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_pack_end) (void)hipEventDestroy(ev);
    for (auto &v : c->ev_stage_done) for (auto ev : v) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_job_tail) (void)hipEventDestroy(ev);
    if (c->ev_first_copy) (void)hipEventDestroy(c->ev_first_copy);
    if (c->ev_user) (void)hipEventDestroy(c->ev_user);
    if (c->pack_stream) (void)hipStreamDestroy(c->pack_stream);
    for (auto s : c->dma) (void)hipStreamDestroy(s);
    if (c->staging) (void)hipFree(c->staging);
    if (c->dev_tiles) (void)hipFree(c->dev_tiles);
    if (c->dev_rtiles) (void)hipFree(c->dev_rtiles);
    if (c->dev_pairs) (void)hipFree(c->dev_pairs);
    if (c->dev_flag) (void)hipFree(c->dev_flag);
    if (c->host_flag) (void)hipHostFree(c->host_flag);
    if (c->ev_verify_start) (void)hipEventDestroy(c->ev_verify_start);
    if (c->ev_verify_done) (void)hipEventDestroy(c->ev_verify_done);
    if (c->ev_derived) (void)hipEventDestroy(c->ev_derived);
    if (c->ring) (void)hipHostFree(c->ring);
    for (auto &sp : c->spares) { sp.close_all(); unlink(sp.path.c_str()); }
    for (auto &kv : c->kept) kv.second.close_all();
    free(c->hdr_buf);
    delete c;
    return rc;
}

}  // extern "C"
