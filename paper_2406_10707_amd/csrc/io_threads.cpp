// The I/O threads: wait for a chunk's copy event, write the ring slot to the file, free the slot;
// the thread that writes a snapshot's last chunk commits the file and applies retention. On restore
// the same threads read file chunks into ring slots.
#include "engine_internal.hpp"

using namespace dsllm;

static void finish_d2h_stats(ckpt_ctx *c, Snap *s) {
    // called by the I/O thread that owns the snapshot's last chunk, after all tail events completed
    double pack_sum = 0, req_d2h = 0, span = 0, req_pack = 0;
    float ms = 0;
    const uint64_t n_sc = s->plan->n_superchunks;
    for (uint64_t i = 0; i < n_sc; i++)
        if (hipEventElapsedTime(&ms, c->ev_pack_start[i], c->ev_pack_end[i]) == hipSuccess) pack_sum += ms;
    for (size_t k = 0; k < c->dma.size(); k++) {
        if (hipEventElapsedTime(&ms, s->ev_boundary, c->ev_job_tail[k]) == hipSuccess && ms > req_d2h) req_d2h = ms;
        if (hipEventElapsedTime(&ms, c->ev_first_copy, c->ev_job_tail[k]) == hipSuccess && ms > span) span = ms;
    }
    if (hipEventElapsedTime(&ms, s->ev_boundary, c->ev_packed[n_sc - 1]) == hipSuccess) req_pack = ms;
    std::lock_guard<std::mutex> lk(c->mu);
    c->ev_boundary_free.push_back(s->ev_boundary);   // back to the pool
    s->ev_boundary = nullptr;
    s->pack_ms_sum = pack_sum;
    s->req_to_d2h_end_ms = req_d2h;
    s->d2h_span_ms = span;
    s->req_to_pack_end_ms = req_pack;
    s->d2h_done = true;
    c->cv_state.notify_all();
}

// O_DIRECT cannot take its data from the pinned ring (the kernel refuses device-mapped pages as a
// direct-I/O source or target: EFAULT), so direct I/O goes through a small aligned bounce buffer
// owned by the I/O thread.
constexpr uint64_t kBounceBytes = 4ull << 20;

static bool direct_write(int fd, uint8_t *bounce, const uint8_t *src, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        uint64_t m = n < kBounceBytes ? n : kBounceBytes;
        memcpy(bounce, src, m);
        if (!pwrite_all(fd, bounce, m, off, err)) return false;
        src += m; off += m; n -= m;
    }
    return true;
}

static bool direct_read(int fd, uint8_t *bounce, uint8_t *dst, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        uint64_t m = n < kBounceBytes ? n : kBounceBytes;
        if (!pread_all(fd, bounce, m, off, err)) return false;
        memcpy(dst, bounce, m);
        dst += m; off += m; n -= m;
    }
    return true;
}

// Turns the committed file of `iter` into a spare whose pages a later snapshot overwrites. c->mu held.
void dsllm::retire_locked(ckpt_ctx *c, uint64_t iter) {
    auto it = c->kept.find(iter);
    if (it == c->kept.end()) return;
    FileSlot sp = it->second;
    c->kept.erase(it);
    std::string spare = c->out_dir + "/.spare_" + std::to_string(getpid()) + "_" + std::to_string(c->spare_seq++) + ".dsl";
    if (rename(sp.path.c_str(), spare.c_str()) == 0) { sp.path = spare; c->spares.push_back(sp); }
    else sp.close_all();   // somebody removed or replaced the file: drop it
}

void dsllm::io_thread_main(ckpt_ctx *c) {
    (void)hipSetDevice(c->device);
    uint8_t *bounce = nullptr;
    if (c->cfg.o_direct && posix_memalign(reinterpret_cast<void **>(&bounce), 4096, kBounceBytes) != 0) bounce = nullptr;
    struct BounceFree { uint8_t *&p; ~BounceFree() { free(p); } } bounce_free{bounce};
    for (;;) {
        IoJob job;
        {
            std::unique_lock<std::mutex> lk(c->mu);
            c->cv_io.wait(lk, [&] { return !c->io_q.empty(); });
            job = c->io_q.front();
            c->io_q.pop_front();
        }
        if (job.kind == IoJob::STOP) return;
        uint8_t *slot_ptr = c->ring + job.slot * c->cfg.dma_chunk_bytes;
        std::string err;
        if (job.kind == IoJob::READ) {
            uint8_t *piece = slot_ptr + job.slot_off;
            bool ok = c->cfg.o_direct ? (bounce ? direct_read(job.fd, bounce, piece, job.nbytes, job.file_off, &err) : (err = "no bounce buffer", false))
                                      : pread_all(job.fd, piece, job.nbytes, job.file_off, &err);
            if (!ok) c->latch(CKPT_EIO, err);
            std::lock_guard<std::mutex> lk(c->mu);
            if (--c->slot_reads_left[job.slot] == 0) {   // the chunk's last piece
                c->slot_state[job.slot] = SLOT_READ_DONE;
                c->cv_state.notify_all();
            }
            continue;
        }
        // WRITE: the chunk's copy must have landed in the slot first
        Snap *s = job.snap.get();
        auto tw0 = Clock::now();
        hipError_t he = hipEventSynchronize(c->ev_slot[job.slot]);
        auto tw1 = Clock::now();
        s->io_wait_us += uint64_t(ms_between(tw0, tw1) * 1000.0);
        if (he != hipSuccess) c->fail_snapshot(s, CKPT_EHIP, std::string("copy event: ") + hipGetErrorString(he));
        if (job.file_off == s->plan->header_bytes) {
            std::lock_guard<std::mutex> lk(c->mu);
            s->t_first_chunk = Clock::now();
            s->have_first_chunk = true;
        }
        if (job.last) {
            for (size_t k = 0; k < c->dma.size(); k++) {
                he = hipEventSynchronize(c->ev_job_tail[k]);
                if (he != hipSuccess) c->fail_snapshot(s, CKPT_EHIP, std::string("tail event: ") + hipGetErrorString(he));
            }
            finish_d2h_stats(c, s);
        }
        if (s->map) memcpy(s->map + job.file_off, slot_ptr, job.nbytes);   // page-cache/tmpfs sink: parallel across threads
        else if (s->fd >= 0) {
            bool ok = c->cfg.o_direct ? (bounce ? direct_write(s->fd, bounce, slot_ptr, job.nbytes, job.file_off, &err) : (err = "no bounce buffer", false))
                                      : pwrite_all(s->fd, slot_ptr, job.nbytes, job.file_off, &err);
            if (!ok) c->fail_snapshot(s, CKPT_EIO, s->tmp_path + ": " + err);
        }
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->slot_state[job.slot] = SLOT_FREE;
            c->cv_state.notify_all();
        }
        s->io_copy_us += uint64_t(ms_between(tw1, Clock::now()) * 1000.0);
        if (s->chunks_left.fetch_sub(1) == 1) {
            // last chunk written: commit. Whether the file gets its final name depends on this snapshot's own
            // record of failures, not on the context-wide latch (a call in between may have taken and cleared that).
            if (s->fd >= 0) {
                const bool retain = c->cfg.keep_last > 0;
                const bool sync = c->cfg.fsync_on_commit != 0;
                if (s->map && sync && msync(s->map, s->plan->file_bytes(), MS_SYNC) != 0)
                    c->fail_snapshot(s, CKPT_EIO, s->tmp_path + ": msync: " + strerror(errno));
                if (sync && fsync(s->fd) != 0) c->fail_snapshot(s, CKPT_EIO, s->tmp_path + ": fsync: " + strerror(errno));
                FileSlot fs;
                fs.path = s->final_path; fs.fd = s->fd; fs.map = s->map; fs.map_bytes = s->plan->file_bytes(); fs.bytes = s->plan->file_bytes();
                s->fd = -1; s->map = nullptr;
                bool had_error;
                { std::lock_guard<std::mutex> lk(c->mu); had_error = s->failed; }
                // a file gets its final name only when whole
                if (!had_error && rename(s->tmp_path.c_str(), s->final_path.c_str()) != 0) {
                    c->fail_snapshot(s, CKPT_EIO, s->final_path + ": rename: " + strerror(errno));
                    had_error = true;
                }
                std::string derr;
                if (!had_error && sync && !fsync_dir(c->out_dir, &derr)) c->fail_snapshot(s, CKPT_EIO, derr);   // the name is there, its durability is not
                if (retain && !had_error) {
                    // files older than the newest keep_last become spares, overwritten in place later
                    std::lock_guard<std::mutex> lk(c->mu);
                    auto dup = c->kept.find(s->iter);
                    if (dup != c->kept.end()) { dup->second.close_all(); c->kept.erase(dup); }
                    c->kept[s->iter] = fs;
                    c->committed_iters.push_back(s->iter);
                    while (c->committed_iters.size() > size_t(c->cfg.keep_last)) {
                        const uint64_t old = c->committed_iters.front();
                        c->committed_iters.pop_front();
                        if (old == s->iter) continue;
                        if (c->tier2_active && c->tier2_active->iter == old) { c->tier2_retire_after = true; continue; }   // still being read
                        retire_locked(c, old);
                    }
                } else {
                    fs.close_all();
                    if (had_error) unlink(s->tmp_path.c_str());   // a torn file, under its temporary (or spare) name: gone
                }
            }
            std::lock_guard<std::mutex> lk(c->mu);
            s->t_committed = Clock::now();
            s->committed = true;
            if (!s->failed) tier2_offer_locked(c, job.snap);
            c->cv_state.notify_all();
        }
    }
}

