// The snapshot engine behind the C ABI of include/ckpt.h.
//
// Threads: the caller (records the boundary event, never waits for copies), one submit thread
// (enqueues pack kernels and device-to-host copies, blocks on ring back-pressure so the caller does
// not), and n I/O threads (wait for a chunk's copy event, write the ring slot to the file, free the
// slot; on restore they read file chunks into ring slots). This is the producer/consumer circular
// host cache of the paper's design, with the device-to-host copies gated by HIP events.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include <errno.h>
#include <fcntl.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <sys/statvfs.h>
#include <unistd.h>

#include "plan.hpp"

namespace dsllm {
hipError_t launch_pack(const ckpt_tile *dev_tiles, uint64_t n_tiles, void *slot_base, uint64_t slot_data_off, hipStream_t stream);
hipError_t launch_scatter(const ckpt_tile *dev_tiles, uint64_t n_tiles, const void *slot_base, uint64_t slot_data_off, hipStream_t stream);
}  // namespace dsllm

using namespace dsllm;
using Clock = std::chrono::steady_clock;

static thread_local std::string g_last_error;
static int fail(int code, const std::string &msg) { g_last_error = msg; return code; }
static double ms_between(Clock::time_point a, Clock::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); }

// Progress lines on stderr when DSLLM_CKPT_TRACE is set in the environment (set-up stages only).
static void trace(const char *what) {
    static const bool on = getenv("DSLLM_CKPT_TRACE") != nullptr;
    if (on) { fprintf(stderr, "[dsllm_ckpt] %s\n", what); fflush(stderr); }
}

struct ckpt_plan { Plan plan; };

namespace {

// An open checkpoint file. With retention (keep_last > 0) files, descriptors and mappings live on
// after the commit: a retired file is renamed to a hidden spare name and a later snapshot writes
// into the same pages through the same mapping, so the steady-state flush is plain memcpy.
struct FileSlot {
    std::string path;
    int fd = -1;
    uint8_t *map = nullptr;           // whole-file shared mapping when the sink is written through mmap
    uint64_t map_bytes = 0;
    void close_all() {
        if (map) munmap(map, map_bytes);
        if (fd >= 0) ::close(fd);
        map = nullptr; fd = -1;
    }
};

struct Snap {
    uint64_t iter = 0;
    int fd = -1;
    uint8_t *map = nullptr;
    std::string tmp_path, final_path;
    std::atomic<uint64_t> chunks_left{0};
    hipEvent_t ev_boundary = nullptr;
    bool submitted = false, packs_submitted = false, d2h_done = false, committed = false, window_closed = false;
    Clock::time_point t_request, t_submitted, t_committed, t_first_chunk;
    bool have_first_chunk = false;
    double call_ms = 0, backpressure_ms = 0;
    std::atomic<uint64_t> io_wait_us{0}, io_copy_us{0};   // summed over the I/O threads
    double pack_ms_sum = -1, req_to_d2h_end_ms = -1, d2h_span_ms = -1, req_to_pack_end_ms = -1;
    std::vector<uint8_t> host_capture;      // the host-resident objects as they were when the snapshot was requested
    int tier2_state = CKPT_TIER2_NONE;      // ckpt_tier2_state
    double tier2_ms = -1;                   // host: copy to the second tier, open to rename
};

struct IoJob {
    enum Kind { WRITE, READ, STOP } kind = STOP;
    std::shared_ptr<Snap> snap;   // WRITE
    int fd = -1;                  // READ
    uint64_t slot = 0, file_off = 0, nbytes = 0;
    bool last = false;
    uint64_t seq = 0;             // READ: chunk sequence number
};

enum SlotState : int { SLOT_FREE = 0, SLOT_BUSY = 1, SLOT_READ_DONE = 2 };

}  // namespace

struct ckpt_ctx {
    ResolvedConfig cfg;
    int device = 0;
    std::string out_dir;
    bool registered = false;
    Plan plan;

    // device resources
    uint8_t *ring = nullptr;          // pinned host
    uint64_t n_slots = 0;
    uint8_t *staging = nullptr;       // device
    uint64_t n_stage = 0;
    ckpt_tile *dev_tiles = nullptr;
    hipStream_t pack_stream = nullptr;
    std::vector<hipStream_t> dma;
    std::vector<hipEvent_t> ev_slot;                      // per ring slot: copy into/out of the slot done
    std::vector<hipEvent_t> ev_pack_start, ev_packed;     // per super-chunk
    std::vector<std::vector<hipEvent_t>> ev_stage_done;   // [stage slot][dma stream]
    std::vector<hipEvent_t> ev_job_tail;                  // per dma stream
    hipEvent_t ev_first_copy = nullptr, ev_user = nullptr;
    uint8_t *hdr_buf = nullptr;                           // 4 KiB-aligned scratch for header writes
    uint64_t ring_next = 0;                               // global chunk counter -> ring slot

    // threads and queues
    std::mutex mu;
    std::condition_variable cv_submit, cv_io, cv_state;   // submit queue / io queue / any state change
    std::deque<std::shared_ptr<Snap>> submit_q;
    std::deque<IoJob> io_q;
    std::vector<int> slot_state;
    bool stopping = false;
    std::thread submit_thread;
    std::vector<std::thread> io_threads;
    std::map<uint64_t, std::shared_ptr<Snap>> snaps;
    std::shared_ptr<Snap> last_snap;       // most recent request
    std::shared_ptr<Snap> prev_job;        // submit thread: job before the current one
    int async_code = 0;
    std::string async_err;
    bool restoring = false;
    // retention: committed iterations in commit order, and retired files whose pages are reused
    std::deque<uint64_t> committed_iters;
    std::vector<FileSlot> spares;
    std::map<uint64_t, FileSlot> kept;     // committed files that still carry their names
    uint64_t spare_seq = 0;
    // second tier: committed files are copied on to a slower, durable directory by a thread of their own
    bool tier2_on = false, tier2_direct = false, tier2_stop = false;
    std::string tier2_dir;
    int tier2_threads = 2, tier2_keep = 1;
    std::thread tier2_thread;
    std::condition_variable cv_tier2;
    std::shared_ptr<Snap> tier2_waiting;   // newest committed snapshot not yet picked up (latest wins)
    std::shared_ptr<Snap> tier2_active;    // being copied: its first-tier file must not be recycled
    bool tier2_retire_after = false;       // the active file fell out of the newest keep_last meanwhile
    std::deque<uint64_t> tier2_files;      // iterations present in the second tier, oldest first
    int tier2_code = 0;                    // first failure of a second-tier copy, reported by ckpt_wait_second_tier
    std::string tier2_err;

    void latch(int code, const std::string &msg) {
        std::lock_guard<std::mutex> lk(mu);
        if (async_code == 0) { async_code = code; async_err = msg; }
        cv_state.notify_all();
    }
};

#define HIP_TRY(ctx, expr)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(CKPT_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

static std::string file_name_for(const std::string &dir, uint64_t iter) {
    char buf[64];
    snprintf(buf, sizeof buf, "/ckpt_iter%020llu.dsl", (unsigned long long)iter);
    return dir + buf;
}

static bool pwrite_all(int fd, const uint8_t *p, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        size_t want = n > (1ull << 30) ? size_t(1ull << 30) : size_t(n);
        ssize_t w = pwrite(fd, p, want, off_t(off));
        if (w < 0) { if (errno == EINTR) continue; *err = std::string("pwrite: ") + strerror(errno); return false; }
        p += w; off += uint64_t(w); n -= uint64_t(w);
    }
    return true;
}

static bool pread_all(int fd, uint8_t *p, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        size_t want = n > (1ull << 30) ? size_t(1ull << 30) : size_t(n);
        ssize_t r = pread(fd, p, want, off_t(off));
        if (r < 0) { if (errno == EINTR) continue; *err = std::string("pread: ") + strerror(errno); return false; }
        if (r == 0) { *err = "pread: unexpected end of file"; return false; }
        p += r; off += uint64_t(r); n -= uint64_t(r);
    }
    return true;
}

// ------------------------------------------------------------------ I/O threads

static void finish_d2h_stats(ckpt_ctx *c, Snap *s) {
    // called by the I/O thread that owns the snapshot's last chunk, after all tail events completed
    double pack_sum = 0, req_d2h = 0, span = 0, req_pack = 0;
    float ms = 0;
    for (uint64_t i = 0; i < c->plan.n_superchunks; i++)
        if (hipEventElapsedTime(&ms, c->ev_pack_start[i], c->ev_packed[i]) == hipSuccess) pack_sum += ms;
    for (size_t k = 0; k < c->dma.size(); k++) {
        if (hipEventElapsedTime(&ms, s->ev_boundary, c->ev_job_tail[k]) == hipSuccess && ms > req_d2h) req_d2h = ms;
        if (hipEventElapsedTime(&ms, c->ev_first_copy, c->ev_job_tail[k]) == hipSuccess && ms > span) span = ms;
    }
    if (hipEventElapsedTime(&ms, s->ev_boundary, c->ev_packed[c->plan.n_superchunks - 1]) == hipSuccess) req_pack = ms;
    (void)hipEventDestroy(s->ev_boundary);
    std::lock_guard<std::mutex> lk(c->mu);
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
static void retire_locked(ckpt_ctx *c, uint64_t iter) {
    auto it = c->kept.find(iter);
    if (it == c->kept.end()) return;
    FileSlot sp = it->second;
    c->kept.erase(it);
    std::string spare = c->out_dir + "/.spare_" + std::to_string(getpid()) + "_" + std::to_string(c->spare_seq++) + ".dsl";
    if (rename(sp.path.c_str(), spare.c_str()) == 0) { sp.path = spare; c->spares.push_back(sp); }
    else sp.close_all();   // somebody removed or replaced the file: drop it
}

// Hands a freshly committed snapshot to the second tier. A snapshot still waiting there is
// superseded: the slower tier always takes the newest state it can get. c->mu held.
static void tier2_offer_locked(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    if (!c->tier2_on) return;
    if (c->tier2_waiting) c->tier2_waiting->tier2_state = CKPT_TIER2_SKIPPED;
    sp->tier2_state = CKPT_TIER2_QUEUED;
    c->tier2_waiting = sp;
    c->cv_tier2.notify_all();
}

static void io_thread_main(ckpt_ctx *c) {
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
            bool ok = c->cfg.o_direct ? (bounce ? direct_read(job.fd, bounce, slot_ptr, job.nbytes, job.file_off, &err) : (err = "no bounce buffer", false))
                                      : pread_all(job.fd, slot_ptr, job.nbytes, job.file_off, &err);
            if (!ok) c->latch(CKPT_EIO, err);
            std::lock_guard<std::mutex> lk(c->mu);
            c->slot_state[job.slot] = SLOT_READ_DONE;
            c->cv_state.notify_all();
            continue;
        }
        // WRITE: the chunk's copy must have landed in the slot first
        Snap *s = job.snap.get();
        auto tw0 = Clock::now();
        hipError_t he = hipEventSynchronize(c->ev_slot[job.slot]);
        auto tw1 = Clock::now();
        s->io_wait_us += uint64_t(ms_between(tw0, tw1) * 1000.0);
        if (he != hipSuccess) c->latch(CKPT_EHIP, std::string("copy event: ") + hipGetErrorString(he));
        if (job.file_off == c->plan.header_bytes) {
            std::lock_guard<std::mutex> lk(c->mu);
            s->t_first_chunk = Clock::now();
            s->have_first_chunk = true;
        }
        if (job.last) {
            for (size_t k = 0; k < c->dma.size(); k++) {
                he = hipEventSynchronize(c->ev_job_tail[k]);
                if (he != hipSuccess) c->latch(CKPT_EHIP, std::string("tail event: ") + hipGetErrorString(he));
            }
            finish_d2h_stats(c, s);
        }
        if (s->map) memcpy(s->map + job.file_off, slot_ptr, job.nbytes);   // page-cache/tmpfs sink: parallel across threads
        else if (s->fd >= 0) {
            bool ok = c->cfg.o_direct ? (bounce ? direct_write(s->fd, bounce, slot_ptr, job.nbytes, job.file_off, &err) : (err = "no bounce buffer", false))
                                      : pwrite_all(s->fd, slot_ptr, job.nbytes, job.file_off, &err);
            if (!ok) c->latch(CKPT_EIO, s->tmp_path + ": " + err);
        }
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->slot_state[job.slot] = SLOT_FREE;
            c->cv_state.notify_all();
        }
        s->io_copy_us += uint64_t(ms_between(tw1, Clock::now()) * 1000.0);
        if (s->chunks_left.fetch_sub(1) == 1) {
            // last chunk written: commit
            if (s->fd >= 0) {
                const bool retain = c->cfg.keep_last > 0;
                if (s->map && c->cfg.fsync_on_commit && msync(s->map, c->plan.file_bytes(), MS_SYNC) != 0)
                    c->latch(CKPT_EIO, s->tmp_path + ": msync: " + strerror(errno));
                if (c->cfg.fsync_on_commit && fsync(s->fd) != 0) c->latch(CKPT_EIO, s->tmp_path + ": fsync: " + strerror(errno));
                FileSlot fs;
                fs.path = s->final_path; fs.fd = s->fd; fs.map = s->map; fs.map_bytes = c->plan.file_bytes();
                s->fd = -1; s->map = nullptr;
                bool had_error;
                { std::lock_guard<std::mutex> lk(c->mu); had_error = c->async_code != 0; }
                // a file gets its final name only when whole
                if (!had_error && rename(s->tmp_path.c_str(), s->final_path.c_str()) != 0) {
                    c->latch(CKPT_EIO, s->final_path + ": rename: " + strerror(errno));
                    had_error = true;
                }
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
                    if (had_error) unlink(s->tmp_path.c_str());
                }
            }
            std::lock_guard<std::mutex> lk(c->mu);
            s->t_committed = Clock::now();
            s->committed = true;
            if (c->async_code == 0) tier2_offer_locked(c, job.snap);
            c->cv_state.notify_all();
        }
    }
}

// ------------------------------------------------------------------ second tier

// Copies one committed first-tier file to the second-tier directory: n threads take 8 MiB blocks in
// turn, from the kept mapping when there is one (tmpfs pages: a memory read), else with pread;
// fsync, rename, then older second-tier files beyond tier2_keep are removed.
static void tier2_copy(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    const uint64_t total = c->plan.file_bytes(), blk = 8ull << 20;
    const uint64_t n_blk = (total + blk - 1) / blk;
    auto t0 = Clock::now();
    const uint8_t *src_map = nullptr;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        auto it = c->kept.find(sp->iter);
        if (it != c->kept.end() && it->second.map) src_map = it->second.map;
    }
    std::string err;
    int src_fd = -1;
    if (!src_map) {
        src_fd = open(sp->final_path.c_str(), O_RDONLY);
        if (src_fd < 0) err = sp->final_path + ": open: " + strerror(errno);
    }
    const std::string dst_final = file_name_for(c->tier2_dir, sp->iter), dst_tmp = dst_final + ".tmp";
    int dst_fd = -1;
    if (err.empty()) {
        dst_fd = open(dst_tmp.c_str(), O_WRONLY | O_CREAT | O_TRUNC | (c->tier2_direct ? O_DIRECT : 0), 0644);
        if (dst_fd < 0) err = dst_tmp + ": open: " + strerror(errno);
    }
    if (err.empty()) {
        std::atomic<uint64_t> next{0};
        std::mutex emu;
        auto worker = [&] {
            uint8_t *buf = nullptr;
            const bool need_buf = c->tier2_direct || !src_map;
            if (need_buf && posix_memalign(reinterpret_cast<void **>(&buf), 4096, blk) != 0) {
                std::lock_guard<std::mutex> lk(emu);
                if (err.empty()) err = "no memory for a copy buffer";
                return;
            }
            for (;;) {
                const uint64_t b = next.fetch_add(1);
                if (b >= n_blk) break;
                { std::lock_guard<std::mutex> lk(emu); if (!err.empty()) break; }
                const uint64_t off = b * blk, n = std::min(blk, total - off);   // file sizes are 4 KiB multiples
                std::string e;
                const uint8_t *from;
                if (src_map) {
                    if (buf) { memcpy(buf, src_map + off, n); from = buf; } else from = src_map + off;
                } else {
                    if (!pread_all(src_fd, buf, n, off, &e)) { std::lock_guard<std::mutex> lk(emu); if (err.empty()) err = sp->final_path + ": " + e; break; }
                    from = buf;
                }
                if (!pwrite_all(dst_fd, from, n, off, &e)) { std::lock_guard<std::mutex> lk(emu); if (err.empty()) err = dst_tmp + ": " + e; break; }
            }
            free(buf);
        };
        std::vector<std::thread> th;
        for (int i = 1; i < c->tier2_threads; i++) th.emplace_back(worker);
        worker();
        for (auto &t : th) t.join();
        if (err.empty() && fsync(dst_fd) != 0) err = dst_tmp + ": fsync: " + strerror(errno);
    }
    if (dst_fd >= 0) close(dst_fd);
    if (src_fd >= 0) close(src_fd);
    if (err.empty() && rename(dst_tmp.c_str(), dst_final.c_str()) != 0) err = dst_final + ": rename: " + strerror(errno);
    if (!err.empty()) unlink(dst_tmp.c_str());
    std::vector<uint64_t> drop;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (!err.empty() && c->tier2_code == 0) { c->tier2_code = CKPT_EIO; c->tier2_err = "second tier: " + err; }
        sp->tier2_ms = ms_between(t0, Clock::now());
        sp->tier2_state = err.empty() ? CKPT_TIER2_DONE : CKPT_TIER2_FAILED;
        if (err.empty()) {
            c->tier2_files.push_back(sp->iter);
            while (c->tier2_keep > 0 && c->tier2_files.size() > size_t(c->tier2_keep)) {
                if (c->tier2_files.front() != sp->iter) drop.push_back(c->tier2_files.front());
                c->tier2_files.pop_front();
            }
        }
    }
    for (uint64_t it : drop) unlink(file_name_for(c->tier2_dir, it).c_str());
}

static void tier2_thread_main(ckpt_ctx *c) {
    for (;;) {
        std::shared_ptr<Snap> sp;
        {
            std::unique_lock<std::mutex> lk(c->mu);
            c->cv_tier2.wait(lk, [&] { return c->tier2_stop || c->tier2_waiting; });
            if (!c->tier2_waiting) return;
            sp = c->tier2_waiting;
            c->tier2_waiting.reset();
            // with retention the first-tier file may have been recycled already (it was committed, then two
            // newer snapshots followed before this thread came round): then there is nothing left to copy
            if (c->cfg.keep_last > 0 && c->kept.find(sp->iter) == c->kept.end()) {
                sp->tier2_state = CKPT_TIER2_SKIPPED;
                c->cv_state.notify_all();
                continue;
            }
            sp->tier2_state = CKPT_TIER2_COPYING;
            c->tier2_active = sp;
            c->tier2_retire_after = false;
        }
        tier2_copy(c, sp);
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->tier2_active.reset();
            if (c->tier2_retire_after) retire_locked(c, sp->iter);
            c->tier2_retire_after = false;
            c->cv_state.notify_all();
        }
    }
}

// ------------------------------------------------------------------ submit thread

static void submit_one(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    Snap *s = sp.get();
    const Plan &p = c->plan;
    const uint64_t CH = c->cfg.dma_chunk_bytes, SC = c->cfg.pack_superchunk_bytes;
    const size_t nk = c->dma.size();
    auto hip_fail = [&](const char *what, hipError_t e) { c->latch(CKPT_EHIP, std::string(what) + ": " + hipGetErrorString(e)); };
    hipError_t e;

    // one snapshot's copies at a time: the previous one's last copy is over before this one's
    // boundary on the device timeline anyway (the caller closed its window), so this costs nothing there
    if (c->prev_job) {
        for (size_t k = 0; k < nk; k++) if ((e = hipEventSynchronize(c->ev_job_tail[k])) != hipSuccess) hip_fail("tail sync", e);
        std::unique_lock<std::mutex> lk(c->mu);
        // with retention the previous commit is also what retires an older file into the spare pool this
        // snapshot is about to draw from: wait for it (it follows the last copy by one chunk write)
        c->cv_state.wait(lk, [&] { return c->prev_job->d2h_done && (c->cfg.keep_last == 0 || c->prev_job->committed); });
    }

    // file and header
    const bool use_mmap = c->cfg.io_mode == CKPT_IO_MMAP;
    memcpy(c->hdr_buf, p.header.data(), p.header_bytes);
    for (int i = 0; i < 8; i++) c->hdr_buf[16 + i] = uint8_t(s->iter >> (8 * i));
    FileSlot reuse;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (!c->spares.empty()) { reuse = c->spares.back(); c->spares.pop_back(); }
    }
    std::string ferr;
    if (reuse.fd >= 0) {
        // a retired file of this registration: same size, pages allocated, still open (and mapped);
        // every byte of it is rewritten (header, data and padding), so nothing is truncated
        s->tmp_path = reuse.path;
        s->fd = reuse.fd;
        s->map = reuse.map;
    } else {
        int flags = (use_mmap ? O_RDWR : O_WRONLY) | O_CREAT | O_TRUNC | (c->cfg.o_direct ? O_DIRECT : 0);
        s->fd = open(s->tmp_path.c_str(), flags, 0644);
        if (s->fd < 0) ferr = std::string("open: ") + strerror(errno);
        else if (use_mmap) {
            // stores into a mapping cannot report "no space left" as an error code: check the room first
            struct statvfs vfs;
            if (fstatvfs(s->fd, &vfs) == 0 && uint64_t(vfs.f_bavail) * vfs.f_frsize < p.file_bytes()) ferr = "not enough free space for the checkpoint file";
            else if (ftruncate(s->fd, off_t(p.file_bytes())) != 0) ferr = std::string("ftruncate: ") + strerror(errno);
            else {
                void *m = mmap(nullptr, p.file_bytes(), PROT_READ | PROT_WRITE, MAP_SHARED, s->fd, 0);
                if (m == MAP_FAILED) ferr = std::string("mmap: ") + strerror(errno);
                else s->map = static_cast<uint8_t *>(m);
            }
        }
    }
    if (ferr.empty() && s->fd >= 0) {
        if (s->map) memcpy(s->map, c->hdr_buf, p.header_bytes);
        else if (!pwrite_all(s->fd, c->hdr_buf, p.header_bytes, 0, &ferr)) {}
    }
    if (!ferr.empty()) {
        c->latch(CKPT_EIO, s->tmp_path + ": " + ferr);
        if (s->map) munmap(s->map, p.file_bytes());
        if (s->fd >= 0) close(s->fd);
        s->map = nullptr; s->fd = -1;
    }

    if ((e = hipStreamWaitEvent(c->pack_stream, s->ev_boundary, 0)) != hipSuccess) hip_fail("wait boundary", e);
    if (p.n_direct)   // these copies read the tensors themselves
        for (size_t k = 0; k < nk; k++)
            if ((e = hipStreamWaitEvent(c->dma[k], s->ev_boundary, 0)) != hipSuccess) hip_fail("wait boundary", e);
    double bp_ms = 0;
    // Pack launches run `ahead` super-chunks in front of the copies: as far as staging allows when the
    // window closes with the last pack (policy PACK: get the reads of the tensors over with), two
    // otherwise (under the paper's rule nothing is gained by packing earlier, and a burst of pack
    // kernels would only compete with the forward pass). Pack sc waits, on the device, for the copies of
    // super-chunk sc - ahead, which also frees its staging slot (ahead <= n_stage, copies are in order).
    // The copies further down may block this thread on ring back-pressure; pack launches are
    // therefore enqueued before the copies they do not depend on.
    const uint64_t ahead = c->cfg.window_policy == CKPT_WINDOW_PACK ? c->n_stage : std::min<uint64_t>(c->n_stage, 2);
    auto enqueue_pack = [&](uint64_t sc) {
        const uint64_t stage = sc % c->n_stage;
        if (sc >= ahead)
            for (size_t k = 0; k < nk; k++)
                if ((e = hipStreamWaitEvent(c->pack_stream, c->ev_stage_done[(sc - ahead) % c->n_stage][k], 0)) != hipSuccess) hip_fail("wait stage", e);
        if ((e = hipEventRecord(c->ev_pack_start[sc], c->pack_stream)) != hipSuccess) hip_fail("record", e);
        const uint64_t t0 = p.sc_first_tile[sc], t1 = p.sc_first_tile[sc + 1];
        if ((e = launch_pack(c->dev_tiles + t0, t1 - t0, c->staging + stage * SC, sc * SC, c->pack_stream)) != hipSuccess) hip_fail("pack launch", e);
        if ((e = hipEventRecord(c->ev_packed[sc], c->pack_stream)) != hipSuccess) hip_fail("record", e);
        if (sc + 1 == p.n_superchunks) {   // every read of the tensors is now in the pack stream
            std::lock_guard<std::mutex> lk(c->mu);
            s->packs_submitted = true;
            c->cv_state.notify_all();
        }
    };
    for (uint64_t sc = 0; sc < std::min<uint64_t>(ahead, p.n_superchunks); sc++) enqueue_pack(sc);
    for (uint64_t sc = 0; sc < p.n_superchunks; sc++) {
        const uint64_t stage = sc % c->n_stage;
        uint8_t *stage_base = c->staging + stage * SC;
        for (size_t k = 0; k < nk; k++)
            if ((e = hipStreamWaitEvent(c->dma[k], c->ev_packed[sc], 0)) != hipSuccess) hip_fail("wait packed", e);

        const uint64_t c0 = sc * (SC / CH);
        const uint64_t c1 = std::min<uint64_t>(p.n_chunks, c0 + SC / CH);
        for (uint64_t ch = c0; ch < c1; ch++) {
            const size_t k = ch % nk;
            const uint64_t slot = c->ring_next++ % c->n_slots;
            {
                std::unique_lock<std::mutex> lk(c->mu);
                if (c->slot_state[slot] != SLOT_FREE) {
                    auto w0 = Clock::now();
                    c->cv_state.wait(lk, [&] { return c->slot_state[slot] == SLOT_FREE; });
                    bp_ms += ms_between(w0, Clock::now());
                }
                c->slot_state[slot] = SLOT_BUSY;
            }
            const uint64_t nbytes = p.chunk_bytes(ch);
            if (ch == 0 && (e = hipEventRecord(c->ev_first_copy, c->dma[k])) != hipSuccess) hip_fail("record", e);
            // the chunk's segments: packed bytes out of staging, large tensors out of their own memory,
            // the padding behind those zero-filled here (the slot belongs to this thread until the copy event)
            uint8_t *slot_base = c->ring + slot * CH;
            for (uint64_t j = p.chunk_first_seg[ch]; j < p.chunk_first_seg[ch + 1]; j++) {
                const ckpt_segment &sg = p.segs[j];
                uint8_t *dst = slot_base + (sg.data_off - ch * CH);
                if (sg.kind == CKPT_SEG_ZERO) { memset(dst, 0, sg.nbytes); continue; }
                if (sg.kind == CKPT_SEG_HOST) {   // from the copy taken at the request
                    const TensorInfo &ti = p.tensors[sg.tensor];
                    memcpy(dst, s->host_capture.data() + ti.capture_off + (sg.src - ti.dev_addr), sg.nbytes);
                    continue;
                }
                const void *src = sg.kind == CKPT_SEG_DIRECT ? reinterpret_cast<const void *>(sg.src)
                                                             : static_cast<const void *>(stage_base + (sg.data_off - sc * SC));
                e = hipMemcpyAsync(dst, src, sg.nbytes, hipMemcpyDeviceToHost, c->dma[k]);
                if (e != hipSuccess) hip_fail("hipMemcpyAsync D2H", e);
            }
            if ((e = hipEventRecord(c->ev_slot[slot], c->dma[k])) != hipSuccess) hip_fail("record", e);
            const bool last = ch + 1 == p.n_chunks;
            if (ch + 1 == c1)
                for (size_t kk = 0; kk < nk; kk++)
                    if ((e = hipEventRecord(c->ev_stage_done[stage][kk], c->dma[kk])) != hipSuccess) hip_fail("record", e);
            if (last)
                for (size_t kk = 0; kk < nk; kk++)
                    if ((e = hipEventRecord(c->ev_job_tail[kk], c->dma[kk])) != hipSuccess) hip_fail("record", e);
            IoJob job;
            job.kind = IoJob::WRITE;
            job.snap = sp;
            job.slot = slot;
            job.file_off = p.header_bytes + ch * CH;
            job.nbytes = nbytes;
            job.last = last;
            {
                std::lock_guard<std::mutex> lk(c->mu);
                c->io_q.push_back(std::move(job));
            }
            c->cv_io.notify_one();
        }
        if (sc + ahead < p.n_superchunks) enqueue_pack(sc + ahead);
    }
    std::vector<uint8_t>().swap(s->host_capture);   // every byte of it is in a ring slot by now
    std::lock_guard<std::mutex> lk(c->mu);
    s->backpressure_ms = bp_ms;
    s->t_submitted = Clock::now();
    s->submitted = true;
    c->prev_job = sp;
    c->cv_state.notify_all();
}

static void submit_thread_main(ckpt_ctx *c) {
    (void)hipSetDevice(c->device);
    for (;;) {
        std::shared_ptr<Snap> sp;
        {
            std::unique_lock<std::mutex> lk(c->mu);
            c->cv_submit.wait(lk, [&] { return c->stopping || !c->submit_q.empty(); });
            if (c->submit_q.empty()) return;
            sp = c->submit_q.front();
            c->submit_q.pop_front();
        }
        submit_one(c, sp);
    }
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

    std::unique_ptr<ckpt_ctx> c(new ckpt_ctx);
    c->cfg = rc;
    c->device = cfg->device;
    c->out_dir = cfg->out_dir;
    c->n_slots = rc.host_ring_bytes / rc.dma_chunk_bytes;
    trace("init: creating streams and events");
    c->slot_state.assign(c->n_slots, SLOT_FREE);
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
    trace("init: starting threads");
    c->submit_thread = std::thread(submit_thread_main, c.get());
    for (int i = 0; i < rc.n_io_threads; i++) c->io_threads.emplace_back(io_thread_main, c.get());
    *out = c.release();
    trace("init: done");
    return CKPT_OK;
}

static bool preallocate_file(const std::string &path, uint64_t bytes, int n_threads, bool map_it, bool o_direct, FileSlot *out, std::string *err);

int ckpt_register_tensors(ckpt_ctx *c, const ckpt_tensor_desc *tensors, size_t n) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    if (c->registered) return fail(CKPT_ESTATE, "tensors already registered in this context");
    HIP_TRY(c, hipSetDevice(c->device));
    for (size_t k = 0; tensors && k < n; k++)
        if (!tensors[k].dev_ptr) return fail(CKPT_EINVAL, "tensor " + std::to_string(k) + ": null device pointer");
    std::string err;
    Plan p;
    int r = build_plan(tensors, n, c->cfg, &p, &err);
    if (r) return fail(r, err);
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
    for (uint64_t s = 0; s < p.n_superchunks; s++) {
        hipEvent_t a, b;
        HIP_TRY(c, hipEventCreate(&a));
        HIP_TRY(c, hipEventCreate(&b));
        c->ev_pack_start.push_back(a);
        c->ev_packed.push_back(b);
    }
    c->ev_stage_done.resize(c->n_stage);
    for (uint64_t s = 0; s < c->n_stage; s++)
        for (size_t k = 0; k < c->dma.size(); k++) {
            hipEvent_t ev;
            HIP_TRY(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
            c->ev_stage_done[s].push_back(ev);
        }
    if (posix_memalign(reinterpret_cast<void **>(&c->hdr_buf), 4096, p.header_bytes) != 0) return fail(CKPT_ENOMEM, "header buffer");
    c->plan = std::move(p);
    c->registered = true;
    for (int i = 0; i < c->cfg.prealloc_files; i++) {
        std::string spare = c->out_dir + "/.spare_" + std::to_string(getpid()) + "_" + std::to_string(c->spare_seq++) + ".dsl";
        FileSlot fs;
        if (!preallocate_file(spare, c->plan.file_bytes(), std::min(c->cfg.n_io_threads, 8), c->cfg.io_mode == CKPT_IO_MMAP, c->cfg.o_direct, &fs, &err))
            return fail(CKPT_EIO, err);
        c->spares.push_back(fs);
    }
    return CKPT_OK;
}

// Creates a file of `bytes` bytes with all its pages allocated (zero-filled), several threads writing.
static bool preallocate_file(const std::string &path, uint64_t bytes, int n_threads, bool map_it, bool o_direct, FileSlot *out, std::string *err) {
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

static int take_async_error(ckpt_ctx *c) {
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->async_code == 0) return CKPT_OK;
    int code = c->async_code;
    g_last_error = c->async_err;
    c->async_code = 0;
    c->async_err.clear();
    return code;
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
    sp->chunks_left = c->plan.n_chunks;
    sp->t_request = t0;
    if (c->plan.n_host) {   // host memory is not ordered with the stream: read it now, the caller may change it after this call
        sp->host_capture.resize(c->plan.host_bytes);
        for (const auto &t : c->plan.tensors)
            if (t.host) memcpy(sp->host_capture.data() + t.capture_off, reinterpret_cast<const void *>(t.dev_addr), t.nbytes);
    }
    HIP_TRY(c, hipEventCreate(&sp->ev_boundary));
    hipError_t e = hipEventRecord(sp->ev_boundary, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) { (void)hipEventDestroy(sp->ev_boundary); return fail(CKPT_EHIP, std::string("record boundary: ") + hipGetErrorString(e)); }
    {
        std::lock_guard<std::mutex> lk(c->mu);
        auto old = c->snaps.find(iter);
        if (old != c->snaps.end() && old->second->ev_boundary) (void)hipEventDestroy(old->second->ev_boundary);
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
    std::shared_ptr<Snap> sp;
    {
        std::unique_lock<std::mutex> lk(c->mu);
        sp = c->last_snap;
        if (!sp || sp->window_closed) return CKPT_OK;
        // a device-side wait means something only for events that have been recorded: every copy of the
        // pending snapshot must have been enqueued (policy D2H), or every pack launch (policy PACK)
        const bool pack_only = c->cfg.window_policy == CKPT_WINDOW_PACK;
        c->cv_state.wait(lk, [&] { return sp->submitted || (pack_only && sp->packs_submitted); });
    }
    HIP_TRY(c, hipSetDevice(c->device));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (c->cfg.window_policy == CKPT_WINDOW_PACK) {
        hipEvent_t ev = c->ev_packed[c->plan.n_superchunks - 1];
        HIP_TRY(c, hipStreamWaitEvent(st, ev, 0));
        if (host_block) HIP_TRY(c, hipEventSynchronize(ev));
    } else {
        for (size_t k = 0; k < c->dma.size(); k++) HIP_TRY(c, hipStreamWaitEvent(st, c->ev_job_tail[k], 0));
        if (host_block)
            for (size_t k = 0; k < c->dma.size(); k++) HIP_TRY(c, hipEventSynchronize(c->ev_job_tail[k]));
    }
    std::lock_guard<std::mutex> lk(c->mu);
    sp->window_closed = true;
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
        }
    }
    return take_async_error(c);
}

int ckpt_enable_second_tier(ckpt_ctx *c, const char *dir, int32_t n_threads, int32_t o_direct, int32_t keep_last) {
    if (!c || !dir || !*dir) return fail(CKPT_EINVAL, "null argument");
    if (n_threads < 0 || n_threads > 64 || keep_last < 0) return fail(CKPT_EINVAL, "second tier: n_threads must be 0..64 and keep_last >= 0");
    struct stat st;
    if (stat(dir, &st) != 0 || !S_ISDIR(st.st_mode)) return fail(CKPT_EIO, std::string(dir) + ": not a directory");
    std::lock_guard<std::mutex> lk(c->mu);
    if (c->tier2_on) return fail(CKPT_ESTATE, "second tier already enabled");
    if (!c->snaps.empty()) return fail(CKPT_ESTATE, "second tier must be enabled before the first snapshot");
    if (std::string(dir) == c->out_dir) return fail(CKPT_EINVAL, "second tier must be another directory than out_dir");
    c->tier2_dir = dir;
    c->tier2_threads = n_threads ? n_threads : 2;
    c->tier2_direct = o_direct != 0;
    c->tier2_keep = keep_last;
    c->tier2_on = true;
    c->tier2_thread = std::thread(tier2_thread_main, c);
    return CKPT_OK;
}

int ckpt_wait_second_tier(ckpt_ctx *c, uint64_t iter) {
    if (!c) return fail(CKPT_EINVAL, "null context");
    {
        std::unique_lock<std::mutex> lk(c->mu);
        if (!c->tier2_on) return fail(CKPT_ESTATE, "no second tier enabled");
        if (iter == CKPT_ITER_ALL) {
            c->cv_state.wait(lk, [&] {
                for (auto &kv : c->snaps) if (!kv.second->committed) return false;
                return !c->tier2_waiting && !c->tier2_active;
            });
        } else {
            auto it = c->snaps.find(iter);
            if (it == c->snaps.end()) return fail(CKPT_EINVAL, "no snapshot was requested for this iteration");
            auto sp = it->second;
            c->cv_state.wait(lk, [&] {
                return sp->committed && (sp->tier2_state == CKPT_TIER2_NONE || sp->tier2_state == CKPT_TIER2_DONE || sp->tier2_state == CKPT_TIER2_SKIPPED ||
                                         sp->tier2_state == CKPT_TIER2_FAILED);
            });
            if (sp->tier2_state == CKPT_TIER2_SKIPPED) return fail(CKPT_ESTATE, "superseded by a newer snapshot before the second tier got to it");
            if (sp->tier2_state == CKPT_TIER2_NONE) return fail(CKPT_ESTATE, "the snapshot failed in the first tier and was never offered to the second");
        }
        if (c->tier2_code) {
            int code = c->tier2_code;
            g_last_error = c->tier2_err;
            c->tier2_code = 0;
            c->tier2_err.clear();
            return code;
        }
    }
    return CKPT_OK;
}

int ckpt_second_tier_file_name(ckpt_ctx *c, uint64_t iter, char *buf, size_t cap) {
    if (!c || !buf) return fail(CKPT_EINVAL, "null argument");
    if (!c->tier2_on) return fail(CKPT_ESTATE, "no second tier enabled");
    std::string s = file_name_for(c->tier2_dir, iter);
    if (s.size() + 1 > cap) return fail(CKPT_EINVAL, "buffer too small");
    memcpy(buf, s.c_str(), s.size() + 1);
    return CKPT_OK;
}

int ckpt_get_layout(ckpt_ctx *c, ckpt_layout *out) {
    if (!c || !out) return fail(CKPT_EINVAL, "null argument");
    if (!c->registered) return fail(CKPT_ESTATE, "no tensors registered");
    fill_layout(c->plan, out);
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
    o->payload_bytes = c->plan.payload_bytes;
    o->data_bytes = c->plan.data_bytes;
    o->file_bytes = c->plan.file_bytes();
    o->d2h_done = s.d2h_done;
    o->committed = s.committed;
    o->pack_launches = int32_t(c->plan.n_superchunks);
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

// Everything of a restore that can fail half-way; the caller cleans up the ring afterwards.
static int restore_body(ckpt_ctx *c, int fd, const char *path, hipStream_t stream, uint64_t base, uint64_t *issued_out, uint64_t *iter_out) {
    const Plan &p = c->plan;
    const uint64_t CH = c->cfg.dma_chunk_bytes, SC = c->cfg.pack_superchunk_bytes;
    const size_t nk = c->dma.size();
    struct stat st;
    if (fstat(fd, &st) != 0) return fail(CKPT_EIO, std::string(path) + ": fstat: " + strerror(errno));
    // header: read the first 4 KiB unit, check the fixed fields, then compare the whole header with
    // the registration's (everything but the iteration field must be identical)
    std::string err;
    if (uint64_t(st.st_size) < kAlign) return fail(CKPT_EFORMAT, "file shorter than one header unit");
    uint8_t *hb = c->hdr_buf;
    if (!pread_all(fd, hb, kAlign, 0, &err)) return fail(CKPT_EIO, err);
    auto le = [&](const uint8_t *q, int n) { uint64_t v = 0; for (int i = 0; i < n; i++) v |= uint64_t(q[i]) << (8 * i); return v; };
    if (memcmp(hb, p.header.data(), 8) != 0 || le(hb + 8, 4) != 1 || le(hb + 12, 4) != kAlign || le(hb + 56, 8) != 0)
        return fail(CKPT_EFORMAT, "bad magic, version or alignment");
    const uint64_t f_hb = le(hb + 32, 8), f_db = le(hb + 40, 8), f_fb = le(hb + 48, 8), f_iter = le(hb + 16, 8);
    if (f_hb % kAlign || f_hb < kAlign || f_fb != f_hb + f_db || f_fb != uint64_t(st.st_size))
        return fail(CKPT_EFORMAT, "size fields inconsistent with the file (truncated?)");
    if (le(hb + 24, 8) != p.tensors.size() || f_hb != p.header_bytes || f_db != p.data_bytes)
        return fail(CKPT_EMISMATCH, "tensor count or sizes differ from the registration");
    if (p.header_bytes > kAlign && !pread_all(fd, hb + kAlign, p.header_bytes - kAlign, kAlign, &err)) return fail(CKPT_EIO, err);
    if (memcmp(hb, p.header.data(), 16) != 0 || memcmp(hb + 24, p.header.data() + 24, p.header_bytes - 24) != 0)
        return fail(CKPT_EMISMATCH, "tensor table differs from the registration");

    // earlier work on the caller's stream (which may read or write the tensors) comes first
    HIP_TRY(c, hipEventRecord(c->ev_user, stream));
    HIP_TRY(c, hipStreamWaitEvent(c->pack_stream, c->ev_user, 0));
    if (p.n_direct)   // these copies write the tensors themselves
        for (size_t k = 0; k < nk; k++) HIP_TRY(c, hipStreamWaitEvent(c->dma[k], c->ev_user, 0));

    uint64_t &issued = *issued_out;   // chunks whose file read has been handed to the I/O threads
    auto issue_reads_upto = [&](uint64_t upto) -> int {
        for (; issued < upto && issued < p.n_chunks; issued++) {
            const uint64_t slot = (base + issued) % c->n_slots;
            if (issued >= c->n_slots) HIP_TRY(c, hipEventSynchronize(c->ev_slot[slot]));   // previous chunk's copy out of the slot
            IoJob job;
            job.kind = IoJob::READ;
            job.fd = fd;
            job.slot = slot;
            job.file_off = p.header_bytes + issued * CH;
            job.nbytes = p.chunk_bytes(issued);
            {
                std::lock_guard<std::mutex> lk(c->mu);
                c->slot_state[slot] = SLOT_BUSY;
                c->io_q.push_back(job);
            }
            c->cv_io.notify_one();
        }
        return CKPT_OK;
    };
    for (uint64_t sc = 0; sc < p.n_superchunks; sc++) {
        const uint64_t stage = sc % c->n_stage;
        uint8_t *stage_base = c->staging + stage * SC;
        if (sc >= c->n_stage)   // staging slot still being scattered from
            for (size_t k = 0; k < nk; k++) HIP_TRY(c, hipStreamWaitEvent(c->dma[k], c->ev_packed[sc - c->n_stage], 0));
        const uint64_t c0 = sc * (SC / CH), c1 = std::min<uint64_t>(p.n_chunks, c0 + SC / CH);
        for (uint64_t ch = c0; ch < c1; ch++) {
            int r = issue_reads_upto(ch + c->n_slots);
            if (r != CKPT_OK) return r;
            const uint64_t slot = (base + ch) % c->n_slots;
            {
                std::unique_lock<std::mutex> lk(c->mu);
                c->cv_state.wait(lk, [&] { return c->slot_state[slot] == SLOT_READ_DONE; });
                if (c->async_code) { g_last_error = c->async_err; return c->async_code; }
            }
            const size_t k = ch % nk;
            const uint8_t *slot_base = c->ring + slot * CH;
            for (uint64_t j = p.chunk_first_seg[ch]; j < p.chunk_first_seg[ch + 1]; j++) {
                const ckpt_segment &sg = p.segs[j];
                if (sg.kind == CKPT_SEG_ZERO) continue;
                if (sg.kind == CKPT_SEG_HOST) {   // the slot has been read: host objects are put back by this thread
                    memcpy(reinterpret_cast<void *>(sg.src), slot_base + (sg.data_off - ch * CH), sg.nbytes);
                    continue;
                }
                void *dst = sg.kind == CKPT_SEG_DIRECT ? reinterpret_cast<void *>(sg.src) : static_cast<void *>(stage_base + (sg.data_off - sc * SC));
                HIP_TRY(c, hipMemcpyAsync(dst, slot_base + (sg.data_off - ch * CH), sg.nbytes, hipMemcpyHostToDevice, c->dma[k]));
            }
            HIP_TRY(c, hipEventRecord(c->ev_slot[slot], c->dma[k]));
        }
        for (size_t k = 0; k < nk; k++) {
            HIP_TRY(c, hipEventRecord(c->ev_stage_done[stage][k], c->dma[k]));
            HIP_TRY(c, hipStreamWaitEvent(c->pack_stream, c->ev_stage_done[stage][k], 0));
        }
        const uint64_t t0 = p.sc_first_tile[sc], t1 = p.sc_first_tile[sc + 1];
        HIP_TRY(c, launch_scatter(c->dev_tiles + t0, t1 - t0, stage_base, sc * SC, c->pack_stream));
        HIP_TRY(c, hipEventRecord(c->ev_packed[sc], c->pack_stream));
    }
    HIP_TRY(c, hipStreamWaitEvent(stream, c->ev_packed[p.n_superchunks - 1], 0));
    if (p.n_direct)   // the last copies into large tensors are not followed by a scatter kernel
        for (size_t k = 0; k < nk; k++) {
            HIP_TRY(c, hipEventRecord(c->ev_job_tail[k], c->dma[k]));
            HIP_TRY(c, hipStreamWaitEvent(stream, c->ev_job_tail[k], 0));
        }
    if (iter_out) *iter_out = f_iter;
    return CKPT_OK;
}

int ckpt_restore(ckpt_ctx *c, const char *path, void *stream, uint64_t *iter_out) {
    if (!c || !path) return fail(CKPT_EINVAL, "null argument");
    if (!c->registered) return fail(CKPT_ESTATE, "no tensors registered");
    {
        std::lock_guard<std::mutex> lk(c->mu);
        for (auto &kv : c->snaps) if (!kv.second->committed) return fail(CKPT_ESTATE, "a snapshot is still in flight");
        if (c->restoring) return fail(CKPT_ESTATE, "restore already in progress");
        c->restoring = true;
    }
    int rc = CKPT_OK;
    uint64_t issued = 0;
    const uint64_t base = c->ring_next;
    int fd = -1;
    hipError_t he = hipSetDevice(c->device);
    if (he != hipSuccess) rc = fail(CKPT_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(he));
    if (rc == CKPT_OK) {
        fd = open(path, O_RDONLY | (c->cfg.o_direct ? O_DIRECT : 0));
        if (fd < 0) rc = fail(CKPT_EIO, std::string(path) + ": open: " + strerror(errno));
    }
    if (rc == CKPT_OK) rc = restore_body(c, fd, path, static_cast<hipStream_t>(stream), base, &issued, iter_out);
    // the ring goes back to the snapshot path: all host-to-device copies out of it must be over and
    // every read handed to the I/O threads must have returned, whether or not the restore succeeded
    for (auto s : c->dma) (void)hipStreamSynchronize(s);
    {
        std::unique_lock<std::mutex> lk(c->mu);
        c->cv_state.wait(lk, [&] {
            for (uint64_t i = 0; i < issued; i++) if (c->slot_state[(base + i) % c->n_slots] == SLOT_BUSY) return false;
            return true;
        });
        for (auto &s : c->slot_state) s = SLOT_FREE;
        c->restoring = false;
    }
    c->ring_next = base + issued;
    if (fd >= 0) close(fd);
    if (rc == CKPT_OK) rc = take_async_error(c);
    else { std::lock_guard<std::mutex> lk(c->mu); c->async_code = 0; c->async_err.clear(); }
    return rc;
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
        }
        rc = take_async_error(c);
        if (rc == CKPT_OK && c->tier2_code) { rc = c->tier2_code; g_last_error = c->tier2_err; }
    }
    (void)hipSetDevice(c->device);
    if (c->pack_stream) (void)hipStreamSynchronize(c->pack_stream);
    for (auto s : c->dma) (void)hipStreamSynchronize(s);
    for (auto &kv : c->snaps) if (kv.second->ev_boundary) (void)hipEventDestroy(kv.second->ev_boundary);
    for (auto ev : c->ev_slot) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_pack_start) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_packed) (void)hipEventDestroy(ev);
    for (auto &v : c->ev_stage_done) for (auto ev : v) (void)hipEventDestroy(ev);
    for (auto ev : c->ev_job_tail) (void)hipEventDestroy(ev);
    if (c->ev_first_copy) (void)hipEventDestroy(c->ev_first_copy);
    if (c->ev_user) (void)hipEventDestroy(c->ev_user);
    if (c->pack_stream) (void)hipStreamDestroy(c->pack_stream);
    for (auto s : c->dma) (void)hipStreamDestroy(s);
    if (c->staging) (void)hipFree(c->staging);
    if (c->dev_tiles) (void)hipFree(c->dev_tiles);
    if (c->ring) (void)hipHostFree(c->ring);
    for (auto &sp : c->spares) { sp.close_all(); unlink(sp.path.c_str()); }
    for (auto &kv : c->kept) kv.second.close_all();
    free(c->hdr_buf);
    delete c;
    return rc;
}

}  // extern "C"
