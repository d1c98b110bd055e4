// Internals shared by the engine's source files: the context behind the C ABI, the per-snapshot
// record, the jobs of the I/O threads, and the small helpers all of them use.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
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

#include <dirent.h>
#include <errno.h>
#include <signal.h>
#include <fcntl.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <sys/statvfs.h>
#include <unistd.h>

#include "plan.hpp"

namespace dsllm {
// t_start / t_stop (each may be null): events that receive the kernel's own start and end time
hipError_t launch_pack(const ckpt_tile *dev_tiles, uint64_t n_tiles, void *slot_base, uint64_t slot_data_off, hipStream_t stream,
                       hipEvent_t t_start = nullptr, hipEvent_t t_stop = nullptr);
hipError_t launch_scatter(const ckpt_tile *dev_tiles, uint64_t n_tiles, const void *slot_base, uint64_t slot_data_off, hipStream_t stream);
hipError_t launch_verify_pairs(const PairTile *dev_tiles, uint64_t n_tiles, uint32_t *dev_flag, hipStream_t stream);
hipError_t launch_derive_pairs(const PairTile *dev_tiles, uint64_t n_tiles, hipStream_t stream);
}  // namespace dsllm

using namespace dsllm;
using Clock = std::chrono::steady_clock;


namespace dsllm {
extern thread_local std::string g_last_error;   // text behind ckpt_last_error(), per calling thread
inline int fail(int code, const std::string &msg) { g_last_error = msg; return code; }
inline double ms_between(Clock::time_point a, Clock::time_point b) { return std::chrono::duration<double, std::milli>(b - a).count(); }

// Progress lines on stderr when DSLLM_CKPT_TRACE is set in the environment (set-up stages only).
inline void trace(const char *what) {
    static const bool on = getenv("DSLLM_CKPT_TRACE") != nullptr;
    if (on) { fprintf(stderr, "[dsllm_ckpt] %s\n", what); fflush(stderr); }
}
}  // namespace dsllm

struct ckpt_plan { dsllm::Plan plan; };

namespace dsllm {

// An open checkpoint file. With retention (keep_last > 0) files, descriptors and mappings live on
// after the commit: a retired file is renamed to a hidden spare name and a later snapshot writes
// into the same pages through the same mapping, so the steady-state flush is plain memcpy.
struct FileSlot {
    std::string path;
    int fd = -1;
    uint8_t *map = nullptr;           // whole-file shared mapping when the sink is written through mmap
    uint64_t map_bytes = 0;
    uint64_t bytes = 0;               // size of the file (a spare is reused only for a snapshot of exactly this size)
    void close_all() {
        if (map) munmap(map, map_bytes);
        if (fd >= 0) ::close(fd);
        map = nullptr; fd = -1;
    }
};

struct Snap {
    uint64_t iter = 0;
    // The plan this snapshot is written with: the registration's version-1 plan, or its version-2 plan when
    // derived tensors were declared and the check on the captured state found every pair to hold. Chosen by the
    // submit thread before the first pack launch; null until then.
    const Plan *plan = nullptr;
    const ckpt_tile *dev_tiles = nullptr;   // that plan's tile table on the device
    double verify_ms = -1;                  // device time of the derivation check (-1: none)
    double window_wait_ms = 0;              // host: time the caller spent in ckpt_wait_immutable_window_end for this snapshot
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
    int policy = CKPT_WINDOW_D2H;           // window policy in force when the snapshot was requested
    int tier2_state = CKPT_TIER2_NONE;      // ckpt_tier2_state
    double tier2_ms = -1;                   // host: copy to the second tier, open to rename
    // A failure of THIS snapshot (open, header, copy, event, chunk write, sync): its file never gets a final
    // name, whatever happens to the context-wide latch in the meantime. Guarded by the context mutex.
    bool failed = false;
    int fail_code = 0;
    std::string fail_msg;
};

struct IoJob {
    enum Kind { WRITE, READ, STOP } kind = STOP;
    std::shared_ptr<Snap> snap;   // WRITE
    int fd = -1;                  // READ
    uint64_t slot = 0, file_off = 0, nbytes = 0;
    uint64_t slot_off = 0;        // READ: where in the slot this piece of the chunk goes
    bool last = false;
    uint64_t seq = 0;             // READ: chunk sequence number
};

constexpr uint64_t kReadPiecesPerChunk = 8;   // restore reads a chunk in this many pieces, spread over the I/O threads
constexpr int kBoundaryEvents = 8;          // boundary events created at set-up (snapshots in flight at a time)
constexpr size_t kMaxSnapRecords = 1024;   // per-snapshot records (measurements, states) kept per context

enum SlotState : int { SLOT_FREE = 0, SLOT_BUSY = 1, SLOT_READ_DONE = 2 };

}  // namespace dsllm

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
    // data reduction (format version 2): declared pairs, the plan without the derived tensors, the check's tables
    DerivedPairs pairs;
    bool have_rplan = false;
    Plan rplan;
    ckpt_tile *dev_rtiles = nullptr;
    PairTile *dev_pairs = nullptr;
    uint32_t *dev_flag = nullptr, *host_flag = nullptr;   // verdict of the check: device word, pinned host word it is copied to
    hipEvent_t ev_verify_start = nullptr, ev_verify_done = nullptr, ev_derived = nullptr;
    hipStream_t pack_stream = nullptr;
    std::vector<hipStream_t> dma;
    std::vector<hipEvent_t> ev_slot;                      // per ring slot: copy into/out of the slot done
    std::vector<hipEvent_t> ev_pack_start, ev_pack_end, ev_packed;   // per super-chunk: the kernel's start and end (timing), its completion in the pack stream (ordering)
    std::vector<std::vector<hipEvent_t>> ev_stage_done;   // [stage slot][dma stream]
    std::vector<hipEvent_t> ev_job_tail;                  // per dma stream
    hipEvent_t ev_first_copy = nullptr, ev_user = nullptr;
    uint8_t *hdr_buf = nullptr;                           // 4 KiB-aligned scratch for header writes
    uint64_t ring_next = 0;                               // global chunk counter -> ring slot
    double init_d2h_gbps = -1;                            // one ring slot copied device-to-host at set-up, timed (-1: could not be measured)

    // threads and queues
    std::mutex mu;
    std::condition_variable cv_submit, cv_io, cv_state;   // submit queue / io queue / any state change
    std::deque<std::shared_ptr<Snap>> submit_q;
    std::deque<IoJob> io_q;
    std::vector<int> slot_state;
    std::vector<uint32_t> slot_reads_left;                // restore: pieces of the slot's chunk still being read
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
    bool tier2_on = false, tier2_enabling = false, tier2_direct = false, tier2_stop = false;
    std::string tier2_dir;
    int tier2_threads = 4, tier2_keep = 1, tier2_mode = CKPT_TIER2_NEWEST;
    std::thread tier2_thread, tier2_unlinker;   // the latter is touched by the second-tier thread only (and by destroy after joining it)
    std::condition_variable cv_tier2;
    std::shared_ptr<Snap> tier2_waiting;   // newest committed snapshot not yet picked up (latest wins)
    std::shared_ptr<Snap> tier2_active;    // being copied: its first-tier file must not be recycled
    bool tier2_removals_pending = false;   // superseded second-tier files are still being unlinked
    bool tier2_retire_after = false;       // the active file fell out of the newest keep_last meanwhile
    std::deque<uint64_t> tier2_files;      // iterations present in the second tier, oldest first
    int tier2_code = 0;                    // first failure of a second-tier copy, reported by ckpt_wait_second_tier
    std::string tier2_err;

    std::vector<hipEvent_t> ev_boundary_free;             // boundary events, created at set-up, handed out per request

    void latch(int code, const std::string &msg) {
        std::lock_guard<std::mutex> lk(mu);
        if (async_code == 0) { async_code = code; async_err = msg; }
        cv_state.notify_all();
    }
    // Marks one snapshot as failed (first failure wins) and latches the error for the caller's next call.
    void fail_snapshot(dsllm::Snap *s, int code, const std::string &msg) {
        std::lock_guard<std::mutex> lk(mu);
        if (!s->failed) { s->failed = true; s->fail_code = code; s->fail_msg = msg; }
        if (async_code == 0) { async_code = code; async_err = msg; }
        cv_state.notify_all();
    }
};

#define HIP_TRY(ctx, expr)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail(CKPT_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

namespace dsllm {
// size of the file a snapshot of this registration is expected to have (what spare files are made for)
inline uint64_t expected_file_bytes(const ckpt_ctx *c) { return c->have_rplan ? c->rplan.file_bytes() : c->plan.file_bytes(); }
inline std::string file_name_for(const std::string &dir, uint64_t iter) {
    char buf[64];
    snprintf(buf, sizeof buf, "/ckpt_iter%020llu.dsl", (unsigned long long)iter);
    return dir + buf;
}

// Makes a rename in `dir` durable: the directory entry itself has to reach the disk.
inline bool fsync_dir(const std::string &dir, std::string *err) {
    int fd = open(dir.c_str(), O_RDONLY | O_DIRECTORY);
    if (fd < 0) { *err = dir + ": open: " + strerror(errno); return false; }
    const bool ok = fsync(fd) == 0;
    if (!ok) *err = dir + ": fsync: " + strerror(errno);
    close(fd);
    return ok;
}

inline bool pwrite_all(int fd, const uint8_t *p, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        size_t want = n > (1ull << 30) ? size_t(1ull << 30) : size_t(n);
        ssize_t w = pwrite(fd, p, want, off_t(off));
        if (w < 0) { if (errno == EINTR) continue; *err = std::string("pwrite: ") + strerror(errno); return false; }
        p += w; off += uint64_t(w); n -= uint64_t(w);
    }
    return true;
}

inline bool pread_all(int fd, uint8_t *p, uint64_t n, uint64_t off, std::string *err) {
    while (n) {
        size_t want = n > (1ull << 30) ? size_t(1ull << 30) : size_t(n);
        ssize_t r = pread(fd, p, want, off_t(off));
        if (r < 0) { if (errno == EINTR) continue; *err = std::string("pread: ") + strerror(errno); return false; }
        if (r == 0) { *err = "pread: unexpected end of file"; return false; }
        p += r; off += uint64_t(r); n -= uint64_t(r);
    }
    return true;
}


// io_threads.cpp
void io_thread_main(ckpt_ctx *c);
void retire_locked(ckpt_ctx *c, uint64_t iter);
// second_tier.cpp
void tier2_offer_locked(ckpt_ctx *c, const std::shared_ptr<Snap> &sp);
void tier2_thread_main(ckpt_ctx *c);
// submit.cpp
void submit_thread_main(ckpt_ctx *c);
// pack_image.hip
int pack_scratch_setup();
// engine.cpp
int take_async_error(ckpt_ctx *c);
bool preallocate_file(const std::string &path, uint64_t bytes, int n_threads, bool map_it, bool o_direct, FileSlot *out, std::string *err);
}  // namespace dsllm

