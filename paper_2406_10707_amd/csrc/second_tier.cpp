// The second storage tier: committed first-tier files are copied on to a slower, durable directory.
#include "engine_internal.hpp"

using namespace dsllm;

// Hands a freshly committed snapshot to the second tier. A snapshot still waiting there is
// superseded: the slower tier always takes the newest state it can get. c->mu held.
void dsllm::tier2_offer_locked(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    if (!c->tier2_on) return;
    if (c->tier2_waiting) c->tier2_waiting->tier2_state = CKPT_TIER2_SKIPPED;
    sp->tier2_state = CKPT_TIER2_QUEUED;
    c->tier2_waiting = sp;
    c->cv_tier2.notify_all();
}


// Copies one committed first-tier file to the second-tier directory: n threads take 8 MiB blocks in
// turn, from the kept mapping when there is one (tmpfs pages: a memory read), else with pread;
// fsync, rename, then older second-tier files beyond tier2_keep are removed.
static void tier2_copy(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    const uint64_t total = sp->plan->file_bytes(), blk = 8ull << 20;
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
        // direct I/O straight out of the first tier's mapping (page-aligned offsets, page-cache or tmpfs pages);
        // if the kernel refuses those pages the block goes through an aligned buffer, as without a mapping
        std::atomic<bool> from_map_ok{true};
        auto worker = [&] {
            uint8_t *buf = nullptr;
            auto need_buf = [&]() -> bool {
                if (buf || posix_memalign(reinterpret_cast<void **>(&buf), 4096, blk) == 0) return true;
                buf = nullptr;
                std::lock_guard<std::mutex> lk(emu);
                if (err.empty()) err = "no memory for a copy buffer";
                return false;
            };
            for (;;) {
                const uint64_t b = next.fetch_add(1);
                if (b >= n_blk) break;
                { std::lock_guard<std::mutex> lk(emu); if (!err.empty()) break; }
                const uint64_t off = b * blk, n = std::min(blk, total - off);   // file sizes are 4 KiB multiples
                std::string e;
                const uint8_t *from;
                if (src_map) {
                    if (!c->tier2_direct) from = src_map + off;
                    else {
                        if (from_map_ok && pwrite_all(dst_fd, src_map + off, n, off, &e)) continue;
                        from_map_ok = false;
                        e.clear();
                        if (!need_buf()) break;
                        memcpy(buf, src_map + off, n);
                        from = buf;
                    }
                } else {
                    if (!need_buf()) break;
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
    else fsync_dir(c->tier2_dir, &err);   // this tier is the durable one: the new name has to be on the disk too
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
    // removing a file of tens of GB takes seconds on a disk file system: off this thread, which has the next copy to start
    if (c->tier2_unlinker.joinable()) c->tier2_unlinker.join();
    if (!drop.empty()) {
        { std::lock_guard<std::mutex> lk(c->mu); c->tier2_removals_pending = true; }
        c->tier2_unlinker = std::thread([c, drop] {
            for (uint64_t it : drop) unlink(file_name_for(c->tier2_dir, it).c_str());
            std::lock_guard<std::mutex> lk(c->mu);
            c->tier2_removals_pending = false;
            c->cv_state.notify_all();
        });
    }
}

void dsllm::tier2_thread_main(ckpt_ctx *c) {
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
            c->cv_state.notify_all();   // the waiting place is free again (mode EVERY: the next snapshot may start)
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


extern "C" {

int ckpt_enable_second_tier(ckpt_ctx *c, const char *dir, int32_t n_threads, int32_t o_direct, int32_t keep_last, int32_t mode) {
    if (!c || !dir || !*dir) return fail(CKPT_EINVAL, "null argument");
    if (mode != CKPT_TIER2_NEWEST && mode != CKPT_TIER2_EVERY) return fail(CKPT_EINVAL, "second tier: unknown mode");
    if (n_threads < 0 || n_threads > 64 || keep_last < 0) return fail(CKPT_EINVAL, "second tier: n_threads must be 0..64 and keep_last >= 0");
    struct stat st;
    if (stat(dir, &st) != 0 || !S_ISDIR(st.st_mode)) return fail(CKPT_EIO, std::string(dir) + ": not a directory");
    bool want_spare = false;
    std::string spare;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (c->tier2_on || c->tier2_enabling) return fail(CKPT_ESTATE, "second tier already enabled");
        if (!c->snaps.empty()) return fail(CKPT_ESTATE, "second tier must be enabled before the first snapshot");
        if (std::string(dir) == c->out_dir) return fail(CKPT_EINVAL, "second tier must be another directory than out_dir");
        c->tier2_enabling = true;   // snapshots are refused until the tier is ready (ckpt_snapshot_async checks this)
        want_spare = c->registered && c->cfg.prealloc_files > 0;
        if (want_spare) spare = c->out_dir + "/.spare_" + std::to_string(getpid()) + "_" + std::to_string(c->spare_seq++) + ".dsl";
    }
    // the file under copy to this tier is exempt from recycling: one more spare keeps page allocation off the
    // write path. Writing a whole file of zeros takes seconds to minutes: not under the context's mutex.
    FileSlot fs;
    std::string err;
    const bool spare_ok = !want_spare || preallocate_file(spare, expected_file_bytes(c), std::min(c->cfg.n_io_threads, 8),
                                                          c->cfg.io_mode == CKPT_IO_MMAP, c->cfg.o_direct, &fs, &err);
    std::lock_guard<std::mutex> lk(c->mu);
    c->tier2_enabling = false;
    if (!spare_ok) return fail(CKPT_EIO, err);
    if (want_spare) c->spares.push_back(fs);
    c->tier2_dir = dir;
    c->tier2_threads = n_threads ? n_threads : 4;
    c->tier2_direct = o_direct != 0;
    c->tier2_keep = keep_last;
    c->tier2_mode = mode;
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
                return !c->tier2_waiting && !c->tier2_active && !c->tier2_removals_pending;
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

}  // extern "C"
