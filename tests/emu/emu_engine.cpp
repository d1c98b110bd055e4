// The whole snapshot engine on the CPU, against the model runtime of hip/hip_runtime.h in this
// folder, meant to be built with -fsanitize=thread: caller thread, submit thread, I/O threads and one
// thread per stream all run for real, so ThreadSanitizer sees every pair of accesses that the
// engine's event graph fails to order (the update writing tensors a pack kernel still reads, a copy
// reading staging before the pack wrote it, a ring slot reused before it was written out, ...).
// The files are compared with images built here by plain memcpy.
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include <atomic>
#include <functional>

#include <errno.h>
#include <signal.h>
#include <sys/stat.h>
#include <sys/uio.h>
#include <unistd.h>

#include "../../include/ckpt.h"
#include "hip/hip_runtime.h"

thread_local dim3 threadIdx, blockIdx, blockDim, gridDim;

// Every pwrite of the engine comes through here (hip/hip_runtime.h redirects the name). The hook sees
// (fd, offset, size) and returns 0 to let the write happen or an errno value to make it fail.
static std::function<int(int, off_t, size_t)> g_pwrite_hook;
ssize_t emu_pwrite(int fd, const void *buf, size_t n, off_t off) {
    if (g_pwrite_hook) {
        const int e = g_pwrite_hook(fd, off, n);
        if (e) { errno = e; return -1; }
    }
    struct iovec iov = {const_cast<void *>(buf), n};
    return pwritev(fd, &iov, 1, off);
}

static uint64_t rng_state;
static uint64_t rnd() {
    rng_state += 0x9E3779B97F4A7C15ull;
    uint64_t z = rng_state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

#define REQUIRE(cond)                                                                        \
    do {                                                                                     \
        if (!(cond)) { printf("FAILED %s line %d: %s (%s)\n", #cond, __LINE__, ckpt_last_error(), what.c_str()); return 1; } \
    } while (0)

struct Tensor { uint8_t *base; uint64_t lead, nbytes; std::string name; int64_t shape; bool host = false; };

static std::vector<uint8_t> read_file(const std::string &p) {
    std::vector<uint8_t> out;
    FILE *f = fopen(p.c_str(), "rb");
    if (!f) return out;
    fseek(f, 0, SEEK_END);
    long n = ftell(f);
    fseek(f, 0, SEEK_SET);
    out.resize(n);
    if (n && fread(out.data(), 1, n, f) != size_t(n)) out.clear();
    fclose(f);
    return out;
}

static int scenario(const std::string &dir, int policy, int keep_last, int io_mode, uint64_t ring_bytes, uint64_t staging_bytes, int n_tensors,
                    uint64_t direct_min = 0, bool second_tier = false, bool host_objects = false, int tier2_mode = CKPT_TIER2_NEWEST) {
    std::string what = "policy " + std::to_string(policy) + " keep_last " + std::to_string(keep_last) + " io_mode " + std::to_string(io_mode) +
                       " direct_min " + std::to_string(direct_min) + (second_tier ? (tier2_mode == CKPT_TIER2_EVERY ? " second tier (every snapshot)" : " second tier") : "") + (host_objects ? " host objects" : "");
    const std::string title = what;
    std::vector<Tensor> ts;
    for (int k = 0; k < n_tensors; k++) {
        Tensor t;
        t.lead = k < 16 ? k : rnd() % 16;
        switch (rnd() % 4) {
            case 0: t.nbytes = 1 + rnd() % 100; break;
            case 1: t.nbytes = 4096 - 8 + rnd() % 17; break;
            case 2: t.nbytes = 32768 * (1 + rnd() % 3) - 20 + rnd() % 41; break;
            default: t.nbytes = 1 + rnd() % 150000; break;
        }
        t.base = static_cast<uint8_t *>(aligned_alloc(16, (t.lead + t.nbytes + 15) / 16 * 16));
        for (uint64_t i = 0; i < t.lead + t.nbytes; i++) t.base[i] = uint8_t(rnd());
        t.host = host_objects && k % 7 == 3;      // every seventh object lives on the "host": the caller owns it, no stream orders it
        t.name = "t" + std::to_string(k);
        t.shape = int64_t(t.nbytes);
        ts.push_back(t);
    }
    std::vector<ckpt_tensor_desc> descs;
    for (auto &t : ts) {
        ckpt_tensor_desc d{};
        d.name = t.name.c_str(); d.dtype = CKPT_U8 | (t.host ? CKPT_PLACE_HOST : 0); d.ndim = 1; d.shape = &t.shape; d.dev_ptr = t.base + t.lead; d.nbytes = t.nbytes;
        descs.push_back(d);
    }
    ckpt_config cfg{};
    cfg.device = 0;
    cfg.out_dir = dir.c_str();
    cfg.host_ring_bytes = ring_bytes;
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 256 << 10;
    cfg.dev_staging_bytes = staging_bytes;
    cfg.n_dma_streams = 2;
    cfg.n_io_threads = 3;
    cfg.window_policy = policy;
    cfg.io_mode = io_mode;
    cfg.keep_last = keep_last;
    cfg.prealloc_files = keep_last ? 1 : 0;
    cfg.direct_min_bytes = direct_min;
    // leftovers of other runs in the directory: the spare of a process that is gone must disappear, that of a live one stay
    const std::string stale = dir + "/.spare_4194000_7.dsl", alive = dir + "/.spare_1_0.dsl";
    { FILE *f = fopen(stale.c_str(), "wb"); fputs("x", f); fclose(f); f = fopen(alive.c_str(), "wb"); fputs("x", f); fclose(f); }
    ckpt_ctx *ctx = nullptr;
    REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
    REQUIRE(access(stale.c_str(), F_OK) != 0 && access(alive.c_str(), F_OK) == 0);
    unlink(alive.c_str());
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
    const std::string dir2 = dir + "/tier2";
    if (second_tier) {
        mkdir(dir2.c_str(), 0755);
        REQUIRE(ckpt_wait_second_tier(ctx, CKPT_ITER_ALL) == CKPT_ESTATE);      // not enabled yet
        REQUIRE(ckpt_enable_second_tier(ctx, dir.c_str(), 2, 0, 1, tier2_mode) == CKPT_EINVAL);   // same directory as the first tier
        REQUIRE(ckpt_enable_second_tier(ctx, dir2.c_str(), 2, 0, 1, 7) == CKPT_EINVAL);           // unknown mode
        REQUIRE(ckpt_enable_second_tier(ctx, dir2.c_str(), 2, 0, tier2_mode == CKPT_TIER2_EVERY ? 0 : 1, tier2_mode) == CKPT_OK);
        REQUIRE(ckpt_enable_second_tier(ctx, dir2.c_str(), 2, 0, 1, tier2_mode) == CKPT_ESTATE);
    }
    ckpt_layout lay;
    REQUIRE(ckpt_get_layout(ctx, &lay) == CKPT_OK);
    ckpt_plan *plan = nullptr;
    REQUIRE(ckpt_plan_create(descs.data(), descs.size(), &cfg, &plan) == CKPT_OK);
    std::vector<uint64_t> offs(descs.size());
    REQUIRE(ckpt_plan_offsets(plan, offs.data(), offs.size()) == CKPT_OK);

    hipStream_t compute;
    hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
    const int iters = 6;
    std::vector<std::vector<uint8_t>> expect(iters + 1);
    for (int it = 1; it <= iters; it++) {
        // forward/backward stand-in: reads every tensor (must be allowed to overlap the snapshot)
        emu_submit(compute, [&ts] { volatile uint64_t sum = 0; for (auto &t : ts) if (!t.host) for (uint64_t i = 0; i < t.nbytes; i += 64) sum = sum + t.base[t.lead + i]; });
        REQUIRE(ckpt_wait_immutable_window_end(ctx, compute, 0) == CKPT_OK);
        // update: mutates every byte, then the expected image of this boundary is taken, in stream order
        emu_submit(compute, [&ts, it] { for (auto &t : ts) if (!t.host) for (uint64_t i = 0; i < t.nbytes; i++) t.base[t.lead + i] = uint8_t(t.base[t.lead + i] * 31 + it); });
        std::vector<uint8_t> *img = &expect[it];
        img->assign(lay.file_bytes, 0);
        emu_submit(compute, [&ts, &offs, &lay, plan, img, it] {
            ckpt_plan_header(plan, uint64_t(it), img->data(), lay.header_bytes);
            for (size_t k = 0; k < ts.size(); k++) if (!ts[k].host) memcpy(img->data() + offs[k], ts[k].base + ts[k].lead, ts[k].nbytes);
        });
        // host objects: the caller's thread owns them; their state at the request is what the file must hold
        for (size_t k = 0; k < ts.size(); k++) if (ts[k].host) memcpy(img->data() + offs[k], ts[k].base + ts[k].lead, ts[k].nbytes);
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);
        // ... and may change them the moment the call has returned
        for (auto &t : ts) if (t.host) for (uint64_t i = 0; i < t.nbytes; i++) t.base[t.lead + i] = uint8_t(t.base[t.lead + i] * 13 + it);
    }
    REQUIRE(ckpt_flush(ctx, CKPT_ITER_ALL) == CKPT_OK);
    hipStreamSynchronize(compute);
    char name[4096];
    for (int it = 1; it <= iters; it++) {
        REQUIRE(ckpt_file_name(ctx, uint64_t(it), name, sizeof name) == CKPT_OK);
        std::vector<uint8_t> got = read_file(name);
        const bool should_exist = keep_last == 0 || it > iters - keep_last;
        if (!should_exist) { REQUIRE(got.empty()); continue; }
        what = "iteration " + std::to_string(it);
        REQUIRE(got == expect[it]);
        ckpt_stats st;
        REQUIRE(ckpt_get_stats(ctx, uint64_t(it), &st) == CKPT_OK && st.committed == 1 && st.d2h_done == 1);
    }
    if (second_tier) {
        // the slower tier ends with the newest snapshot, whole; older ones were copied or skipped, never torn
        what = "second tier";
        REQUIRE(ckpt_wait_second_tier(ctx, CKPT_ITER_ALL) == CKPT_OK);
        int done = 0;
        for (int it = 1; it <= iters; it++) {
            ckpt_stats st;
            REQUIRE(ckpt_get_stats(ctx, uint64_t(it), &st) == CKPT_OK);
            REQUIRE(st.tier2_state == CKPT_TIER2_DONE || st.tier2_state == CKPT_TIER2_SKIPPED);
            REQUIRE((st.tier2_state == CKPT_TIER2_DONE) == (ckpt_wait_second_tier(ctx, uint64_t(it)) == CKPT_OK));
            done += st.tier2_state == CKPT_TIER2_DONE;
            REQUIRE(ckpt_second_tier_file_name(ctx, uint64_t(it), name, sizeof name) == CKPT_OK);
            std::vector<uint8_t> got = read_file(name);
            if (tier2_mode == CKPT_TIER2_EVERY) { REQUIRE(st.tier2_state == CKPT_TIER2_DONE && got == expect[it]); }   // none skipped, all kept
            else if (it == iters) { REQUIRE(st.tier2_state == CKPT_TIER2_DONE && got == expect[it]); }
            else REQUIRE(got.empty());      // second-tier retention keeps one file
        }
        printf("   second tier: %d of %d snapshots copied, the others superseded\n", done, iters);
    }
    // restore the newest file into poisoned tensors; bytes around the tensors must stay untouched
    for (auto &t : ts) memset(t.base, 0xA5, (t.lead + t.nbytes + 15) / 16 * 16);
    uint64_t got_iter = 0;
    REQUIRE(ckpt_file_name(ctx, uint64_t(iters), name, sizeof name) == CKPT_OK);
    REQUIRE(ckpt_restore(ctx, name, compute, &got_iter) == CKPT_OK && got_iter == uint64_t(iters));
    hipStreamSynchronize(compute);
    for (size_t k = 0; k < ts.size(); k++) {
        what = "restore tensor " + std::to_string(k);
        REQUIRE(memcmp(ts[k].base + ts[k].lead, expect[iters].data() + offs[k], ts[k].nbytes) == 0);
        for (uint64_t i = 0; i < ts[k].lead; i++) REQUIRE(ts[k].base[i] == 0xA5);
        for (uint64_t i = ts[k].lead + ts[k].nbytes; i < (ts[k].lead + ts[k].nbytes + 15) / 16 * 16; i++) REQUIRE(ts[k].base[i] == 0xA5);
    }
    // errors: a file of the wrong size, then the directory disappears under a snapshot
    what = "error paths";
    std::string bad = dir + "/bad.dsl";
    { FILE *f = fopen(bad.c_str(), "wb"); fwrite(expect[iters].data(), 1, expect[iters].size() - 4096, f); fclose(f); }
    REQUIRE(ckpt_restore(ctx, bad.c_str(), compute, nullptr) == CKPT_EFORMAT);
    REQUIRE(ckpt_snapshot_async(ctx, 100, compute) == CKPT_OK);
    REQUIRE(ckpt_snapshot_async(ctx, 101, compute) == CKPT_ESTATE);       // window of 100 not closed
    REQUIRE(ckpt_flush(ctx, 100) == CKPT_OK);
    REQUIRE(ckpt_flush(ctx, 555) == CKPT_EINVAL);
    hipStreamSynchronize(compute);
    REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    ckpt_plan_destroy(plan);
    hipStreamDestroy(compute);
    for (auto &t : ts) free(t.base);
    printf("ok %s: %d tensors (%llu direct), %llu data bytes, %llu super-chunks, %llu chunks, %llu segments\n", title.c_str(),
           n_tensors, (unsigned long long)lay.n_direct_tensors, (unsigned long long)lay.data_bytes, (unsigned long long)lay.n_superchunks,
           (unsigned long long)lay.n_chunks, (unsigned long long)lay.n_segments);
    return 0;
}

// ---- a chunk write fails, the caller takes the latched error through a call about ANOTHER iteration,
// then the failed snapshot's last chunk is written: its file must never get a final name.
static int failed_chunk_scenario(const std::string &dir, int keep_last) {
    std::string what = "failed chunk, keep_last " + std::to_string(keep_last);
    const int n_tensors = 24;
    std::vector<Tensor> ts;
    for (int k = 0; k < n_tensors; k++) {
        Tensor t;
        t.lead = k % 16;
        t.nbytes = 20000 + 7919 * k;
        t.base = static_cast<uint8_t *>(aligned_alloc(16, (t.lead + t.nbytes + 15) / 16 * 16));
        for (uint64_t i = 0; i < t.lead + t.nbytes; i++) t.base[i] = uint8_t(rnd());
        t.name = "t" + std::to_string(k);
        t.shape = int64_t(t.nbytes);
        ts.push_back(t);
    }
    std::vector<ckpt_tensor_desc> descs;
    for (auto &t : ts) {
        ckpt_tensor_desc d{};
        d.name = t.name.c_str(); d.dtype = CKPT_U8; d.ndim = 1; d.shape = &t.shape; d.dev_ptr = t.base + t.lead; d.nbytes = t.nbytes;
        descs.push_back(d);
    }
    ckpt_config cfg{};
    cfg.out_dir = dir.c_str();
    cfg.host_ring_bytes = 256 << 10;
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 256 << 10;
    cfg.n_dma_streams = 2;
    cfg.n_io_threads = 3;
    cfg.io_mode = CKPT_IO_PWRITE;
    cfg.keep_last = keep_last;
    cfg.prealloc_files = keep_last ? 1 : 0;
    ckpt_ctx *ctx = nullptr;
    REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
    ckpt_layout lay;
    REQUIRE(ckpt_get_layout(ctx, &lay) == CKPT_OK && lay.n_chunks >= 6);
    hipStream_t compute;
    hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
    auto update = [&](int it) { emu_submit(compute, [&ts, it] { for (auto &t : ts) for (uint64_t i = 0; i < t.nbytes; i++) t.base[t.lead + i] = uint8_t(t.base[t.lead + i] * 31 + it); }); };
    char name[4096];
    for (int it = 1; it <= 2; it++) {
        update(it);
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);
        REQUIRE(ckpt_flush(ctx, uint64_t(it)) == CKPT_OK);
    }
    // snapshot 3: the write of chunk 1 fails; the write of the last chunk is held back until told to go
    std::mutex m;
    std::condition_variable cv;
    bool failed_seen = false, go = false;
    const off_t bad_off = off_t(lay.header_bytes + 1 * lay.dma_chunk_bytes), last_off = off_t(lay.header_bytes + (lay.n_chunks - 1) * lay.dma_chunk_bytes);
    g_pwrite_hook = [&](int, off_t off, size_t) -> int {
        std::unique_lock<std::mutex> lk(m);
        if (off == bad_off) { failed_seen = true; cv.notify_all(); return ENOSPC; }
        if (off == last_off) cv.wait(lk, [&] { return go; });
        return 0;
    };
    update(3);
    REQUIRE(ckpt_snapshot_async(ctx, 3, compute) == CKPT_OK);
    { std::unique_lock<std::mutex> lk(m); cv.wait(lk, [&] { return failed_seen; }); }
    // the caller asks about iteration 2 (committed long ago): it is handed the latched error, which clears the latch
    int r = ckpt_flush(ctx, 2);
    for (int spin = 0; r == CKPT_OK && spin < 2000; spin++) { usleep(1000); r = ckpt_flush(ctx, 2); }   // the latch follows the failed write by a moment
    REQUIRE(r == CKPT_EIO);
    { std::lock_guard<std::mutex> lk(m); go = true; cv.notify_all(); }
    REQUIRE(ckpt_flush(ctx, 3) == CKPT_EIO);          // the failed snapshot still says so itself
    REQUIRE(ckpt_flush(ctx, 3) == CKPT_EIO);          // ... every time it is asked about
    g_pwrite_hook = nullptr;
    REQUIRE(ckpt_file_name(ctx, 3, name, sizeof name) == CKPT_OK);
    REQUIRE(access(name, F_OK) != 0);                  // no file under the final name
    REQUIRE(access((std::string(name) + ".tmp").c_str(), F_OK) != 0);
    uint64_t latest = 0;
    REQUIRE(ckpt_find_latest(dir.c_str(), &latest, nullptr, 0) == CKPT_OK && latest == 2);
    // the context goes on working, and with retention the spare pool is not poisoned by the torn file
    for (int it = 4; it <= 6; it++) {
        update(it);
        std::vector<uint8_t> img(lay.file_bytes, 0);
        ckpt_plan *plan = nullptr;
        REQUIRE(ckpt_plan_create(descs.data(), descs.size(), &cfg, &plan) == CKPT_OK);
        std::vector<uint64_t> offs(descs.size());
        REQUIRE(ckpt_plan_offsets(plan, offs.data(), offs.size()) == CKPT_OK);
        emu_submit(compute, [&, it] {
            ckpt_plan_header(plan, uint64_t(it), img.data(), lay.header_bytes);
            for (size_t k = 0; k < ts.size(); k++) memcpy(img.data() + offs[k], ts[k].base + ts[k].lead, ts[k].nbytes);
        });
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);
        REQUIRE(ckpt_flush(ctx, uint64_t(it)) == CKPT_OK);
        hipStreamSynchronize(compute);
        REQUIRE(ckpt_file_name(ctx, uint64_t(it), name, sizeof name) == CKPT_OK);
        REQUIRE(read_file(name) == img);
        ckpt_plan_destroy(plan);
    }
    REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    hipStreamDestroy(compute);
    for (auto &t : ts) free(t.base);
    printf("ok %s\n", what.c_str());
    return 0;
}

// ---- nothing is enqueued before the boundary: the caller's host is ahead of its device (the stream still has a long
// forward pass to run when the snapshot is requested). Until the device reaches the boundary the library must not put
// anything on its own streams: work parked behind an unsignalled event slows every launch of the caller (measured on
// the GPU). Then the snapshot proceeds and the file is the state at the boundary.
static hipStream_t g_callers_stream = nullptr;
static std::atomic<bool> g_boundary_held{false};
static std::atomic<int> g_early_submissions{0};
static void count_early(hipStream_t s) { if (g_boundary_held.load() && s != g_callers_stream) g_early_submissions++; }

static int held_boundary_scenario(const std::string &dir, int policy) {
    std::string what = "held boundary, policy " + std::to_string(policy);
    std::vector<Tensor> ts;
    for (int k = 0; k < 20; k++) {
        Tensor t;
        t.lead = (5 * k) % 16;
        t.nbytes = 30000 + 6101 * k;
        t.base = static_cast<uint8_t *>(aligned_alloc(16, (t.lead + t.nbytes + 15) / 16 * 16));
        for (uint64_t i = 0; i < t.lead + t.nbytes; i++) t.base[i] = uint8_t(rnd());
        t.name = "t" + std::to_string(k);
        t.shape = int64_t(t.nbytes);
        ts.push_back(t);
    }
    std::vector<ckpt_tensor_desc> descs;
    for (auto &t : ts) {
        ckpt_tensor_desc d{};
        d.name = t.name.c_str(); d.dtype = CKPT_U8; d.ndim = 1; d.shape = &t.shape; d.dev_ptr = t.base + t.lead; d.nbytes = t.nbytes;
        descs.push_back(d);
    }
    ckpt_config cfg{};
    cfg.out_dir = dir.c_str();
    cfg.host_ring_bytes = 256 << 10;
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 128 << 10;
    cfg.n_dma_streams = 2;
    cfg.n_io_threads = 2;
    cfg.window_policy = policy;
    ckpt_ctx *ctx = nullptr;
    REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
    ckpt_layout lay;
    REQUIRE(ckpt_get_layout(ctx, &lay) == CKPT_OK && lay.n_superchunks >= 4);
    ckpt_plan *plan = nullptr;
    REQUIRE(ckpt_plan_create(descs.data(), descs.size(), &cfg, &plan) == CKPT_OK);
    std::vector<uint64_t> offs(descs.size());
    REQUIRE(ckpt_plan_offsets(plan, offs.data(), offs.size()) == CKPT_OK);
    hipStream_t compute;
    hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
    g_callers_stream = compute;
    g_emu_submit_hook = count_early;
    char name[4096];
    for (int it = 1; it <= 3; it++) {
        std::mutex m;
        std::condition_variable cv;
        bool release = false;
        std::vector<uint8_t> img(lay.file_bytes, 0);
        // the "forward pass and update" the device has not finished yet: it ends when the test lets it
        g_boundary_held = true;
        emu_submit(compute, [&, it] {
            { std::unique_lock<std::mutex> lk(m); cv.wait(lk, [&] { return release; }); }
            for (auto &t : ts) for (uint64_t i = 0; i < t.nbytes; i++) t.base[t.lead + i] = uint8_t(t.base[t.lead + i] * 29 + it);
            ckpt_plan_header(plan, uint64_t(it), img.data(), lay.header_bytes);
            for (size_t k = 0; k < ts.size(); k++) memcpy(img.data() + offs[k], ts[k].base + ts[k].lead, ts[k].nbytes);
            g_boundary_held = false;      // the next thing in this stream is the boundary event
        });
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);      // returns at once, boundary not reached
        usleep(150 * 1000);                                                          // time for a premature enqueue to happen
        REQUIRE(g_early_submissions.load() == 0);
        { std::lock_guard<std::mutex> lk(m); release = true; cv.notify_all(); }
        REQUIRE(ckpt_wait_immutable_window_end(ctx, compute, 0) == CKPT_OK);
        REQUIRE(ckpt_flush(ctx, uint64_t(it)) == CKPT_OK);
        hipStreamSynchronize(compute);
        REQUIRE(g_early_submissions.load() == 0);
        REQUIRE(ckpt_file_name(ctx, uint64_t(it), name, sizeof name) == CKPT_OK);
        REQUIRE(read_file(name) == img);
    }
    g_emu_submit_hook = nullptr;
    ckpt_plan_destroy(plan);
    REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    hipStreamDestroy(compute);
    for (auto &t : ts) free(t.base);
    printf("ok %s\n", what.c_str());
    return 0;
}

// ---- data reduction: bf16 copies declared as roundings of f32 masters. The update keeps them so (version-2
// files, the copies left out) except at one iteration, where one element is off (that snapshot must be the full
// version-1 file). Every file against an image built here; restore of both versions into poisoned memory.
static uint16_t rne_bits(uint32_t u) { return (u & 0x7FFFFFFFu) > 0x7F800000u ? uint16_t((u >> 16) | 0x40u) : uint16_t((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16); }

static int derived_scenario(const std::string &dir, int policy, int keep_last, int io_mode, uint64_t direct_min) {
    std::string what = "derived tensors, policy " + std::to_string(policy) + " keep_last " + std::to_string(keep_last) + " direct_min " + std::to_string(direct_min);
    const std::string title = what;
    const int n_params = 9;
    struct Param { uint8_t *p_base, *m_base, *x_base; uint64_t p_lead, m_lead, numel; std::string pn, mn, xn; int64_t shape; int64_t xshape; };
    std::vector<Param> ps(n_params);
    for (int k = 0; k < n_params; k++) {
        Param &q = ps[k];
        q.numel = k == 0 ? 3 : (k == 1 ? 8192 : (k == 2 ? 8193 : 1 + rnd() % 40000));
        q.p_lead = k % 2 ? 2 * (rnd() % 8) : 0;          // element-aligned, some not 8-byte aligned: the element-wise path
        q.m_lead = k % 3 == 1 ? 4 * (rnd() % 4) : 0;
        q.p_base = static_cast<uint8_t *>(aligned_alloc(16, (q.p_lead + 2 * q.numel + 15) / 16 * 16));
        q.m_base = static_cast<uint8_t *>(aligned_alloc(16, (q.m_lead + 4 * q.numel + 15) / 16 * 16));
        q.x_base = static_cast<uint8_t *>(aligned_alloc(16, (4 * q.numel + 15) / 16 * 16));      // a third tensor per parameter, never derived
        q.pn = "w" + std::to_string(k) + ".p_bf16"; q.mn = "w" + std::to_string(k) + ".master"; q.xn = "w" + std::to_string(k) + ".m";
        q.shape = int64_t(q.numel); q.xshape = int64_t(q.numel);
    }
    std::vector<ckpt_tensor_desc> descs;
    std::vector<uint32_t> derived, source;
    for (auto &q : ps) {
        ckpt_tensor_desc d{};
        derived.push_back(uint32_t(descs.size())); source.push_back(uint32_t(descs.size() + 1));
        d.name = q.pn.c_str(); d.dtype = CKPT_BF16; d.ndim = 1; d.shape = &q.shape; d.dev_ptr = q.p_base + q.p_lead; d.nbytes = 2 * q.numel; descs.push_back(d);
        d.name = q.mn.c_str(); d.dtype = CKPT_F32; d.dev_ptr = q.m_base + q.m_lead; d.nbytes = 4 * q.numel; descs.push_back(d);
        d.name = q.xn.c_str(); d.dtype = CKPT_F32; d.shape = &q.xshape; d.dev_ptr = q.x_base; d.nbytes = 4 * q.numel; descs.push_back(d);
    }
    ckpt_config cfg{};
    cfg.out_dir = dir.c_str();
    cfg.host_ring_bytes = 256 << 10;
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 256 << 10;
    cfg.n_dma_streams = 2;
    cfg.n_io_threads = 3;
    cfg.window_policy = policy;
    cfg.io_mode = io_mode;
    cfg.keep_last = keep_last;
    cfg.prealloc_files = keep_last ? 1 : 0;
    cfg.direct_min_bytes = direct_min;
    ckpt_ctx *ctx = nullptr;
    REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
    { uint32_t bad_d = 1, bad_s = 0; REQUIRE(ckpt_declare_derived(ctx, &bad_d, &bad_s, 1) == CKPT_OK); }      // f32 "derived" from bf16: caught at registration
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_EINVAL);
    REQUIRE(ckpt_declare_derived(ctx, derived.data(), source.data(), derived.size()) == CKPT_OK);
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
    REQUIRE(ckpt_declare_derived(ctx, derived.data(), source.data(), derived.size()) == CKPT_ESTATE);
    ckpt_plan *plan1 = nullptr, *plan2 = nullptr;
    REQUIRE(ckpt_plan_create(descs.data(), descs.size(), &cfg, &plan1) == CKPT_OK);
    REQUIRE(ckpt_plan_create_derived(descs.data(), descs.size(), &cfg, derived.data(), source.data(), derived.size(), &plan2) == CKPT_OK);
    ckpt_layout lay1, lay2, layc;
    REQUIRE(ckpt_plan_layout(plan1, &lay1) == CKPT_OK && ckpt_plan_layout(plan2, &lay2) == CKPT_OK && ckpt_get_layout(ctx, &layc) == CKPT_OK);
    REQUIRE(lay1.version == 1 && lay2.version == 2 && lay2.n_derived_tensors == uint64_t(n_params) && lay2.data_bytes < lay1.data_bytes);
    REQUIRE(layc.data_bytes == lay1.data_bytes && layc.reduced_data_bytes == lay2.data_bytes && layc.reduced_header_bytes == lay2.header_bytes);
    std::vector<uint64_t> offs1(descs.size()), offs2(descs.size());
    REQUIRE(ckpt_plan_offsets(plan1, offs1.data(), offs1.size()) == CKPT_OK && ckpt_plan_offsets(plan2, offs2.data(), offs2.size()) == CKPT_OK);

    hipStream_t compute;
    hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
    const int iters = 6, broken_iter = 3;
    std::vector<std::vector<uint8_t>> expect(iters + 1);
    std::vector<int> expect_version(iters + 1, 2);
    expect_version[broken_iter] = 1;
    for (int it = 1; it <= iters; it++) {
        REQUIRE(ckpt_wait_immutable_window_end(ctx, compute, 0) == CKPT_OK);
        // the update: new master bits (all kinds of patterns, NaNs and ties among them), the bf16 copy re-rounded from them
        emu_submit(compute, [&ps, it, broken_iter] {
            for (size_t k = 0; k < ps.size(); k++) {
                Param &q = ps[k];
                for (uint64_t e = 0; e < q.numel; e++) {
                    uint32_t u = uint32_t((e * 2654435761ull + k * 40503ull + uint64_t(it) * 0x9E3779B9ull) ^ (e << 17));
                    if (e % 97 == 5) u = 0x7F800001u + uint32_t(e);            // NaNs
                    if (e % 89 == 7) u = (u & 0xFFFF0000u) | 0x8000u;          // ties
                    memcpy(q.m_base + q.m_lead + 4 * e, &u, 4);
                    uint16_t b = rne_bits(u);
                    memcpy(q.p_base + q.p_lead + 2 * e, &b, 2);
                    uint32_t x = u * 31u + uint32_t(it);
                    memcpy(q.x_base + 4 * e, &x, 4);
                }
            }
            if (it == broken_iter) { Param &q = ps[4]; q.p_base[q.p_lead + 2 * (q.numel - 1)] ^= 1; }   // one bit of one element: the pair no longer holds
        });
        std::vector<uint8_t> *img = &expect[it];
        const bool v2 = expect_version[it] == 2;
        img->assign(v2 ? lay2.file_bytes : lay1.file_bytes, 0);
        emu_submit(compute, [&, img, it, v2] {
            ckpt_plan_header(v2 ? plan2 : plan1, uint64_t(it), img->data(), v2 ? lay2.header_bytes : lay1.header_bytes);
            const std::vector<uint64_t> &offs = v2 ? offs2 : offs1;
            for (size_t j = 0; j < descs.size(); j++) {
                if (v2 && j % 3 == 0) continue;      // the bf16 copies are described, not stored
                memcpy(img->data() + offs[j], descs[j].dev_ptr, descs[j].nbytes);
            }
        });
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);
    }
    REQUIRE(ckpt_flush(ctx, CKPT_ITER_ALL) == CKPT_OK);
    hipStreamSynchronize(compute);
    char name[4096];
    for (int it = 1; it <= iters; it++) {
        ckpt_stats st;
        REQUIRE(ckpt_get_stats(ctx, uint64_t(it), &st) == CKPT_OK && st.committed == 1);
        what = "iteration " + std::to_string(it);
        REQUIRE(st.format_version == expect_version[it]);
        REQUIRE(st.data_bytes == (expect_version[it] == 2 ? lay2.data_bytes : lay1.data_bytes));
        REQUIRE(ckpt_file_name(ctx, uint64_t(it), name, sizeof name) == CKPT_OK);
        std::vector<uint8_t> got = read_file(name);
        const bool should_exist = keep_last == 0 || it > iters - keep_last;
        if (!should_exist) { REQUIRE(got.empty()); continue; }
        REQUIRE(got == expect[it]);
    }
    // restore the newest (version 2) file into poisoned memory: stored tensors come back, derived ones are recomputed
    auto poison = [&] { for (auto &q : ps) { memset(q.p_base, 0xA5, (q.p_lead + 2 * q.numel + 15) / 16 * 16); memset(q.m_base, 0xA5, (q.m_lead + 4 * q.numel + 15) / 16 * 16); memset(q.x_base, 0xA5, (4 * q.numel + 15) / 16 * 16); } };
    auto check_restored = [&](int it) -> bool {
        const bool v2 = expect_version[it] == 2;
        const std::vector<uint64_t> &offs = v2 ? offs2 : offs1;
        for (size_t k = 0; k < ps.size(); k++) {
            Param &q = ps[k];
            if (memcmp(q.m_base + q.m_lead, expect[it].data() + offs[3 * k + 1], 4 * q.numel) != 0) return false;
            if (memcmp(q.x_base, expect[it].data() + offs[3 * k + 2], 4 * q.numel) != 0) return false;
            for (uint64_t e = 0; e < q.numel; e++) {
                uint32_t u; uint16_t b;
                memcpy(&u, q.m_base + q.m_lead + 4 * e, 4); memcpy(&b, q.p_base + q.p_lead + 2 * e, 2);
                uint16_t want = rne_bits(u);
                if (!v2) memcpy(&want, expect[it].data() + offs[3 * k] + 2 * e, 2);
                if (b != want) return false;
            }
            for (uint64_t i = 0; i < q.p_lead; i++) if (q.p_base[i] != 0xA5) return false;                                   // bytes around the tensors untouched
            for (uint64_t i = q.p_lead + 2 * q.numel; i < (q.p_lead + 2 * q.numel + 15) / 16 * 16; i++) if (q.p_base[i] != 0xA5) return false;
            for (uint64_t i = 0; i < q.m_lead; i++) if (q.m_base[i] != 0xA5) return false;
        }
        return true;
    };
    uint64_t got_iter = 0;
    what = "restore of a version-2 file";
    poison();
    REQUIRE(ckpt_file_name(ctx, uint64_t(iters), name, sizeof name) == CKPT_OK);
    REQUIRE(ckpt_restore(ctx, name, compute, &got_iter) == CKPT_OK && got_iter == uint64_t(iters));
    hipStreamSynchronize(compute);
    REQUIRE(check_restored(iters));
    if (keep_last == 0) {
        what = "restore of the version-1 file";
        poison();
        REQUIRE(ckpt_file_name(ctx, uint64_t(broken_iter), name, sizeof name) == CKPT_OK);
        REQUIRE(ckpt_restore(ctx, name, compute, &got_iter) == CKPT_OK && got_iter == uint64_t(broken_iter));
        hipStreamSynchronize(compute);
        REQUIRE(check_restored(broken_iter));
    }
    REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    // a registration that declares nothing refuses the version-2 file
    if (keep_last == 0) {
        what = "version-2 file, nothing declared";
        REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
        REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
        REQUIRE(ckpt_file_name(ctx, uint64_t(iters), name, sizeof name) == CKPT_OK);
        REQUIRE(ckpt_restore(ctx, name, compute, nullptr) == CKPT_EMISMATCH);
        REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    }
    ckpt_plan_destroy(plan1); ckpt_plan_destroy(plan2);
    hipStreamDestroy(compute);
    for (auto &q : ps) { free(q.p_base); free(q.m_base); free(q.x_base); }
    printf("ok %s: version-2 files %llu data bytes instead of %llu\n", title.c_str(), (unsigned long long)lay2.data_bytes, (unsigned long long)lay1.data_bytes);
    return 0;
}

// ---- crash consistency: the process ends itself (SIGKILL) at its kill_at-th file write, somewhere in the
// middle of a flush. Tensor bytes are a closed form of (tensor, byte, iteration), so the parent can tell what
// every file that carries a final name must hold. variant 0: plain files; 1: retention with recycled files;
// 2: second tier that takes every snapshot.
static uint8_t crash_byte(uint64_t k, uint64_t j, uint64_t it) { return uint8_t((j * 2654435761ull + k * 40503ull + it * 97ull) >> 8); }

static int crash_child(const std::string &dir, int variant, long kill_at) {
    std::string what = "crash child";
    const int n_tensors = 12, iters = 5;
    std::vector<Tensor> ts;
    for (int k = 0; k < n_tensors; k++) {
        Tensor t;
        t.lead = 0;
        t.nbytes = 30000 + 9973 * k;
        t.base = static_cast<uint8_t *>(aligned_alloc(16, (t.nbytes + 15) / 16 * 16));
        t.name = "t" + std::to_string(k);
        t.shape = int64_t(t.nbytes);
        ts.push_back(t);
    }
    std::vector<ckpt_tensor_desc> descs;
    for (auto &t : ts) {
        ckpt_tensor_desc d{};
        d.name = t.name.c_str(); d.dtype = CKPT_U8; d.ndim = 1; d.shape = &t.shape; d.dev_ptr = t.base; d.nbytes = t.nbytes;
        descs.push_back(d);
    }
    const std::string dir2 = dir + "/tier2";
    ckpt_config cfg{};
    cfg.out_dir = dir.c_str();
    cfg.host_ring_bytes = 256 << 10;
    cfg.dma_chunk_bytes = 64 << 10;
    cfg.pack_superchunk_bytes = 256 << 10;
    cfg.n_io_threads = 3;
    cfg.io_mode = CKPT_IO_PWRITE;
    cfg.keep_last = variant == 1 ? 1 : 0;
    cfg.prealloc_files = variant == 1 ? 1 : 0;
    ckpt_ctx *ctx = nullptr;
    REQUIRE(ckpt_init(&cfg, &ctx) == CKPT_OK);
    REQUIRE(ckpt_register_tensors(ctx, descs.data(), descs.size()) == CKPT_OK);
    if (variant == 2) { mkdir(dir2.c_str(), 0755); REQUIRE(ckpt_enable_second_tier(ctx, dir2.c_str(), 2, 0, 0, CKPT_TIER2_EVERY) == CKPT_OK); }
    std::atomic<long> writes{0};
    g_pwrite_hook = [&](int, off_t, size_t) -> int {
        if (++writes == kill_at) raise(SIGKILL);
        return 0;
    };
    hipStream_t compute;
    hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
    for (int it = 1; it <= iters; it++) {
        REQUIRE(ckpt_wait_immutable_window_end(ctx, compute, 0) == CKPT_OK);
        emu_submit(compute, [&ts, it] { for (size_t k = 0; k < ts.size(); k++) for (uint64_t j = 0; j < ts[k].nbytes; j++) ts[k].base[j] = crash_byte(k, j, uint64_t(it)); });
        REQUIRE(ckpt_snapshot_async(ctx, uint64_t(it), compute) == CKPT_OK);
    }
    REQUIRE(ckpt_flush(ctx, CKPT_ITER_ALL) == CKPT_OK);
    if (variant == 2) REQUIRE(ckpt_wait_second_tier(ctx, CKPT_ITER_ALL) == CKPT_OK);
    hipStreamSynchronize(compute);
    REQUIRE(ckpt_destroy(ctx) == CKPT_OK);
    hipStreamDestroy(compute);
    printf("survived with %ld writes\n", writes.load());
    return 0;
}

int main(int argc, char **argv) {
    if (argc < 2) { printf("usage: emu_engine <scratch dir> [seed] | --failed-chunk <dir> | --crash <dir> <variant> <kill at write>\n"); return 2; }
    if (std::string(argv[1]) == "--failed-chunk" && argc >= 3) {
        rng_state = 11;
        const std::string root = argv[2];
        for (int keep : {0, 1}) {
            const std::string d = root + "/k" + std::to_string(keep);
            mkdir(d.c_str(), 0755);
            if (failed_chunk_scenario(d, keep)) return 1;
        }
        return 0;
    }
    if (std::string(argv[1]) == "--crash" && argc >= 5) return crash_child(argv[2], atoi(argv[3]), atol(argv[4]));
    if (std::string(argv[1]) == "--held-boundary" && argc >= 3) {
        rng_state = 17;
        const std::string root = argv[2];
        int n = 0;
        for (int policy : {CKPT_WINDOW_D2H, CKPT_WINDOW_PACK}) {
            const std::string d = root + "/h" + std::to_string(n++);
            mkdir(d.c_str(), 0755);
            if (held_boundary_scenario(d, policy)) return 1;
        }
        return 0;
    }
    if (std::string(argv[1]) == "--derived" && argc >= 3) {
        rng_state = argc > 3 ? strtoull(argv[3], 0, 10) : 5;
        const std::string root = argv[2];
        int n = 0;
        auto sub = [&] { std::string d = root + "/d" + std::to_string(n++); mkdir(d.c_str(), 0755); return d; };
        if (derived_scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 0)) return 1;
        if (derived_scenario(sub(), CKPT_WINDOW_D2H, 1, CKPT_IO_MMAP, 0)) return 1;      // recycled spares change size when the version changes
        if (derived_scenario(sub(), CKPT_WINDOW_PACK, 2, CKPT_IO_MMAP, 0)) return 1;
        if (derived_scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 30000)) return 1;  // hybrid: large tensors by direct copy
        return 0;
    }
    rng_state = argc > 2 ? strtoull(argv[2], 0, 10) : 1;
    std::string root = argv[1];
    int n = 0;
    auto sub = [&] { std::string d = root + "/s" + std::to_string(n++); mkdir(d.c_str(), 0755); return d; };
    // ring of 4 slots (much smaller than the data), staging of 2 super-chunks: the paper's rule
    if (scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 256 << 10, 0, 60)) return 1;
    // retention with recycled, mapped files
    if (scenario(sub(), CKPT_WINDOW_D2H, 2, CKPT_IO_MMAP, 256 << 10, 0, 60)) return 1;
    // update released after the pack; staging holds everything
    if (scenario(sub(), CKPT_WINDOW_PACK, 1, CKPT_IO_MMAP, 512 << 10, 64 << 20, 60)) return 1;
    // update released after the pack with only two staging slots (packs depend on copies)
    if (scenario(sub(), CKPT_WINDOW_PACK, 0, CKPT_IO_PWRITE, 128 << 10, 0, 40)) return 1;
    // hybrid: tensors of 30000 bytes and more are copied out of (and on restore into) their own memory
    if (scenario(sub(), CKPT_WINDOW_D2H, 1, CKPT_IO_MMAP, 256 << 10, 0, 60, 30000)) return 1;
    // second tier behind a recycling first tier (the file being copied on must not be recycled under the copy)
    if (scenario(sub(), CKPT_WINDOW_D2H, 1, CKPT_IO_MMAP, 256 << 10, 0, 60, 0, true)) return 1;
    // second tier behind a first tier that keeps every file (read back by path)
    if (scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 256 << 10, 0, 40, 0, true)) return 1;
    // a second tier that takes every snapshot, behind a first tier that recycles its files
    if (scenario(sub(), CKPT_WINDOW_D2H, 1, CKPT_IO_MMAP, 256 << 10, 0, 60, 0, true, false, CKPT_TIER2_EVERY)) return 1;
    // host-resident objects among the tensors, changed by the caller right after each request; with direct copies too
    if (scenario(sub(), CKPT_WINDOW_D2H, 1, CKPT_IO_MMAP, 256 << 10, 0, 60, 0, false, true)) return 1;
    if (scenario(sub(), CKPT_WINDOW_PACK, 0, CKPT_IO_PWRITE, 128 << 10, 0, 60, 0, false, true)) return 1;
    if (scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 256 << 10, 0, 60, 30000, false, true)) return 1;
    // hybrid with everything direct that may be: the pack kernel sees only what is under 4 KiB
    if (scenario(sub(), CKPT_WINDOW_D2H, 0, CKPT_IO_PWRITE, 128 << 10, 0, 60, 4096)) return 1;
    return 0;
}
