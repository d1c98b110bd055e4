// The submit thread: enqueues a snapshot's pack launches and device-to-host copies, and blocks on
// ring back-pressure so that the caller never does.
#include "engine_internal.hpp"

using namespace dsllm;

static void submit_one(ckpt_ctx *c, const std::shared_ptr<Snap> &sp) {
    Snap *s = sp.get();
    const uint64_t CH = c->cfg.dma_chunk_bytes, SC = c->cfg.pack_superchunk_bytes;
    const size_t nk = c->dma.size();
    auto hip_fail = [&](const char *what, hipError_t e) { c->fail_snapshot(s, CKPT_EHIP, std::string(what) + ": " + hipGetErrorString(e)); };
    hipError_t e;
    double tier2_wait_ms = 0;

    // one snapshot's copies at a time: the previous one's last copy is over before this one's
    // boundary on the device timeline anyway (the caller closed its window), so this costs nothing there
    if (c->prev_job) {
        for (size_t k = 0; k < nk; k++) if ((e = hipEventSynchronize(c->ev_job_tail[k])) != hipSuccess) hip_fail("tail sync", e);
        std::unique_lock<std::mutex> lk(c->mu);
        // with retention the previous commit is also what retires an older file into the spare pool this
        // snapshot is about to draw from: wait for it (it follows the last copy by one chunk write)
        c->cv_state.wait(lk, [&] { return c->prev_job->d2h_done && (c->cfg.keep_last == 0 || c->prev_job->committed); });
        // a second tier that must receive every snapshot: the previous one has to be on its way there before
        // this one may start (at most one file waits for the slower tier while another is being copied);
        // this is where a slow tier holds training back, through the window wait
        if (c->tier2_on && c->tier2_mode == CKPT_TIER2_EVERY) {
            auto w0 = Clock::now();
            c->cv_state.wait(lk, [&] { return c->prev_job->committed && !c->tier2_waiting; });
            tier2_wait_ms = ms_between(w0, Clock::now());
        }
    }

    // Everything below comes after the boundary on the device timeline. This thread first waits, on the host, until
    // the device has reached the boundary, and only then enqueues the snapshot's kernels and copies. A caller's
    // host thread may be whole steps ahead of its device; work enqueued at request time would sit behind an
    // unsignalled event at the head of the pack and copy queues all that while, and the command processor pays
    // for blocked queues on every dispatch of the caller's own stream: measured, 12 to 20 us per kernel launch, which
    // made every step between a request and its boundary 1.7 % slower (the Adam phase of the 7B workload 42.1
    // instead of 36.2 ms, its GEMM phase +1.1 %). The device-side wait below stays as the ordering guarantee.
    if ((e = hipEventSynchronize(s->ev_boundary)) != hipSuccess) hip_fail("boundary sync", e);
    if ((e = hipStreamWaitEvent(c->pack_stream, s->ev_boundary, 0)) != hipSuccess) hip_fail("wait boundary", e);

    // Data reduction: with derived tensors declared, the captured state is checked on the device first (every bf16
    // copy against the rounding of its f32 source). The verdict decides which of the registration's two plans this
    // snapshot is written with; this thread waits for it (some milliseconds after the boundary), the caller does not.
    const Plan *chosen = &c->plan;
    const ckpt_tile *chosen_tiles = c->dev_tiles;
    if (c->have_rplan) {
        bool launched = true;
        if ((e = hipEventRecord(c->ev_verify_start, c->pack_stream)) != hipSuccess) { hip_fail("record", e); launched = false; }
        if (launched && (e = launch_verify_pairs(c->dev_pairs, c->plan.pair_tiles.size(), c->dev_flag, c->pack_stream)) != hipSuccess) { hip_fail("verify launch", e); launched = false; }
        if (launched && (e = hipMemcpyAsync(c->host_flag, c->dev_flag, sizeof(uint32_t), hipMemcpyDeviceToHost, c->pack_stream)) != hipSuccess) { hip_fail("verdict copy", e); launched = false; }
        if (launched && (e = hipEventRecord(c->ev_verify_done, c->pack_stream)) != hipSuccess) { hip_fail("record", e); launched = false; }
        if (launched && (e = hipEventSynchronize(c->ev_verify_done)) != hipSuccess) { hip_fail("verdict sync", e); launched = false; }
        if (launched && *c->host_flag == 0) { chosen = &c->rplan; chosen_tiles = c->dev_rtiles; }   // anything else: the full file
        float vms = 0;
        if (launched && hipEventElapsedTime(&vms, c->ev_verify_start, c->ev_verify_done) == hipSuccess) s->verify_ms = vms;
    }
    const Plan &p = *chosen;
    s->chunks_left = p.n_chunks;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        s->plan = chosen;
        s->dev_tiles = chosen_tiles;
    }

    // file and header
    const bool use_mmap = c->cfg.io_mode == CKPT_IO_MMAP;
    memcpy(c->hdr_buf, p.header.data(), p.header_bytes);
    for (int i = 0; i < 8; i++) c->hdr_buf[16 + i] = uint8_t(s->iter >> (8 * i));
    FileSlot reuse;
    std::vector<FileSlot> wrong_size;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        while (!c->spares.empty() && reuse.fd < 0) {
            FileSlot f = c->spares.back();
            c->spares.pop_back();
            if (f.bytes == p.file_bytes()) reuse = f; else wrong_size.push_back(f);
        }
    }
    // a spare of another size (the previous snapshot had the other format version) cannot be overwritten in place
    for (auto &f : wrong_size) { f.close_all(); unlink(f.path.c_str()); }
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
        c->fail_snapshot(s, CKPT_EIO, s->tmp_path + ": " + ferr);
        if (s->map) munmap(s->map, p.file_bytes());
        if (s->fd >= 0) { close(s->fd); unlink(s->tmp_path.c_str()); }
        s->map = nullptr; s->fd = -1;
    }

    if (p.n_direct)   // these copies read the tensors themselves
        for (size_t k = 0; k < nk; k++)
            if ((e = hipStreamWaitEvent(c->dma[k], s->ev_boundary, 0)) != hipSuccess) hip_fail("wait boundary", e);
    double bp_ms = 0;
    // Pack launches run ahead of the copies: as far as staging allows when the window closes with the last pack
    // (policy PACK: get the reads of the tensors over with), `ahead` = two staging slots otherwise (under the
    // paper's rule nothing is gained by packing earlier, and a burst of pack kernels would only compete with the
    // forward pass). Pack sc needs the staging slot that the copies of super-chunk sc - ahead read (ahead <= n_stage,
    // copies are in order): this thread waits for those copies on the host and launches the pack then.
    const uint64_t ahead = s->policy == CKPT_WINDOW_PACK ? c->n_stage : std::min<uint64_t>(c->n_stage, 2);
    auto enqueue_pack = [&](uint64_t sc) {
        const uint64_t stage = sc % c->n_stage;
        if (sc >= ahead)
            for (size_t k = 0; k < nk; k++) {
                // host first (this thread sleeps until the staging slot is free), so that the pack queue never holds a
                // launch parked behind an unsignalled event while the copies run: see the boundary wait above.
                hipEvent_t freed = c->ev_stage_done[(sc - ahead) % c->n_stage][k];
                if ((e = hipEventSynchronize(freed)) != hipSuccess) hip_fail("stage sync", e);
                if ((e = hipStreamWaitEvent(c->pack_stream, freed, 0)) != hipSuccess) hip_fail("wait stage", e);
            }
        const uint64_t t0 = p.sc_first_tile[sc], t1 = p.sc_first_tile[sc + 1];
        if ((e = launch_pack(s->dev_tiles + t0, t1 - t0, c->staging + stage * SC, sc * SC, c->pack_stream, c->ev_pack_start[sc], c->ev_pack_end[sc])) != hipSuccess)
            hip_fail("pack launch", e);
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
        // The next pack launch goes out one round late, after this super-chunk's copies have been enqueued: its host-side
        // wait is for the copies of the previous super-chunk, and the copy engines have this one's to go on with. The
        // pack of super-chunk sc + 1 was launched a round ago, before the copies above that wait for it.
        if (sc >= 1 && sc - 1 + ahead < p.n_superchunks) enqueue_pack(sc - 1 + ahead);
    }
    std::vector<uint8_t>().swap(s->host_capture);   // every byte of it is in a ring slot by now
    std::lock_guard<std::mutex> lk(c->mu);
    s->backpressure_ms = bp_ms + tier2_wait_ms;
    s->t_submitted = Clock::now();
    s->submitted = true;
    c->prev_job = sp;
    c->cv_state.notify_all();
}

void dsllm::submit_thread_main(ckpt_ctx *c) {
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

