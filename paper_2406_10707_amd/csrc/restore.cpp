// Restore: the snapshot path run backwards (file -> ring slots -> device -> scatter kernel).
#include "engine_internal.hpp"

using namespace dsllm;

static int restore_body(ckpt_ctx *c, int fd, const char *path, hipStream_t stream, uint64_t base, uint64_t *issued_out, uint64_t *iter_out) {
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
    const uint64_t version = le(hb + 8, 4);
    if (memcmp(hb, c->plan.header.data(), 8) != 0 || (version != 1 && version != 2) || le(hb + 12, 4) != kAlign || le(hb + 56, 8) != 0)
        return fail(CKPT_EFORMAT, "bad magic, version or alignment");
    // a version-2 file (derived tensors left out) is read with the registration's version-2 plan, which exists
    // only if the same derivations were declared; its derived tensors are recomputed at the end
    if (version == 2 && !c->have_rplan) return fail(CKPT_EMISMATCH, "the file leaves derived tensors out, this registration declares none");
    const Plan &p = version == 2 ? c->rplan : c->plan;
    const ckpt_tile *dev_tiles = version == 2 ? c->dev_rtiles : c->dev_tiles;
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
            // A chunk is read in pieces by as many I/O threads as there are pieces: one thread per whole chunk would
            // leave a small shard (fewer chunks than threads, or one more) waiting for its slowest read.
            const uint64_t nbytes = p.chunk_bytes(issued);
            const uint64_t kReadPieceBytes = CH / kReadPiecesPerChunk;   // CH is a multiple of 32 KiB: pieces are 4 KiB multiples
            const uint64_t n_pieces = (nbytes + kReadPieceBytes - 1) / kReadPieceBytes;
            {
                std::lock_guard<std::mutex> lk(c->mu);
                c->slot_state[slot] = SLOT_BUSY;
                c->slot_reads_left[slot] = uint32_t(n_pieces);
                for (uint64_t q = 0; q < n_pieces; q++) {
                    IoJob job;
                    job.kind = IoJob::READ;
                    job.fd = fd;
                    job.slot = slot;
                    job.slot_off = q * kReadPieceBytes;
                    job.file_off = p.header_bytes + issued * CH + job.slot_off;
                    job.nbytes = std::min<uint64_t>(kReadPieceBytes, nbytes - job.slot_off);
                    c->io_q.push_back(job);
                }
            }
            c->cv_io.notify_all();
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
        HIP_TRY(c, launch_scatter(dev_tiles + t0, t1 - t0, stage_base, sc * SC, c->pack_stream));
        HIP_TRY(c, hipEventRecord(c->ev_packed[sc], c->pack_stream));
    }
    HIP_TRY(c, hipStreamWaitEvent(stream, c->ev_packed[p.n_superchunks - 1], 0));
    if (p.n_direct)   // the last copies into large tensors are not followed by a scatter kernel
        for (size_t k = 0; k < nk; k++) {
            HIP_TRY(c, hipEventRecord(c->ev_job_tail[k], c->dma[k]));
            HIP_TRY(c, hipStreamWaitEvent(stream, c->ev_job_tail[k], 0));
        }
    if (version == 2) {
        // every stored tensor is in place once the pack stream has run its last scatter kernel (and the copy streams
        // their direct copies): the derived tensors are then recomputed from their sources
        if (p.n_direct)
            for (size_t k = 0; k < nk; k++) HIP_TRY(c, hipStreamWaitEvent(c->pack_stream, c->ev_job_tail[k], 0));
        HIP_TRY(c, launch_derive_pairs(c->dev_pairs, c->plan.pair_tiles.size(), c->pack_stream));
        HIP_TRY(c, hipEventRecord(c->ev_derived, c->pack_stream));
        HIP_TRY(c, hipStreamWaitEvent(stream, c->ev_derived, 0));
    }
    if (iter_out) *iter_out = f_iter;
    return CKPT_OK;
}



// True if the file at `path` carries a consistent fixed header for iteration `iter` and has the size it states.
static bool whole_checkpoint(const std::string &path, uint64_t iter) {
    int fd = open(path.c_str(), O_RDONLY);
    if (fd < 0) return false;
    uint8_t h[kFixedHeader];
    struct stat st;
    std::string err;
    bool ok = fstat(fd, &st) == 0 && uint64_t(st.st_size) >= kAlign && pread_all(fd, h, sizeof h, 0, &err);
    close(fd);
    if (!ok) return false;
    auto le = [&](int off, int n) { uint64_t v = 0; for (int i = 0; i < n; i++) v |= uint64_t(h[off + i]) << (8 * i); return v; };
    static const uint8_t magic[8] = {'D', 'S', 'L', 'L', 'M', 'C', 'K', 1};
    if (memcmp(h, magic, 8) != 0 || (le(8, 4) != 1 && le(8, 4) != 2) || le(12, 4) != kAlign || le(56, 8) != 0) return false;
    const uint64_t hb = le(32, 8), db = le(40, 8), fb = le(48, 8);
    return le(16, 8) == iter && hb >= kAlign && hb % kAlign == 0 && db % kAlign == 0 && fb == hb + db && fb == uint64_t(st.st_size);
}

extern "C" {

int ckpt_describe_file(const char *path, char *buf, size_t cap, size_t *needed_out) {
    if (!path) return fail(CKPT_EINVAL, "null argument");
    int fd = open(path, O_RDONLY);
    if (fd < 0) return fail(CKPT_EIO, std::string(path) + ": open: " + strerror(errno));
    struct stat st;
    std::string err;
    uint8_t fixed[kFixedHeader];
    if (fstat(fd, &st) != 0 || uint64_t(st.st_size) < kAlign || !pread_all(fd, fixed, sizeof fixed, 0, &err)) {
        close(fd);
        return fail(CKPT_EFORMAT, std::string(path) + ": shorter than one header unit");
    }
    auto le = [](const uint8_t *q, int n) { uint64_t v = 0; for (int i = 0; i < n; i++) v |= uint64_t(q[i]) << (8 * i); return v; };
    static const uint8_t magic[8] = {'D', 'S', 'L', 'L', 'M', 'C', 'K', 1};
    const uint64_t iter = le(fixed + 16, 8), n = le(fixed + 24, 8), hb = le(fixed + 32, 8), db = le(fixed + 40, 8), fb = le(fixed + 48, 8);
    const uint64_t version = le(fixed + 8, 4);
    if (memcmp(fixed, magic, 8) != 0 || (version != 1 && version != 2) || le(fixed + 12, 4) != kAlign || le(fixed + 56, 8) != 0 || hb < kAlign ||
        hb % kAlign || db % kAlign || fb != hb + db || fb != uint64_t(st.st_size) || hb > (1ull << 32)) {
        close(fd);
        return fail(CKPT_EFORMAT, std::string(path) + ": not a whole checkpoint file");
    }
    std::vector<uint8_t> h(hb);
    const bool got = pread_all(fd, h.data(), hb, 0, &err);
    close(fd);
    if (!got) return fail(CKPT_EIO, std::string(path) + ": " + err);
    static const char *const dtype_name[] = {"?", "bf16", "f32", "f16", "u8", "i32", "i64"};
    std::string text = "iter " + std::to_string(iter) + " tensors " + std::to_string(n) + " header_bytes " + std::to_string(hb) +
                       " data_bytes " + std::to_string(db) + "\n";
    uint64_t pos = kFixedHeader;
    for (uint64_t k = 0; k < n; k++) {
        if (pos + 2 > hb) return fail(CKPT_EFORMAT, "tensor table runs past the header");
        const uint64_t len = le(&h[pos], 2);
        pos += 2;
        if (len == 0 || pos + len + 2 > hb) return fail(CKPT_EFORMAT, "tensor table runs past the header");
        text.append(reinterpret_cast<const char *>(&h[pos]), len);
        pos += len;
        const unsigned dtype = h[pos], ndim = h[pos + 1];
        pos += 2;
        if (dtype < 1 || dtype > 6 || ndim > 8 || pos + 8ull * ndim + 16 + (version == 2 ? 5 : 0) > hb) return fail(CKPT_EFORMAT, "bad tensor table entry");
        text += std::string("\t") + dtype_name[dtype] + "\t";
        if (ndim == 0) text += "-";
        for (unsigned i = 0; i < ndim; i++) { text += (i ? "x" : "") + std::to_string(le(&h[pos], 8)); pos += 8; }
        const uint64_t off = le(&h[pos], 8), nb = le(&h[pos + 8], 8);
        pos += 16;
        uint64_t enc = 0, ref = 0;
        if (version == 2) { enc = h[pos]; ref = le(&h[pos + 1], 4); pos += 5; }
        if (enc > 1 || (enc == 1 && (off != 0 || ref >= n))) return fail(CKPT_EFORMAT, "bad derived-tensor entry");
        if (enc == 0 && (off < hb || off % kAlign || off + nb > fb)) return fail(CKPT_EFORMAT, "tensor lies outside the data region");
        text += "\t" + std::to_string(off) + "\t" + std::to_string(nb) + (enc ? "\tbf16 rounding of tensor " + std::to_string(ref) : "") + "\n";
    }
    if (needed_out) *needed_out = text.size() + 1;
    if (!buf || cap < text.size() + 1) return fail(CKPT_EINVAL, "buffer smaller than the description");
    memcpy(buf, text.c_str(), text.size() + 1);
    return CKPT_OK;
}

int ckpt_find_latest(const char *dir, uint64_t *iter_out, char *path_buf, size_t cap) {
    if (!dir || !*dir) return fail(CKPT_EINVAL, "null argument");
    DIR *d = opendir(dir);
    if (!d) return fail(CKPT_EIO, std::string(dir) + ": opendir: " + strerror(errno));
    std::vector<uint64_t> iters;
    while (struct dirent *e = readdir(d)) {
        const char *n = e->d_name;   // "ckpt_iter" + 20 digits + ".dsl"
        if (strlen(n) != 9 + 20 + 4 || strncmp(n, "ckpt_iter", 9) != 0 || strcmp(n + 29, ".dsl") != 0) continue;
        uint64_t v = 0;
        bool digits = true;
        for (int i = 9; i < 29 && digits; i++) { digits = n[i] >= '0' && n[i] <= '9'; v = v * 10 + uint64_t(n[i] - '0'); }
        if (digits) iters.push_back(v);
    }
    closedir(d);
    std::sort(iters.begin(), iters.end());
    for (auto it = iters.rbegin(); it != iters.rend(); ++it) {
        const std::string path = file_name_for(dir, *it);
        if (!whole_checkpoint(path, *it)) continue;
        if (path_buf) {
            if (path.size() + 1 > cap) return fail(CKPT_EINVAL, "buffer too small");
            memcpy(path_buf, path.c_str(), path.size() + 1);
        }
        if (iter_out) *iter_out = *it;
        return CKPT_OK;
    }
    return fail(CKPT_EINVAL, std::string(dir) + ": no whole checkpoint file found");
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

}  // extern "C"
