#include "plan.hpp"

#include <cstring>

namespace dsllm {

static inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

uint64_t dtype_size(int32_t dtype) {
    switch (dtype) {
        case CKPT_BF16: case CKPT_F16: return 2;
        case CKPT_F32: case CKPT_I32: return 4;
        case CKPT_U8: return 1;
        case CKPT_I64: return 8;
        default: return 0;
    }
}

int resolve_config(const ckpt_config *in, ResolvedConfig *out, std::string *err) {
    ResolvedConfig c;
    c.dma_chunk_bytes = in->dma_chunk_bytes ? in->dma_chunk_bytes : (256ull << 20);
    c.pack_superchunk_bytes = in->pack_superchunk_bytes ? in->pack_superchunk_bytes : (1ull << 30);
    c.host_ring_bytes = in->host_ring_bytes ? in->host_ring_bytes : (8ull << 30);
    c.dev_staging_bytes = in->dev_staging_bytes ? in->dev_staging_bytes : 2 * c.pack_superchunk_bytes;
    c.n_dma_streams = in->n_dma_streams ? in->n_dma_streams : 2;
    c.n_io_threads = in->n_io_threads ? in->n_io_threads : 4;
    c.window_policy = in->window_policy;
    c.o_direct = in->o_direct;
    c.fsync_on_commit = in->fsync_on_commit < 0 ? 0 : 1;   // durable unless the caller opts out
    c.io_mode = in->io_mode;
    c.keep_last = in->keep_last;
    c.prealloc_files = in->prealloc_files;
    c.direct_min_bytes = in->direct_min_bytes;
    if (c.direct_min_bytes != 0 && c.direct_min_bytes < kAlign) { *err = "config: direct_min_bytes must be 0 or at least 4096"; return CKPT_EINVAL; }
    if (c.direct_min_bytes != 0 && in->window_policy != CKPT_WINDOW_D2H) { *err = "config: direct_min_bytes needs window_policy CKPT_WINDOW_D2H"; return CKPT_EINVAL; }
    if (c.keep_last < 0 || c.prealloc_files < 0 || c.prealloc_files > 16) { *err = "config: keep_last must be >= 0 and prealloc_files 0..16"; return CKPT_EINVAL; }
    if (c.prealloc_files > 0 && c.keep_last == 0) { *err = "config: prealloc_files needs keep_last > 0"; return CKPT_EINVAL; }
    if (c.io_mode == CKPT_IO_AUTO) c.io_mode = c.o_direct ? CKPT_IO_PWRITE : CKPT_IO_MMAP;
    if (c.io_mode != CKPT_IO_PWRITE && c.io_mode != CKPT_IO_MMAP) { *err = "config: unknown io_mode"; return CKPT_EINVAL; }
    if (c.io_mode == CKPT_IO_MMAP && c.o_direct) { *err = "config: o_direct needs io_mode pwrite"; return CKPT_EINVAL; }
    for (int r : in->reserved) if (r != 0) { *err = "config: reserved fields must be zero"; return CKPT_EINVAL; }
    if (c.dma_chunk_bytes % kTileBytes != 0) { *err = "config: dma_chunk_bytes must be a multiple of the 32 KiB tile size"; return CKPT_EINVAL; }
    if (c.pack_superchunk_bytes % c.dma_chunk_bytes != 0) { *err = "config: pack_superchunk_bytes must be a multiple of dma_chunk_bytes"; return CKPT_EINVAL; }
    if (c.pack_superchunk_bytes > (64ull << 30)) { *err = "config: pack_superchunk_bytes above 64 GiB"; return CKPT_EINVAL; }
    if (c.n_dma_streams < 1 || c.n_dma_streams > 8) { *err = "config: n_dma_streams must be 1..8"; return CKPT_EINVAL; }
    if (c.n_io_threads < 1 || c.n_io_threads > 64) { *err = "config: n_io_threads must be 1..64"; return CKPT_EINVAL; }
    if (c.window_policy != CKPT_WINDOW_D2H && c.window_policy != CKPT_WINDOW_PACK) { *err = "config: unknown window_policy"; return CKPT_EINVAL; }
    c.host_ring_bytes = c.host_ring_bytes / c.dma_chunk_bytes * c.dma_chunk_bytes;
    if (c.host_ring_bytes < 2 * c.dma_chunk_bytes) c.host_ring_bytes = 2 * c.dma_chunk_bytes;
    c.dev_staging_bytes = c.dev_staging_bytes / c.pack_superchunk_bytes * c.pack_superchunk_bytes;
    if (c.dev_staging_bytes < 2 * c.pack_superchunk_bytes) c.dev_staging_bytes = 2 * c.pack_superchunk_bytes;
    *out = c;
    return CKPT_OK;
}

static void put_le(uint8_t *p, uint64_t v, int n) { for (int i = 0; i < n; i++) p[i] = uint8_t(v >> (8 * i)); }

int build_plan(const ckpt_tensor_desc *descs, size_t n, const ResolvedConfig &cfg, Plan *out, std::string *err, const DerivedPairs *pairs,
               bool omit_derived) {
    if (!descs || n == 0) { *err = "no tensors"; return CKPT_EINVAL; }
    Plan p;
    p.cfg = cfg;
    p.version = pairs && omit_derived ? 2 : 1;
    p.tensors.reserve(n);
    uint64_t table = 0;
    for (size_t k = 0; k < n; k++) {
        const ckpt_tensor_desc &d = descs[k];
        const bool host = (d.dtype & CKPT_PLACE_HOST) != 0;
        const int32_t dtype = d.dtype & ~CKPT_PLACE_HOST;
        uint64_t es = dtype_size(dtype);
        size_t len = d.name ? strlen(d.name) : 0;
        if (len < 1 || len > 65535) { *err = "tensor " + std::to_string(k) + ": name must be 1..65535 bytes"; return CKPT_EINVAL; }
        if (es == 0) { *err = std::string("tensor ") + d.name + ": unknown dtype"; return CKPT_EINVAL; }
        if (d.ndim > 8 || (d.ndim > 0 && !d.shape)) { *err = std::string("tensor ") + d.name + ": bad ndim/shape"; return CKPT_EINVAL; }
        uint64_t numel = 1;
        TensorInfo t;
        for (uint32_t i = 0; i < d.ndim; i++) {
            if (d.shape[i] < 0) { *err = std::string("tensor ") + d.name + ": negative dimension"; return CKPT_EINVAL; }
            numel *= uint64_t(d.shape[i]);
            t.shape.push_back(d.shape[i]);
        }
        if (d.nbytes == 0 || d.nbytes != numel * es) { *err = std::string("tensor ") + d.name + ": nbytes must be > 0 and equal dtype size x shape"; return CKPT_EINVAL; }
        if (!host && uint64_t(d.dev_ptr) % es != 0) { *err = std::string("tensor ") + d.name + ": address not aligned to its element size"; return CKPT_EINVAL; }
        t.name.assign(d.name, len);
        t.dtype = dtype;
        t.host = host;
        t.dev_addr = uint64_t(d.dev_ptr);
        t.nbytes = d.nbytes;
        t.file_off = 0;
        t.direct = !host && cfg.direct_min_bytes != 0 && d.nbytes >= cfg.direct_min_bytes;
        if (host) { t.capture_off = p.host_bytes; p.n_host++; p.host_bytes += d.nbytes; p.host_data_bytes += align_up(d.nbytes, kAlign); }
        if (t.direct) { p.n_direct++; p.direct_bytes += d.nbytes; p.direct_data_bytes += align_up(d.nbytes, kAlign); }
        table += 2 + len + 2 + 8ull * d.ndim + 16;
        p.payload_bytes += d.nbytes;
        p.tensors.push_back(std::move(t));
    }
    if (pairs) {
        // a derived tensor is a bf16 tensor on the device, its source a stored f32 tensor of the same shape on the device
        std::vector<uint8_t> is_derived(n, 0), is_source(n, 0);
        for (size_t i = 0; i < pairs->size(); i++) {
            const uint64_t d = pairs->derived[i], s = pairs->source[i];
            if (d >= n || s >= n || d == s) { *err = "derived pair " + std::to_string(i) + ": index out of range"; return CKPT_EINVAL; }
            const TensorInfo &td = p.tensors[d], &ts = p.tensors[s];
            if (td.dtype != CKPT_BF16 || ts.dtype != CKPT_F32 || td.shape != ts.shape) { *err = "derived pair " + std::to_string(i) + ": needs a bf16 tensor and an f32 source of the same shape"; return CKPT_EINVAL; }
            if (td.host || ts.host) { *err = "derived pair " + std::to_string(i) + ": host-resident objects cannot take part"; return CKPT_EINVAL; }
            if (is_derived[d] || is_derived[s] || is_source[d]) { *err = "derived pair " + std::to_string(i) + ": a tensor is derived twice, or a source is itself derived"; return CKPT_EINVAL; }
            is_derived[d] = 1; is_source[s] = 1;
            const uint64_t numel = ts.nbytes / 4;
            for (uint64_t e = 0; e < numel; e += kPairTileElems) {
                PairTile pt;
                pt.f32_addr = ts.dev_addr + 4 * e;
                pt.bf16_addr = td.dev_addr + 2 * e;
                pt.count = uint32_t(numel - e < kPairTileElems ? numel - e : kPairTileElems);
                pt.pad = 0; pt.reserved = 0;
                p.pair_tiles.push_back(pt);
            }
            if (omit_derived) {
                TensorInfo &t = p.tensors[d];
                t.derived = true; t.source = uint32_t(s);
                if (t.direct) { t.direct = false; p.n_direct--; p.direct_bytes -= t.nbytes; p.direct_data_bytes -= align_up(t.nbytes, kAlign); }
                p.n_derived++; p.derived_bytes += t.nbytes;
            }
        }
    }
    if (p.version == 2) table += 5ull * n;     // enc u8 + ref u32 at the end of every entry
    p.header_bytes = align_up(kFixedHeader + table, kAlign);
    uint64_t off = p.header_bytes;
    for (auto &t : p.tensors) {
        if (t.derived) { t.file_off = 0; continue; }
        t.file_off = off; off += align_up(t.nbytes, kAlign);
    }
    p.data_bytes = off - p.header_bytes;

    // header image (iter left zero; patched per snapshot at byte 16)
    p.header.assign(p.header_bytes, 0);
    uint8_t *h = p.header.data();
    static const uint8_t magic[8] = {'D', 'S', 'L', 'L', 'M', 'C', 'K', 1};
    memcpy(h, magic, 8);
    put_le(h + 8, p.version, 4);
    put_le(h + 12, kAlign, 4);
    put_le(h + 24, n, 8);
    put_le(h + 32, p.header_bytes, 8);
    put_le(h + 40, p.data_bytes, 8);
    put_le(h + 48, p.file_bytes(), 8);
    uint8_t *w = h + kFixedHeader;
    for (const auto &t : p.tensors) {
        put_le(w, t.name.size(), 2); w += 2;
        memcpy(w, t.name.data(), t.name.size()); w += t.name.size();
        *w++ = uint8_t(t.dtype);
        *w++ = uint8_t(t.shape.size());
        for (int64_t s : t.shape) { put_le(w, uint64_t(s), 8); w += 8; }
        put_le(w, t.file_off, 8); w += 8;
        put_le(w, t.nbytes, 8); w += 8;
        if (p.version == 2) { *w++ = t.derived ? 1 : 0; put_le(w, t.derived ? t.source : 0, 4); w += 4; }
    }

    // chunks and super-chunks partition the data region at fixed strides
    const uint64_t SC = cfg.pack_superchunk_bytes, CH = cfg.dma_chunk_bytes;
    p.n_chunks = (p.data_bytes + CH - 1) / CH;
    p.n_superchunks = (p.data_bytes + SC - 1) / SC;

    // tiles: each tensor's padded extent is cut at its start and at every global multiple of the tile size,
    // so no tile crosses a tensor, chunk or super-chunk boundary (those are all multiples of the tile size)
    p.sc_first_tile.assign(p.n_superchunks + 1, 0);
    uint64_t next_sc = 0;
    for (const auto &t : p.tensors) {
        if (t.derived) continue;                               // described, not stored: no place in the data region
        uint64_t d0 = t.file_off - p.header_bytes;             // data-region offset of the tensor
        uint64_t dend = d0 + align_up(t.nbytes, kAlign);
        uint64_t pos = t.direct || t.host ? dend : d0;         // direct tensors and host objects have no tiles
        while (pos < dend) {
            uint64_t stop = (pos / kTileBytes + 1) * kTileBytes;
            if (stop > dend) stop = dend;
            while (next_sc < p.n_superchunks && pos >= next_sc * SC) p.sc_first_tile[next_sc++] = p.tiles.size();
            ckpt_tile tile;
            uint64_t rel = pos - d0;
            uint64_t copy = rel >= t.nbytes ? 0 : (t.nbytes - rel < stop - pos ? t.nbytes - rel : stop - pos);
            tile.src = t.dev_addr + rel;
            tile.dst_off = pos;
            tile.copy_bytes = uint32_t(copy);
            tile.total_bytes = uint32_t(stop - pos);
            tile.reserved = 0;
            p.tiles.push_back(tile);
            pos = stop;
        }
    }
    while (next_sc <= p.n_superchunks) p.sc_first_tile[next_sc++] = p.tiles.size();

    // copy segments: what the DMA engines move for each chunk. Packed extents (payload and padding)
    // come from staging and merge into one segment per run; a direct tensor's payload comes from the
    // tensor itself and its padding is zero-filled on the host. Everything is cut at chunk boundaries.
    p.chunk_first_seg.assign(p.n_chunks + 1, 0);
    uint64_t next_ch = 0;
    auto emit = [&](uint64_t a, uint64_t b, uint32_t kind, uint64_t src, uint32_t tensor) {
        while (a < b) {
            uint64_t stop = (a / CH + 1) * CH;
            if (stop > b) stop = b;
            while (next_ch < p.n_chunks && a >= next_ch * CH) p.chunk_first_seg[next_ch++] = p.segs.size();
            const bool chunk_start = a % CH == 0;
            if (kind == CKPT_SEG_STAGED && !chunk_start && !p.segs.empty() && p.segs.back().kind == CKPT_SEG_STAGED &&
                p.segs.back().data_off + p.segs.back().nbytes == a) {
                p.segs.back().nbytes += stop - a;
            } else {
                ckpt_segment sg;
                sg.data_off = a;
                sg.nbytes = stop - a;
                sg.src = kind == CKPT_SEG_DIRECT || kind == CKPT_SEG_HOST ? src : 0;
                sg.kind = kind;
                sg.tensor = kind == CKPT_SEG_STAGED ? 0 : tensor;
                p.segs.push_back(sg);
            }
            if (kind == CKPT_SEG_DIRECT || kind == CKPT_SEG_HOST) src += stop - a;
            a = stop;
        }
    };
    for (size_t k = 0; k < p.tensors.size(); k++) {
        const TensorInfo &t = p.tensors[k];
        if (t.derived) continue;
        const uint64_t d0 = t.file_off - p.header_bytes, dend = d0 + align_up(t.nbytes, kAlign);
        if (t.direct || t.host) {
            emit(d0, d0 + t.nbytes, t.host ? CKPT_SEG_HOST : CKPT_SEG_DIRECT, t.dev_addr, uint32_t(k));
            emit(d0 + t.nbytes, dend, CKPT_SEG_ZERO, 0, uint32_t(k));
        } else {
            emit(d0, dend, CKPT_SEG_STAGED, 0, 0);
        }
    }
    while (next_ch <= p.n_chunks) p.chunk_first_seg[next_ch++] = p.segs.size();
    if (!verify_plan(p, err)) return CKPT_EINVAL;
    *out = std::move(p);
    return CKPT_OK;
}

bool verify_plan(const Plan &p, std::string *err) {
    const uint64_t SC = p.cfg.pack_superchunk_bytes, CH = p.cfg.dma_chunk_bytes;
    if (p.sc_first_tile.size() != p.n_superchunks + 1 || p.sc_first_tile.back() != p.tiles.size()) { *err = "plan: super-chunk tile index broken"; return false; }
    if (p.chunk_first_seg.size() != p.n_chunks + 1 || p.chunk_first_seg.back() != p.segs.size()) { *err = "plan: chunk segment index broken"; return false; }
    // tiles: the padded extent of every packed tensor is covered exactly, in order; none elsewhere
    size_t i = 0;
    for (size_t k = 0; k < p.tensors.size(); k++) {
        const TensorInfo &ti = p.tensors[k];
        if (ti.direct || ti.host || ti.derived) continue;
        const uint64_t d0 = ti.file_off - p.header_bytes, dend = d0 + align_up(ti.nbytes, kAlign);
        uint64_t expect = d0;
        while (expect < dend) {
            if (i >= p.tiles.size()) { *err = "plan: tiles end before the last packed tensor"; return false; }
            const ckpt_tile &t = p.tiles[i];
            if (t.dst_off != expect || t.total_bytes == 0 || t.total_bytes % 16 || t.dst_off % 16 || t.copy_bytes > t.total_bytes ||
                t.total_bytes > kTileBytes) { *err = "plan: tile " + std::to_string(i) + " malformed"; return false; }
            if (t.dst_off / SC != (t.dst_off + t.total_bytes - 1) / SC) { *err = "plan: tile crosses a super-chunk"; return false; }
            const uint64_t rel = t.dst_off - d0;
            if (t.copy_bytes && (t.src != ti.dev_addr + rel || rel + t.copy_bytes > ti.nbytes)) { *err = "plan: tile source outside its tensor"; return false; }
            if (!t.copy_bytes && rel < ti.nbytes) { *err = "plan: tile drops payload"; return false; }
            if (t.copy_bytes && t.copy_bytes < t.total_bytes && rel + t.copy_bytes != ti.nbytes) { *err = "plan: tile pads inside the payload"; return false; }
            if (t.dst_off + t.total_bytes > dend) { *err = "plan: tile crosses a tensor boundary"; return false; }
            const uint64_t s = t.dst_off / SC;
            if (i < p.sc_first_tile[s] || i >= p.sc_first_tile[s + 1]) { *err = "plan: tile not in its super-chunk's range"; return false; }
            expect += t.total_bytes;
            i++;
        }
    }
    if (i != p.tiles.size()) { *err = "plan: tiles beyond the packed tensors"; return false; }
    // segments: partition of the data region; per tensor the kinds and sources must fit
    uint64_t pos = 0;
    size_t k = 0;
    for (size_t j = 0; j < p.segs.size(); j++) {
        const ckpt_segment &sg = p.segs[j];
        if (sg.data_off != pos || sg.nbytes == 0) { *err = "plan: segment " + std::to_string(j) + " out of order or empty"; return false; }
        if (sg.data_off / CH != (sg.data_off + sg.nbytes - 1) / CH) { *err = "plan: segment crosses a chunk"; return false; }
        const uint64_t ch = sg.data_off / CH;
        if (j < p.chunk_first_seg[ch] || j >= p.chunk_first_seg[ch + 1]) { *err = "plan: segment not in its chunk's range"; return false; }
        // every tensor the segment touches
        uint64_t a = sg.data_off;
        const uint64_t b = sg.data_off + sg.nbytes;
        while (a < b) {
            while (k < p.tensors.size() && (p.tensors[k].derived || a >= p.tensors[k].file_off - p.header_bytes + align_up(p.tensors[k].nbytes, kAlign))) k++;
            if (k >= p.tensors.size()) { *err = "plan: segment beyond last tensor"; return false; }
            const TensorInfo &ti = p.tensors[k];
            const uint64_t d0 = ti.file_off - p.header_bytes, dend = d0 + align_up(ti.nbytes, kAlign);
            const uint64_t stop = b < dend ? b : dend;
            if (!ti.direct && !ti.host) {
                if (sg.kind != CKPT_SEG_STAGED) { *err = "plan: packed tensor under a non-staged segment"; return false; }
            } else if (sg.kind == (ti.host ? CKPT_SEG_HOST : CKPT_SEG_DIRECT)) {
                if (sg.tensor != k || b > d0 + ti.nbytes || sg.src != ti.dev_addr + (sg.data_off - d0)) { *err = "plan: direct segment outside its tensor"; return false; }
            } else if (sg.kind == CKPT_SEG_ZERO) {
                if (sg.tensor != k || sg.data_off < d0 + ti.nbytes || b > dend) { *err = "plan: zero segment outside its tensor's padding"; return false; }
            } else { *err = "plan: direct tensor under a staged segment"; return false; }
            a = stop;
        }
        pos = b;
    }
    if (pos != p.data_bytes) { *err = "plan: segments do not cover the data region"; return false; }
    return true;
}

}  // namespace dsllm
