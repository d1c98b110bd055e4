// Host-side plan of a registration: file offsets, header bytes, pack tiles, DMA chunks.
// Built once per tensor list (the paper's save phases one and two, hoisted out of the per-iteration path).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/ckpt.h"

namespace dsllm {

constexpr uint64_t kAlign = 4096;        // alignment unit of the file format
constexpr uint64_t kFixedHeader = 64;
constexpr uint64_t kTileBytes = 32 * 1024;  // destination bytes one wavefront produces (measured best: 32 KiB, 16 loads in flight per lane)

struct TensorInfo {
    std::string name;
    int32_t dtype;
    std::vector<int64_t> shape;
    uint64_t dev_addr;
    uint64_t nbytes;
    uint64_t file_off;
    bool direct = false;   // copied by the DMA engines from its own memory, not packed
    bool host = false;     // lives in host memory: captured by the CPU at the request, not packed
    uint64_t capture_off = 0;   // host objects: offset in a snapshot's capture buffer
};

struct ResolvedConfig {
    uint64_t host_ring_bytes, dma_chunk_bytes, pack_superchunk_bytes, dev_staging_bytes, direct_min_bytes;
    int n_dma_streams, n_io_threads, window_policy, o_direct, fsync_on_commit, io_mode, keep_last, prealloc_files;
};

struct Plan {
    ResolvedConfig cfg;
    std::vector<TensorInfo> tensors;
    std::vector<uint8_t> header;          // header_bytes long, iter field zero
    uint64_t header_bytes = 0, data_bytes = 0, payload_bytes = 0;
    std::vector<ckpt_tile> tiles;         // ordered by dst_off; none inside a direct tensor
    std::vector<uint64_t> sc_first_tile;  // n_superchunks + 1
    std::vector<ckpt_segment> segs;       // ordered by data_off, partition of the data region
    std::vector<uint64_t> chunk_first_seg;  // n_chunks + 1
    uint64_t n_chunks = 0, n_superchunks = 0, n_direct = 0, direct_bytes = 0, direct_data_bytes = 0;
    uint64_t n_host = 0, host_bytes = 0, host_data_bytes = 0;

    uint64_t file_bytes() const { return header_bytes + data_bytes; }
    uint64_t chunk_bytes(uint64_t c) const {      // last chunk may be short (still a 4 KiB multiple)
        uint64_t b = c * cfg.dma_chunk_bytes;
        return data_bytes - b < cfg.dma_chunk_bytes ? data_bytes - b : cfg.dma_chunk_bytes;
    }
    uint64_t superchunk_bytes(uint64_t s) const {
        uint64_t b = s * cfg.pack_superchunk_bytes;
        return data_bytes - b < cfg.pack_superchunk_bytes ? data_bytes - b : cfg.pack_superchunk_bytes;
    }
};

uint64_t dtype_size(int32_t dtype);
// Fills `cfg` defaults and checks it; returns CKPT_OK or CKPT_EINVAL with `err` set.
int resolve_config(const ckpt_config *in, ResolvedConfig *out, std::string *err);
int build_plan(const ckpt_tensor_desc *tensors, size_t n, const ResolvedConfig &cfg, Plan *out, std::string *err);
// Re-checks every tile and copy segment against the plan's own tensors, chunks and super-chunks
// (defence before any launch or copy).
bool verify_plan(const Plan &p, std::string *err);

}  // namespace dsllm
