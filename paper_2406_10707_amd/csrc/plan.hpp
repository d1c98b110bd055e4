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
    bool derived = false;       // format version 2: not stored, recomputed from tensor `source` (bf16 rounding of an f32 tensor)
    uint32_t source = 0;
};

// One work item of the derivation kernels: `count` elements of an f32 tensor and of its bf16 copy.
constexpr uint32_t kPairTileElems = 8192;
struct PairTile {
    uint64_t f32_addr;
    uint64_t bf16_addr;
    uint32_t count;
    uint32_t pad;
    uint64_t reserved;
};

// Declared derivations: tensor derived[i] (bf16) is the round-to-nearest-even of tensor source[i] (f32, same shape).
struct DerivedPairs {
    std::vector<uint32_t> derived, source;
    size_t size() const { return derived.size(); }
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
    uint32_t version = 1;                 // file format version this plan writes: 2 when tensors are derived
    uint64_t n_derived = 0, derived_bytes = 0;   // tensors described but not stored, and their payload
    std::vector<PairTile> pair_tiles;     // the declared pairs cut into work items (filled in both plans of a registration)

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
// pairs == nullptr: the version-1 plan, every tensor stored (pair_tiles stay empty). With pairs and omit_derived the
// version-2 plan: derived tensors get a table entry and nothing else. With pairs and !omit_derived the version-1
// plan of the same registration (used when a snapshot's pairs do not hold), pair_tiles filled for the check.
int build_plan(const ckpt_tensor_desc *tensors, size_t n, const ResolvedConfig &cfg, Plan *out, std::string *err,
               const DerivedPairs *pairs = nullptr, bool omit_derived = false);
// Re-checks every tile and copy segment against the plan's own tensors, chunks and super-chunks
// (defence before any launch or copy).
bool verify_plan(const Plan &p, std::string *err);

}  // namespace dsllm
