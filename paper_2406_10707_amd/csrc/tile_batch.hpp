// A batch of tensor descriptors small enough to travel in a kernel's arguments (under 4 KiB): what
// build_tiles_kernel turns into entries of the pack kernel's tile table.
#pragma once
#include <cstdint>

namespace dsllm {

constexpr int kTileBatch = 96;

struct TileBatch {
    uint64_t src[kTileBatch];          // device address of the tensor's first byte
    uint64_t data_off[kTileBatch];     // offset of the tensor in the data region (a multiple of 4096)
    uint64_t nbytes[kTileBatch];
    uint32_t first_tile[kTileBatch + 1];   // index of the tensor's first tile in the table; [count] = one past the batch's last
    uint32_t count;
};
static_assert(sizeof(TileBatch) <= 3072, "must fit the kernel argument segment with room to spare");

// tiles the padded extent of a tensor at data-region offset d0 is cut into (cuts at its start and at every multiple of tile_bytes)
inline uint64_t tiles_of(uint64_t d0, uint64_t nbytes, uint64_t tile_bytes) {
    const uint64_t dend = d0 + (nbytes + 4095) / 4096 * 4096;
    return (dend + tile_bytes - 1) / tile_bytes - d0 / tile_bytes;
}

}  // namespace dsllm
