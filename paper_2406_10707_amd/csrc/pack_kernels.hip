// Pack and scatter kernels for gfx950: pure byte movement between scattered tensors and the
// contiguous, 4 KiB-aligned staging image of the checkpoint's data region. HBM-bound.
//
// One wavefront (64 lanes) walks one tile of the descriptor table: up to 32 KiB of destination,
// 16 bytes per lane per step, 1 KiB per wavefront step. The staging side is always 16-byte aligned. The
// tensor side is aligned to its element size only. The pack kernel reads it with 16-byte vector loads at the
// tensor's own addresses (the target supports unaligned vector loads), each of which lies wholly inside the
// tensor; the one word that holds the tensor's last bytes, and everything the scatter kernel writes next to
// a tensor's edges, is built from aligned 16-byte words and byte shifts (v_alignbyte) or written byte by
// byte, so nothing outside a tensor is ever read past its 16-byte line or written at all.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/ckpt.h"
#include "kernel_util.hpp"
#include "tile_batch.hpp"

namespace dsllm {

// tuning constants (overridable at compile time for sweeps)
#ifndef DSLLM_PACK_WAVES_PER_BLOCK
#define DSLLM_PACK_WAVES_PER_BLOCK 4
#endif
#ifndef DSLLM_PACK_UNROLL
#define DSLLM_PACK_UNROLL 8
#endif
// Wave priority of the pack waves (s_setprio, 0..3). The kernel runs beside the training
// step's GEMM waves on the same compute units; with the highest issue priority a pack launch takes
// 4.5 % less time under a running GEMM loop (measured: 5.44 -> 5.68 TB/s per launch) and the step as a
// whole loses less, because the short burst of memory traffic is over sooner.
#ifndef DSLLM_PACK_PRIO
#define DSLLM_PACK_PRIO 3
#endif
// Ten loads in flight need 54 vector registers, which are handed out as 56 (eight need 46, eleven 58 = 64).
#ifndef DSLLM_PACK_ROLL
#define DSLLM_PACK_ROLL 10
#endif
#ifndef DSLLM_PACK_UNROLL_SHIFT
#define DSLLM_PACK_UNROLL_SHIFT 4
#endif
constexpr uint64_t kPackTileBytes = 32 * 1024;   // the planner's tile size (plan.hpp: kTileBytes)
constexpr int kWavesPerBlock = DSLLM_PACK_WAVES_PER_BLOCK;
constexpr int kBlock = 64 * kWavesPerBlock;
constexpr int kUnroll = DSLLM_PACK_UNROLL;             // scatter, aligned path: 16-byte words per lane in flight
constexpr int kRoll = DSLLM_PACK_ROLL;                 // pack: 16-byte words per lane in flight
constexpr int kUnrollShift = DSLLM_PACK_UNROLL_SHIFT;  // scatter, misaligned path: pairs of 16-byte words per lane in flight

// bytes [sh, sh+16) of the 32-byte string lo||hi, for sh = 4*W + b, 1 <= sh <= 15
template <int W>
__device__ __forceinline__ u32x4 funnel(u32x4 lo, u32x4 hi, uint32_t b) {
    uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    u32x4 o;
    o.x = __builtin_amdgcn_alignbyte(w[W + 1], w[W + 0], b);
    o.y = __builtin_amdgcn_alignbyte(w[W + 2], w[W + 1], b);
    o.z = __builtin_amdgcn_alignbyte(w[W + 3], w[W + 2], b);
    o.w = __builtin_amdgcn_alignbyte(w[W + 4], w[W + 3], b);
    return o;
}

// keep the first `keep` bytes (0..16) of v, zero the rest
__device__ __forceinline__ u32x4 keep_bytes(u32x4 v, uint32_t keep) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; j++) {
        uint32_t lo = 4u * j;
        if (keep <= lo) w[j] = 0;
        else if (keep < lo + 4) w[j] &= (1u << (8 * (keep - lo))) - 1u;
    }
    return u32x4{w[0], w[1], w[2], w[3]};
}

// ---------------------------------------------------------------- pack: tensors -> staging

// Output word j (16 bytes, aligned) = the 16 bytes at su + 16 j: one group of 64 U words starting at word g, every
// load of the group issued before its first store. su may have any alignment: the target supports unaligned vector
// loads (a 16-byte load at a 2-byte-aligned address is a single global_load_dwordx4), and all 16 bytes of every
// word lie inside the tensor, so nothing outside it is read.
template <int U>
__device__ __forceinline__ void copy_group(const uint8_t *su, u32x4 *dst, uint32_t g, uint32_t lane) {
    // one 64-bit base per side and constant offsets: a 32-bit word index per load would cost an address register pair each
    const uint8_t *sl = su + 16ull * (g + lane);
    u32x4 *dl = dst + (g + lane);
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; u++) v[u] = ld16_unaligned(sl + 1024 * u);
#pragma unroll
    for (int u = 0; u < U; u++) st16(dl + 64 * u, v[u]);
}

// Output words [0, n) of a tile from the n words at su (same contract as copy_group). A full tile (2048 words, 32
// per lane) runs as a rolling pipeline: kRoll loads are issued, then every store is followed at once by the load
// that reuses its registers, so kRoll loads stay in flight from the first word of the tile to the last instead
// of draining after every group. The fences keep the compiler from hoisting all loads to the front, which costs
// a hundred registers more. Shorter tiles (the last tile of a tensor, small tensors) go group by group.
//
// Measured on MI355X against a shape that keeps the whole tile (32 loads per lane, 138 registers) in flight:
// alone on the card the two are within 1 % of each other and of a plain table-free copy kernel (0.75 of the HBM
// peak on aligned tensors, 0.71 on the fragmented workload); beside a matrix kernel that leaves 64 registers per
// lane free only this one finds room on the SIMDs (0.71 to 0.74 against 0.45 to 0.55).
__device__ __forceinline__ void copy_rolling(const uint8_t *su, u32x4 *dst, uint32_t n, uint32_t lane) {
    uint32_t g = 0;
#pragma unroll 1
    for (; g + 2048 <= n; g += 2048) {
        const uint8_t *sl = su + 16ull * (g + lane);
        u32x4 *dl = dst + g + lane;
        u32x4 v[kRoll];
#pragma unroll
        for (int u = 0; u < kRoll; u++) v[u] = ld16_unaligned(sl + 1024 * u);
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
        for (int k = 0; k < 32; k++) {
            st16(dl + 64 * k, v[k % kRoll]);
            if (k + kRoll < 32) v[k % kRoll] = ld16_unaligned(sl + 1024 * (k + kRoll));
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);
#endif
        }
    }
#pragma unroll 1
    for (; g + 64 * 8 <= n; g += 64 * 8) copy_group<8>(su, dst, g, lane);
    if (g + 64 * 4 <= n) { copy_group<4>(su, dst, g, lane); g += 64 * 4; }
    if (g + 64 * 2 <= n) { copy_group<2>(su, dst, g, lane); g += 64 * 2; }
    if (g + 64 <= n) { copy_group<1>(su, dst, g, lane); g += 64; }
    const uint32_t i = g + lane;
    if (i < n) st16(dst + i, ld16_unaligned(su + 16ull * i));
}

// Output words [lo, hi) of one tile (16-byte words of its destination): source bytes where the tile has them,
// the masked tail word, zero padding behind it. All lanes of the wave in step; the tile's fields are wave-uniform.
__device__ __forceinline__ void pack_range(uint64_t src, u32x4 *dst, uint32_t copy_bytes, uint32_t total_bytes, uint32_t lo, uint32_t hi,
                                           uint32_t lane) {
    const uint32_t n_total = total_bytes >> 4;   // 16-byte words to write
    const uint32_t n_full = copy_bytes >> 4;     // of which fully covered by source bytes
    const uint32_t tail = copy_bytes & 15;       // source bytes in word n_full
    const uint32_t sh = uint32_t(src) & 15;
    if (hi > n_total) hi = n_total;
    if (lo >= hi) return;
    const uint32_t c_hi = hi < n_full ? hi : n_full;            // copy words [lo, c_hi)
    const uint32_t n = c_hi > lo ? c_hi - lo : 0;
    const bool own_tail = tail && lo <= n_full && n_full < hi;  // the range that holds word n_full writes the tail
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src - sh); // the aligned words that cover the tile's source bytes
    const uint32_t b = sh & 3;

    // the n words that lie wholly inside the tensor, read at the tensor's own (possibly misaligned) addresses
    copy_rolling(reinterpret_cast<const uint8_t *>(src) + 16ull * lo, dst + lo, n, lane);
    if (own_tail && lane == 0) {
        // The tail word never comes from an unaligned load (that would read up to 15 bytes past the tensor, possibly
        // into an unmapped page): aligned word n_full holds source bytes, word n_full + 1 only if sh + tail > 16.
        u32x4 v = ld16(s + n_full);
        if (sh != 0) {
            const u32x4 w1 = (sh + tail > 16) ? ld16(s + n_full + 1) : u32x4{0, 0, 0, 0};
            switch (sh >> 2) {
                case 0: v = funnel<0>(v, w1, b); break;
                case 1: v = funnel<1>(v, w1, b); break;
                case 2: v = funnel<2>(v, w1, b); break;
                default: v = funnel<3>(v, w1, b); break;
            }
        }
        st16(dst + n_full, keep_bytes(v, tail));
    }
    // zero padding after the tensor's last byte
    const uint32_t z0 = n_full + (tail ? 1u : 0u);
    for (uint32_t i = (z0 > lo ? z0 : lo) + lane; i < hi; i += 64) st16(dst + i, u32x4{0, 0, 0, 0});
}

__global__ __launch_bounds__(kBlock) void pack_kernel(const ckpt_tile *__restrict__ tiles, uint64_t n_tiles,
                                                     uint8_t *__restrict__ slot_base, uint64_t slot_data_off) {
    const uint32_t lane = threadIdx.x & 63;
#if defined(__HIP_DEVICE_COMPILE__) && DSLLM_PACK_PRIO > 0
    __builtin_amdgcn_s_setprio(DSLLM_PACK_PRIO);
#endif
    // The wavefront's number within the block is made uniform first: the descriptor address is then a
    // scalar value and the descriptor arrives through scalar loads (read-only path, no vector-memory
    // round trip before the first data load); measured, this closes the gap to a table-free copy.
    const uint64_t t = uint64_t(blockIdx.x) * kWavesPerBlock + uniform_u32(threadIdx.x >> 6);
    if (t >= n_tiles) return;
    const ckpt_tile *tp = tiles + t;
    const uint64_t src = uniform_u64(tp->src);
    const uint64_t dst_off = uniform_u64(tp->dst_off);
    u32x4 *dst = reinterpret_cast<u32x4 *>(slot_base + (dst_off - slot_data_off));
    pack_range(src, dst, uniform_u32(tp->copy_bytes), uniform_u32(tp->total_bytes), 0, uint32_t(kPackTileBytes / 16), lane);
}

// ---------------------------------------------------------------- scatter: staging -> tensors

// Writes destination-aligned 16-byte words [first, first+count) of a tensor range whose start is
// misaligned by `sh` bytes relative to the (aligned) staging source: word j takes staging bytes
// [16*j - sh, 16*j - sh + 16).
template <int W>
__device__ __forceinline__ void scatter_shifted(const u32x4 *src, u32x4 *dst_al, uint32_t n_words, uint32_t b, uint32_t lane) {
    // dst_al[j] for j = 1..n_words gets bytes [(16-sh) + 16*(j-1), +16) of src = funnel of src[j-1], src[j] at shift 16-sh
    uint32_t i = lane;
    for (; i + 64 * (kUnrollShift - 1) < n_words; i += 64 * kUnrollShift) {
        u32x4 lo[kUnrollShift], hi[kUnrollShift];
#pragma unroll
        for (int u = 0; u < kUnrollShift; u++) { lo[u] = ld16(src + i + 64 * u); hi[u] = ld16(src + i + 64 * u + 1); }
#pragma unroll
        for (int u = 0; u < kUnrollShift; u++) { DSLLM_KEEP_WHOLE(lo[u]); DSLLM_KEEP_WHOLE(hi[u]); }
#pragma unroll
        for (int u = 0; u < kUnrollShift; u++) st16(dst_al + 1 + i + 64 * u, funnel<W>(lo[u], hi[u], b));
    }
    for (; i < n_words; i += 64) st16(dst_al + 1 + i, funnel<W>(ld16(src + i), ld16(src + i + 1), b));
}

__global__ __launch_bounds__(kBlock) void scatter_kernel(const ckpt_tile *__restrict__ tiles, uint64_t n_tiles,
                                                        const uint8_t *__restrict__ slot_base, uint64_t slot_data_off) {
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t t = uint64_t(blockIdx.x) * kWavesPerBlock + uniform_u32(threadIdx.x >> 6);   // uniform: scalar descriptor loads
    if (t >= n_tiles) return;
    const ckpt_tile *tp = tiles + t;
    const uint64_t dstp = uniform_u64(tp->src);
    const uint64_t off = uniform_u64(tp->dst_off);
    const uint32_t nbytes = uniform_u32(tp->copy_bytes);
    if (nbytes == 0) return;
    const uint8_t *src = slot_base + (off - slot_data_off);   // 16-byte aligned
    uint8_t *dst = reinterpret_cast<uint8_t *>(dstp);
    const uint32_t mis = uint32_t(dstp) & 15;

    if (mis == 0) {
        const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
        u32x4 *d = reinterpret_cast<u32x4 *>(dst);
        const uint32_t n_full = nbytes >> 4;
        uint32_t i = lane;
        for (; i + 64 * (kUnroll - 1) < n_full; i += 64 * kUnroll) {
            u32x4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; u++) v[u] = ld16(s + i + 64 * u);
#pragma unroll
            for (int u = 0; u < kUnroll; u++) st16(d + i + 64 * u, v[u]);
        }
        for (; i < n_full; i += 64) st16(d + i, ld16(s + i));
        const uint32_t tail = nbytes & 15;       // bytes past the last full word: byte stores only
        if (lane < tail) dst[(n_full << 4) + lane] = src[(n_full << 4) + lane];
        return;
    }
    // head: bytes up to the first 16-byte boundary of the destination (byte stores; the neighbouring
    // bytes of that word belong to another tensor and may be written concurrently)
    const uint32_t head = (16 - mis) < nbytes ? (16 - mis) : nbytes;
    if (lane < head) dst[lane] = src[lane];
    const uint32_t rest = nbytes - head;
    const uint32_t n_words = rest >> 4;            // aligned destination words fully inside the range
    if (n_words) {
        // destination word j (1-based from the aligned address below dst) = staging bytes [head + 16*(j-1), +16)
        // = bytes [sh, sh+16) of staging words (j-1, j) with sh = head (1..15)
        const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
        u32x4 *d_al = reinterpret_cast<u32x4 *>(dst - mis);
        const uint32_t b = head & 3;
        // staging word index n_words is read as the upper half for the last destination word; it
        // exists inside the tile because head + 16*n_words <= nbytes <= total_bytes and the upper half
        // is needed only when head > 0, i.e. 16*n_words < nbytes.
        switch (head >> 2) {
            case 0: scatter_shifted<0>(s, d_al, n_words, b, lane); break;
            case 1: scatter_shifted<1>(s, d_al, n_words, b, lane); break;
            case 2: scatter_shifted<2>(s, d_al, n_words, b, lane); break;
            default: scatter_shifted<3>(s, d_al, n_words, b, lane); break;
        }
    }
    const uint32_t tail = rest & 15;
    const uint32_t done = head + (n_words << 4);
    if (lane < tail) dst[done + lane] = src[done + lane];
}

// ---------------------------------------------------------------- tile table built on the device

// The tile table of a tensor list, written by the device itself: one block per tensor, one thread per
// tile. The descriptors travel in the kernel arguments (a batch of up to kTileBatch tensors per
// launch), so nothing is copied from host memory and the launch can be recorded like any other.
// Tile i of a tensor whose padded extent is [d0, dend) of the data region: the extent is cut at its
// start and at every multiple of the tile size, exactly as the host planner cuts it.
__global__ __launch_bounds__(256) void build_tiles_kernel(TileBatch bt, ckpt_tile *__restrict__ table) {
    const uint32_t k = blockIdx.x;
    if (k >= bt.count) return;
    const uint64_t T = kPackTileBytes;
    const uint64_t d0 = bt.data_off[k], nbytes = bt.nbytes[k], src = bt.src[k];
    const uint64_t dend = d0 + (nbytes + 4095) / 4096 * 4096;
    const uint32_t n = bt.first_tile[k + 1] - bt.first_tile[k];
    ckpt_tile *out = table + bt.first_tile[k];
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
        const uint64_t start = i == 0 ? d0 : (d0 / T + i) * T;
        uint64_t stop = (d0 / T + i + 1) * T;
        if (stop > dend) stop = dend;
        const uint64_t rel = start - d0;
        const uint64_t left = rel >= nbytes ? 0 : nbytes - rel;
        ckpt_tile t;
        t.src = src + rel;
        t.dst_off = start;
        t.copy_bytes = uint32_t(left < stop - start ? left : stop - start);
        t.total_bytes = uint32_t(stop - start);
        t.reserved = 0;
        out[i] = t;
    }
}

// ---------------------------------------------------------------- launchers (host)

hipError_t launch_build_tiles(const TileBatch &bt, ckpt_tile *dev_table, hipStream_t stream) {
    if (bt.count == 0) return hipSuccess;
    hipLaunchKernelGGL(build_tiles_kernel, dim3(bt.count), dim3(256), 0, stream, bt, dev_table);
    return hipGetLastError();
}

static inline unsigned grid_for(uint64_t n_tiles) { return unsigned((n_tiles + kWavesPerBlock - 1) / kWavesPerBlock); }

hipError_t launch_pack(const ckpt_tile *dev_tiles, uint64_t n_tiles, void *slot_base, uint64_t slot_data_off, hipStream_t stream,
                       hipEvent_t t_start, hipEvent_t t_stop) {
    if (n_tiles == 0) return hipSuccess;
    if (t_start || t_stop)   // the events take the kernel's own start and end, not the moments two host calls around it were processed
        hipExtLaunchKernelGGL(pack_kernel, dim3(grid_for(n_tiles)), dim3(kBlock), 0, stream, t_start, t_stop, 0, dev_tiles, n_tiles,
                              static_cast<uint8_t *>(slot_base), slot_data_off);
    else
        hipLaunchKernelGGL(pack_kernel, dim3(grid_for(n_tiles)), dim3(kBlock), 0, stream, dev_tiles, n_tiles, static_cast<uint8_t *>(slot_base),
                           slot_data_off);
    return hipGetLastError();
}

hipError_t launch_scatter(const ckpt_tile *dev_tiles, uint64_t n_tiles, const void *slot_base, uint64_t slot_data_off, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(scatter_kernel, dim3(grid_for(n_tiles)), dim3(kBlock), 0, stream, dev_tiles, n_tiles,
                       static_cast<const uint8_t *>(slot_base), slot_data_off);
    return hipGetLastError();
}

}  // namespace dsllm
