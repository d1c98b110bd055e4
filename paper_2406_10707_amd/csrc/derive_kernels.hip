// Kernels of the data reduction (format version 2): a bf16 working copy that is the round-to-nearest-even
// of its f32 master weights is not stored. verify_pairs_kernel checks, on the captured state, that every
// declared pair really is one (so that leaving the copy out loses nothing); derive_pairs_kernel recomputes
// the copies after a restore. Both are HBM-bound streaming kernels: 6 bytes per element read (verify),
// 4 read + 2 written (derive). The rounding is integer arithmetic on the bit pattern, the same definition
// the file format states, so both sides of a comparison take the decision in the same (exact) arithmetic.
//
// One wavefront per tile of up to kPairTileElems elements, descriptor through scalar loads, 16-byte loads
// of the f32 side (4 elements per lane per step) and 8-byte accesses of the bf16 side when both are
// aligned for it; element-wise accesses otherwise (tensors are aligned to their element size only).
#include "kernel_util.hpp"
#include "plan.hpp"

namespace dsllm {

constexpr int kPairWaves = 4;
constexpr int kPairUnroll = 4;

__device__ __forceinline__ uint32_t bf16_rne(uint32_t u) {
    const uint32_t nan = (u >> 16) | 0x0040u;
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u ? nan : rounded) & 0xFFFFu;
}

// the four bf16 patterns of four f32 patterns, packed as they lie in memory
__device__ __forceinline__ u32x2 bf16_rne4(u32x4 m) {
    return u32x2{bf16_rne(m.x) | (bf16_rne(m.y) << 16), bf16_rne(m.z) | (bf16_rne(m.w) << 16)};
}

__device__ __forceinline__ u32x2 ld8(const u32x2 *p) { return __builtin_nontemporal_load((const u32x2 DSLLM_GLOBAL *)p); }
__device__ __forceinline__ void st8(u32x2 *p, u32x2 v) { __builtin_nontemporal_store(v, (u32x2 DSLLM_GLOBAL *)p); }

// WRITE = false: *mismatch is set to 1 if any element of a bf16 tensor differs from the rounding of its source.
// WRITE = true: the bf16 tensors are overwritten with the rounding of their sources.
template <bool WRITE>
__device__ __forceinline__ void pairs_body(const PairTile *__restrict__ tiles, uint64_t n_tiles, uint32_t *mismatch) {
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t t = uint64_t(blockIdx.x) * kPairWaves + uniform_u32(threadIdx.x >> 6);   // uniform: scalar descriptor loads
    if (t >= n_tiles) return;
    const PairTile *tp = tiles + t;
    const uint64_t f32_addr = uniform_u64(tp->f32_addr), bf16_addr = uniform_u64(tp->bf16_addr);
    const uint32_t count = uniform_u32(tp->count);
    const uint32_t *m1 = reinterpret_cast<const uint32_t *>(f32_addr);
    uint16_t *p1 = reinterpret_cast<uint16_t *>(bf16_addr);
    bool bad = false;
    if ((f32_addr & 15) == 0 && (bf16_addr & 7) == 0) {
        const u32x4 *m = reinterpret_cast<const u32x4 *>(f32_addr);
        u32x2 *p = reinterpret_cast<u32x2 *>(bf16_addr);
        const uint32_t n4 = count >> 2;
        uint32_t i = lane;
        for (; i + 64 * (kPairUnroll - 1) < n4; i += 64 * kPairUnroll) {
            u32x4 v[kPairUnroll];
            u32x2 have[kPairUnroll];
#pragma unroll
            for (int u = 0; u < kPairUnroll; u++) {
                v[u] = ld16(m + i + 64 * u);
                if (!WRITE) have[u] = ld8(p + i + 64 * u);
            }
#pragma unroll
            for (int u = 0; u < kPairUnroll; u++) {
                const u32x2 want = bf16_rne4(v[u]);
                if (WRITE) st8(p + i + 64 * u, want);
                else bad |= (want.x != have[u].x) | (want.y != have[u].y);
            }
        }
        for (; i < n4; i += 64) {
            const u32x2 want = bf16_rne4(ld16(m + i));
            if (WRITE) st8(p + i, want);
            else { const u32x2 have = ld8(p + i); bad |= (want.x != have.x) | (want.y != have.y); }
        }
        const uint32_t e = (n4 << 2) + lane;      // up to three elements behind the last group of four
        if (e < count) {
            const uint32_t want = bf16_rne(m1[e]);
            if (WRITE) p1[e] = uint16_t(want);
            else bad |= want != p1[e];
        }
    } else {
        for (uint32_t e = lane; e < count; e += 64) {
            const uint32_t want = bf16_rne(m1[e]);
            if (WRITE) p1[e] = uint16_t(want);
            else bad |= want != p1[e];
        }
    }
    if (!WRITE && bad) *mismatch = 1;     // every lane that found a difference stores the same value: no atomics needed
}

__global__ __launch_bounds__(64 * kPairWaves) void verify_pairs_kernel(const PairTile *__restrict__ tiles, uint64_t n_tiles, uint32_t *mismatch) {
    pairs_body<false>(tiles, n_tiles, mismatch);
}

__global__ __launch_bounds__(64 * kPairWaves) void derive_pairs_kernel(const PairTile *__restrict__ tiles, uint64_t n_tiles) {
    pairs_body<true>(tiles, n_tiles, nullptr);
}

__global__ void clear_word_kernel(uint32_t *word) { *word = 0; }

// Clears the flag and checks every pair; the flag is 1 afterwards if any pair does not hold.
hipError_t launch_verify_pairs(const PairTile *dev_tiles, uint64_t n_tiles, uint32_t *dev_flag, hipStream_t stream) {
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, stream, dev_flag);
    if (n_tiles)
        hipLaunchKernelGGL(verify_pairs_kernel, dim3(unsigned((n_tiles + kPairWaves - 1) / kPairWaves)), dim3(64 * kPairWaves), 0, stream, dev_tiles,
                           n_tiles, dev_flag);
    return hipGetLastError();
}

hipError_t launch_derive_pairs(const PairTile *dev_tiles, uint64_t n_tiles, hipStream_t stream) {
    if (n_tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(derive_pairs_kernel, dim3(unsigned((n_tiles + kPairWaves - 1) / kPairWaves)), dim3(64 * kPairWaves), 0, stream, dev_tiles, n_tiles);
    return hipGetLastError();
}

}  // namespace dsllm
