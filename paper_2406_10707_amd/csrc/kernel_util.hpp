// Small device-side helpers shared by the library's kernels (pack, scatter, derivation check).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dsllm {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Tensor addresses come out of the descriptor table as integers, so the compiler cannot know they
// are global memory and would use flat loads (which also pass through the LDS address check and
// count against two wait counters). Casting to the global address space gives global_load/store.
#if defined(__HIP_DEVICE_COMPILE__)
#define DSLLM_GLOBAL __attribute__((address_space(1)))
// Keeps a loaded 16-byte word whole and in registers of its own. Without it the compiler narrows the
// two loads of the misaligned path to the dwords the shift uses and packs them into overlapping
// registers, which forces a wait after every pair of loads.
#define DSLLM_KEEP_WHOLE(v) asm volatile("" : "+v"(v))
#else
#define DSLLM_GLOBAL
#define DSLLM_KEEP_WHOLE(v) (void)0
#endif
__device__ __forceinline__ u32x4 ld16(const u32x4 *p) { return __builtin_nontemporal_load((const u32x4 DSLLM_GLOBAL *)p); }
typedef u32x4 u32x4_bytealigned __attribute__((aligned(1)));
// 16 bytes from any byte address; all 16 must lie inside the tensor
__device__ __forceinline__ u32x4 ld16_unaligned(const uint8_t *p) { return __builtin_nontemporal_load((const u32x4_bytealigned DSLLM_GLOBAL *)p); }
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, (u32x4 DSLLM_GLOBAL *)p); }

// A value that is the same in every lane of the wavefront, moved to scalar registers. The builtin
// returns a signed int: each half goes through uint32_t before widening, or the low half would be
// sign-extended into the high one.
__device__ __forceinline__ uint32_t uniform_u32(uint32_t v) { return uint32_t(__builtin_amdgcn_readfirstlane(v)); }
__device__ __forceinline__ uint64_t uniform_u64(uint64_t v) {
    const uint32_t lo = uniform_u32(uint32_t(v)), hi = uniform_u32(uint32_t(v >> 32));
    return (uint64_t(hi) << 32) | uint64_t(lo);
}

}  // namespace dsllm
