// Stand-in for <hip/hip_runtime.h> that lets the pack/scatter kernel source be compiled for the HOST
// and run thread by thread under AddressSanitizer: every address the kernels compute is then
// bounds-checked on the CPU before the same code is trusted on a GPU. Only what those kernels use.
#pragma once
#include <cstdint>
#include <cstring>

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
extern thread_local dim3 threadIdx, blockIdx, blockDim, gridDim;

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)

typedef int hipError_t;
static const hipError_t hipSuccess = 0;
typedef void *hipStream_t;
inline hipError_t hipGetLastError() { return hipSuccess; }

// the descriptor is identical in every lane of a wavefront, so the first lane's value is the lane's own;
// like the real builtin this returns a SIGNED int (a careless widening sign-extends, as on the GPU)
#define __builtin_amdgcn_readfirstlane(x) int(x)
// v_alignbyte_b32: low 32 bits of ({hi,lo} >> 8*(shift & 3))
static inline uint32_t emu_alignbyte(uint32_t hi, uint32_t lo, uint32_t shift) {
    return uint32_t(((uint64_t(hi) << 32) | lo) >> (8 * (shift & 3)));
}
#define __builtin_amdgcn_alignbyte(hi, lo, s) emu_alignbyte(hi, lo, s)

template <class F>
static inline void emu_launch(dim3 grid, dim3 block, F body) {
    gridDim = grid;
    blockDim = block;
    for (unsigned b = 0; b < grid.x; b++)
        for (unsigned t = 0; t < block.x; t++) {
            blockIdx = dim3(b);
            threadIdx = dim3(t);
            body();
        }
}
// kernels without barriers or cross-lane traffic can be run one thread after the other
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) emu_launch(grid, block, [&] { kernel(__VA_ARGS__); })
