// Synthetic training proxy kernels for gfx950 (see include/ckpt_proxy.h): bf16 MFMA GEMM,
// element-wise Adam step, seeded state fill, flat-buffer word fill/mutate, contiguous copy.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdint.h>

#include "../../include/ckpt_proxy.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------ counter-based random numbers

__device__ __forceinline__ uint64_t mix(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t mix_host(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static uint64_t stream_key(uint64_t seed, uint64_t tensor, uint64_t tag) { return mix_host(seed ^ mix_host(tensor * 4 + tag)); }

__device__ __forceinline__ float normal_from(uint64_t r) {
    const float u_hi = (float(uint32_t(r >> 40)) + 0.5f) * (1.0f / 16777216.0f);
    const float u_lo = (float(uint32_t(r & 0xFFFFFFu)) + 0.5f) * (1.0f / 16777216.0f);
    return sqrtf(-2.0f * logf(u_hi)) * cosf(6.28318530717958647692f * u_lo);
}

__device__ __forceinline__ uint16_t bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x0040u);
    return uint16_t((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// ------------------------------------------------------------------ state fill and Adam step

__global__ __launch_bounds__(256) void fill_state_kernel(uint16_t *__restrict__ p, float *__restrict__ master, float *__restrict__ m,
                                                        float *__restrict__ v, uint64_t numel, uint64_t k0, uint64_t k1, uint64_t k2) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < numel; i += stride) {
        const uint64_t hi = mix(i);
        const float w = 0.02f * normal_from(mix(k0 ^ hi));
        master[i] = w;
        p[i] = bf16_rne(w);
        m[i] = 0.02f * normal_from(mix(k1 ^ hi));
        const float s = 0.001f * normal_from(mix(k2 ^ hi));
        v[i] = s * s;
    }
}

struct AdamArgs { float lr, beta1, beta2, eps, inv_bc1, inv_bc2; };

__device__ __forceinline__ void adam_one(float &w, float &m, float &v, uint16_t &p, uint64_t key, uint64_t i, const AdamArgs &a) {
    const uint64_t r = mix(key ^ mix(i));
    const float g = 0.001f * (2.0f * (float(uint32_t(r >> 40)) * (1.0f / 16777216.0f)) - 1.0f);
    m = a.beta1 * m + (1.0f - a.beta1) * g;
    v = a.beta2 * v + (1.0f - a.beta2) * (g * g);
    const float mhat = m * a.inv_bc1, vhat = v * a.inv_bc2;
    w = w - a.lr * (mhat / (sqrtf(vhat) + a.eps));
    p = bf16_rne(w);
}

// four elements per thread step: 16-byte accesses to master, m, v and 8-byte ones to the bf16 copy
__global__ __launch_bounds__(256) void adam_kernel(uint16_t *__restrict__ p, float *__restrict__ master, float *__restrict__ m,
                                                  float *__restrict__ v, uint64_t numel, uint64_t key, AdamArgs a) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    const uint64_t n4 = numel >> 2;
    for (uint64_t q = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; q < n4; q += stride) {
        f32x4 w4 = reinterpret_cast<f32x4 *>(master)[q], m4 = reinterpret_cast<f32x4 *>(m)[q], v4 = reinterpret_cast<f32x4 *>(v)[q];
        float w[4] = {w4.x, w4.y, w4.z, w4.w}, mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w};
        uint16_t pb[4];
#pragma unroll
        for (int j = 0; j < 4; j++) adam_one(w[j], mm[j], vv[j], pb[j], key, 4 * q + j, a);
        reinterpret_cast<f32x4 *>(master)[q] = f32x4{w[0], w[1], w[2], w[3]};
        reinterpret_cast<f32x4 *>(m)[q] = f32x4{mm[0], mm[1], mm[2], mm[3]};
        reinterpret_cast<f32x4 *>(v)[q] = f32x4{vv[0], vv[1], vv[2], vv[3]};
        reinterpret_cast<u32x2 *>(p)[q] = u32x2{uint32_t(pb[0]) | (uint32_t(pb[1]) << 16), uint32_t(pb[2]) | (uint32_t(pb[3]) << 16)};
    }
    // ragged tail (numel not a multiple of 4)
    const uint64_t t = (n4 << 2) + uint64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t < numel) adam_one(master[t], m[t], v[t], p[t], key, t, a);
}

// ------------------------------------------------------------------ flat-buffer words, copy

__global__ __launch_bounds__(256) void fill_words_kernel(uint32_t *__restrict__ w, uint64_t n, uint64_t key) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) w[i] = uint32_t(mix(key ^ mix(i)));
}

__global__ __launch_bounds__(256) void mutate_words_kernel(uint32_t *__restrict__ w, uint64_t n, uint32_t step) {
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t i = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) w[i] = w[i] * 1664525u + 1013904223u + step;
}

__global__ __launch_bounds__(256) void devcopy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, uint64_t n16) {
    // each wavefront streams 32 KiB pieces, 16 x 16 bytes per lane in flight, like the pack kernel's aligned path
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t wave = uint64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const uint64_t n_waves = uint64_t(gridDim.x) * 4;
    for (uint64_t base = wave * 2048; base < n16; base += n_waves * 2048) {
        const uint64_t end = base + 2048 < n16 ? base + 2048 : n16;
        uint64_t i = base + lane;
        for (; i + 64 * 15 < end; i += 64 * 16) {
            u32x4 t[16];
#pragma unroll
            for (int u = 0; u < 16; u++) t[u] = __builtin_nontemporal_load(src + i + 64 * u);
#pragma unroll
            for (int u = 0; u < 16; u++) __builtin_nontemporal_store(t[u], dst + i + 64 * u);
        }
        for (; i < end; i += 64) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    }
}

// ------------------------------------------------------------------ bf16 GEMM on the matrix cores

// Block tile (64 T) x (64 T), K step BK, 256 threads = 4 wavefronts in a 2x2 arrangement, each computing a
// (32 T) x (32 T) sub-tile as T x T MFMA 32x32x16 tiles. Both operands are K-contiguous, so an A or B
// fragment (8 consecutive K values of one row/column per lane) is one 16-byte LDS read. LDS rows are
// padded by 16 bytes (80 bytes for BK = 32, 144 for BK = 64), which spreads the 16-byte reads of 16
// consecutive rows over all banks.
//
// T = 2, BK = 32 (128 x 128 block, 64 accumulator registers per lane, three blocks per CU) is LDS-bound: per
// MFMA one fragment read, and with the stores of the next tile the LDS pipe is busier than the matrix pipe.
// T = 4, BK = 64 (256 x 256 block, 144 KiB of LDS, one block per CU, one wave per SIMD, 256 accumulator
// registers per lane) halves the reads per MFMA: eight fragment reads feed sixteen MFMAs and LDS traffic is
// about three quarters of the matrix pipe's time. With one wave per SIMD no other wave hides a wait, so the
// loop is software-pipelined by hand: the fragments of K slice kk+1 are read while the MFMAs of slice kk run,
// the next tile's LDS stores go under the last slice's MFMAs, and scheduling fences keep that order.
template <int T, int BK>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const uint16_t *__restrict__ A, const uint16_t *__restrict__ B,
                                                       uint16_t *__restrict__ C, int M, int N, int K) {
    constexpr int BM = 64 * T, BN = 64 * T, WT = 32 * T;   // block tile and one wave's share of it
    constexpr int LDS_ROW = BK + 8;                        // in bf16 elements: rows padded by 16 bytes (80 or 144 bytes per row)
    constexpr int PIECES = BK / 8;                         // 16-byte pieces per row of a K step
    constexpr int ROWS_PER_PASS = 256 / PIECES, PASSES = BM / ROWS_PER_PASS;
    __shared__ __attribute__((aligned(16))) uint16_t lds_a[2][BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint16_t lds_b[2][BN * LDS_ROW];

    // consecutive block ids go to different XCDs (8 of them, each with its own L2): give each XCD a
    // contiguous range of tiles, walked in strips 8 tiles tall so that neighbours share A and B panels
    const int tiles_m = M / BM, tiles_n = N / BN, n_tiles = tiles_m * tiles_n;
    int bid = blockIdx.x;
    if (n_tiles % 8 == 0) bid = (bid % 8) * (n_tiles / 8) + bid / 8;
    const int strip = 8;
    const int per_strip = strip * tiles_n;
    const int s = bid / per_strip, in_s = bid % per_strip;
    const int rows_here = (tiles_m - s * strip) < strip ? (tiles_m - s * strip) : strip;
    const int tm = s * strip + in_s % rows_here, tn = in_s / rows_here;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const uint16_t *a_blk = A + size_t(tm) * BM * K;
    const uint16_t *b_blk = B + size_t(tn) * BN * K;

    // global -> LDS staging: thread t moves 16 bytes of row (t / PIECES + ROWS_PER_PASS * pass), K offset 8 * (t % PIECES)
    const int ld_row = tid / PIECES, ld_col = (tid % PIECES) * 8;
    u32x4 ra[PASSES], rb[PASSES];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ps++) {
            ra[ps] = *reinterpret_cast<const u32x4 *>(a_blk + size_t(ld_row + ROWS_PER_PASS * ps) * K + kt * BK + ld_col);
            rb[ps] = *reinterpret_cast<const u32x4 *>(b_blk + size_t(ld_row + ROWS_PER_PASS * ps) * K + kt * BK + ld_col);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ps++) {
            *reinterpret_cast<u32x4 *>(&lds_a[buf][(ld_row + ROWS_PER_PASS * ps) * LDS_ROW + ld_col]) = ra[ps];
            *reinterpret_cast<u32x4 *>(&lds_b[buf][(ld_row + ROWS_PER_PASS * ps) * LDS_ROW + ld_col]) = rb[ps];
        }
    };

    f32x16 acc[T][T];
#pragma unroll
    for (int i = 0; i < T; i++)
#pragma unroll
        for (int j = 0; j < T; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.0f;

    const int KT = K / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    bf16x8 fa[2][T], fb[2][T];          // two sets: the fragments of the next K slice are read while this slice's MFMAs run
    auto read_frags = [&](int set, int buf, int kk) {
#pragma unroll
        for (int i = 0; i < T; i++) {
            fa[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&lds_a[buf][(wm * WT + i * 32 + frag_row) * LDS_ROW + kk * 16 + frag_k]));
            fb[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&lds_b[buf][(wn * WT + i * 32 + frag_row) * LDS_ROW + kk * 16 + frag_k]));
        }
    };
    // The scheduler, left alone, sinks every fragment read to just before the MFMA that uses it and waits for it
    // there: with one wave per SIMD nothing hides that LDS latency. The fences below keep the order written
    // here: the reads of slice kk+1 are issued, then the MFMAs of slice kk run while those reads are in flight.
    read_frags(0, 0, 0);
    for (int kt = 0; kt < KT; kt++) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_tile(kt + 1);
#pragma unroll
        for (int kk = 0; kk < BK / 16; kk++) {
            if (kk + 1 < BK / 16) read_frags((kk + 1) & 1, buf, kk + 1);
            // the next tile goes to the other LDS buffer (whose readers left at the previous barrier) under the
            // last slice's MFMAs
            if (kk + 1 == BK / 16 && kt + 1 < KT) store_tile(buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < T; i++)
#pragma unroll
                for (int j = 0; j < T; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        if (kt + 1 < KT) read_frags(0, buf ^ 1, 0);
    }

    // accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile
    uint16_t *c_blk = C + size_t(tm) * BM * N + size_t(tn) * BN;
#pragma unroll
    for (int i = 0; i < T; i++)
#pragma unroll
        for (int j = 0; j < T; j++) {
#if defined(__HIP_DEVICE_COMPILE__)
            asm volatile("" : "+a"(acc[i][j]));      // this tile stays in its accumulator registers up to here
#endif
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int row = wm * WT + i * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                const int col = wn * WT + j * 32 + (lane & 31);
                c_blk[size_t(row) * N + col] = bf16_rne(acc[i][j][r]);
            }
            // one 32x32 tile at a time: without the pin above and this fence all accumulators are copied out at
            // once, the kernel then holds 256 + 256 registers per lane and no other wave fits on its SIMD
            __builtin_amdgcn_sched_barrier(0);
        }
}

unsigned blocks_for(uint64_t n, unsigned per_block) {
    uint64_t b = (n + per_block - 1) / per_block;
    const uint64_t cap = 256 * 16;   // 16 resident blocks' worth per CU; the kernels are grid-stride
    return unsigned(b < 1 ? 1 : (b > cap ? cap : b));
}

int hip_rc() { return hipGetLastError() == hipSuccess ? 0 : -4; }

}  // namespace

extern "C" {

int proxy_gemm_bf16(const void *a, const void *b, void *c, int32_t m, int32_t n, int32_t k, void *stream) {
    if (!a || !b || !c || m <= 0 || n <= 0 || k <= 0 || m % 128 || n % 128 || k % 64) return -1;
    if ((uint64_t(a) | uint64_t(b) | uint64_t(c)) & 15) return -1;
    // the 256 x 256 block tile where the shape allows it and there are enough tiles to fill the card
    if (m % 256 == 0 && n % 256 == 0 && (m / 256) * (n / 256) >= 256)
        hipLaunchKernelGGL((gemm_bf16_kernel<4, 64>), dim3((m / 256) * (n / 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                           static_cast<const uint16_t *>(a), static_cast<const uint16_t *>(b), static_cast<uint16_t *>(c), m, n, k);
    else
        hipLaunchKernelGGL((gemm_bf16_kernel<2, 32>), dim3((m / 128) * (n / 128)), dim3(256), 0, static_cast<hipStream_t>(stream),
                           static_cast<const uint16_t *>(a), static_cast<const uint16_t *>(b), static_cast<uint16_t *>(c), m, n, k);
    return hip_rc();
}

int proxy_fill_state(void *p, void *master, void *m, void *v, uint64_t numel, uint64_t seed, uint64_t tensor, void *stream) {
    if (!p || !master || !m || !v || numel == 0) return -1;
    hipLaunchKernelGGL(fill_state_kernel, dim3(blocks_for(numel, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint16_t *>(p), static_cast<float *>(master), static_cast<float *>(m), static_cast<float *>(v), numel,
                       stream_key(seed, tensor, 0), stream_key(seed, tensor, 1), stream_key(seed, tensor, 2));
    return hip_rc();
}

int proxy_adam_step(void *p, void *master, void *m, void *v, uint64_t numel, uint64_t seed, uint64_t tensor, uint64_t step, float lr,
                    float beta1, float beta2, float eps, void *stream) {
    if (!p || !master || !m || !v || numel == 0 || step == 0) return -1;
    if (((uint64_t(master) | uint64_t(m) | uint64_t(v)) & 15) || (uint64_t(p) & 7)) return -1;
    AdamArgs a;
    a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
    a.inv_bc1 = float(1.0 / (1.0 - pow(double(beta1), double(step))));
    a.inv_bc2 = float(1.0 / (1.0 - pow(double(beta2), double(step))));
    hipLaunchKernelGGL(adam_kernel, dim3(blocks_for((numel + 3) / 4, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint16_t *>(p), static_cast<float *>(master), static_cast<float *>(m), static_cast<float *>(v), numel,
                       stream_key(seed + step, tensor, 3), a);
    return hip_rc();
}

int proxy_fill_words(void *w, uint64_t n, uint64_t seed, void *stream) {
    if (!w || n == 0 || (uint64_t(w) & 3)) return -1;
    hipLaunchKernelGGL(fill_words_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<uint32_t *>(w), n,
                       stream_key(seed, 0, 0));
    return hip_rc();
}

int proxy_mutate_words(void *w, uint64_t n, uint64_t step, void *stream) {
    if (!w || n == 0 || (uint64_t(w) & 3)) return -1;
    hipLaunchKernelGGL(mutate_words_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<uint32_t *>(w), n,
                       uint32_t(step));
    return hip_rc();
}

int proxy_devcopy(void *dst, const void *src, uint64_t nbytes, void *stream) {
    if (!dst || !src || nbytes == 0 || (nbytes & 15) || ((uint64_t(dst) | uint64_t(src)) & 15)) return -1;
    const uint64_t n16 = nbytes >> 4;
    uint64_t pieces = (n16 + 2047) / 2048;
    uint64_t blocks = (pieces + 3) / 4;           // one piece per wavefront up to 4 GiB, grid-stride beyond
    if (blocks > (1u << 15)) blocks = 1u << 15;
    hipLaunchKernelGGL(devcopy_kernel, dim3(unsigned(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<u32x4 *>(dst),
                       static_cast<const u32x4 *>(src), n16);
    return hip_rc();
}

#define PROXY_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return -4; } } while (0)

int proxy_device_alloc(uint64_t nbytes, void **out) {
    if (!out || nbytes == 0) return -1;
    PROXY_TRY(hipMalloc(out, nbytes));
    return 0;
}
int proxy_device_free(void *dev) { if (!dev) return -1; PROXY_TRY(hipFree(dev)); return 0; }
int proxy_host_alloc_pinned(uint64_t nbytes, void **out) {
    if (!out || nbytes == 0) return -1;
    PROXY_TRY(hipHostMalloc(out, nbytes, hipHostMallocDefault));
    for (uint64_t o = 0; o < nbytes; o += 4096) static_cast<volatile char *>(*out)[o] = 0;
    return 0;
}
int proxy_host_free_pinned(void *host) { if (!host) return -1; PROXY_TRY(hipHostFree(host)); return 0; }
int proxy_copy_h2d(void *dst, const void *src, uint64_t n) { if (!dst || !src) return -1; if (n) PROXY_TRY(hipMemcpy(dst, src, n, hipMemcpyHostToDevice)); return 0; }
int proxy_copy_d2h(void *dst, const void *src, uint64_t n) { if (!dst || !src) return -1; if (n) PROXY_TRY(hipMemcpy(dst, src, n, hipMemcpyDeviceToHost)); return 0; }
int proxy_copy_d2d_async(void *dst, const void *src, uint64_t n, void *stream) {
    if (!dst || !src) return -1;
    if (n) PROXY_TRY(hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
    return 0;
}
int proxy_copy_pinned_async(void *dst, const void *src, uint64_t n, int32_t to_host, void *stream) {
    if (!dst || !src) return -1;
    if (n) PROXY_TRY(hipMemcpyAsync(dst, src, n, to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)));
    return 0;
}
int proxy_device_fill_async(void *dev, int32_t byte, uint64_t n, void *stream) {
    if (!dev) return -1;
    if (n) PROXY_TRY(hipMemsetAsync(dev, byte, n, static_cast<hipStream_t>(stream)));
    return 0;
}
int proxy_stream_synchronize(void *stream) { PROXY_TRY(hipStreamSynchronize(static_cast<hipStream_t>(stream))); return 0; }
int proxy_device_synchronize(void) { PROXY_TRY(hipDeviceSynchronize()); return 0; }
int proxy_event_create(void **out) { if (!out) return -1; hipEvent_t e; PROXY_TRY(hipEventCreate(&e)); *out = e; return 0; }
int proxy_event_destroy(void *e) { if (!e) return -1; PROXY_TRY(hipEventDestroy(static_cast<hipEvent_t>(e))); return 0; }
int proxy_event_record(void *e, void *stream) { if (!e) return -1; PROXY_TRY(hipEventRecord(static_cast<hipEvent_t>(e), static_cast<hipStream_t>(stream))); return 0; }
int proxy_event_synchronize(void *e) { if (!e) return -1; PROXY_TRY(hipEventSynchronize(static_cast<hipEvent_t>(e))); return 0; }
int proxy_event_elapsed_ms(void *a, void *b, float *ms) {
    if (!a || !b || !ms) return -1;
    PROXY_TRY(hipEventElapsedTime(ms, static_cast<hipEvent_t>(a), static_cast<hipEvent_t>(b)));
    return 0;
}
int proxy_device_info(char *name, uint64_t cap, int32_t *cus, uint64_t *total, uint64_t *free_, int32_t *ver) {
    int dev = 0;
    PROXY_TRY(hipGetDevice(&dev));
    hipDeviceProp_t p;
    PROXY_TRY(hipGetDeviceProperties(&p, dev));
    if (name && cap) { snprintf(name, cap, "%s (%s)", p.name, p.gcnArchName); }
    if (cus) *cus = p.multiProcessorCount;
    size_t f = 0, t = 0;
    PROXY_TRY(hipMemGetInfo(&f, &t));
    if (total) *total = t;
    if (free_) *free_ = f;
    int v = 0;
    PROXY_TRY(hipRuntimeGetVersion(&v));
    if (ver) *ver = v;
    return 0;
}

int proxy_stream_create(void **out) {
    if (!out) return -1;
    hipStream_t s = nullptr;
    if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) return -4;
    *out = s;
    return 0;
}

int proxy_stream_destroy(void *stream) {
    if (!stream) return -1;
    return hipStreamDestroy(static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : -4;
}

}  // extern "C"
