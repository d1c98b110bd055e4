/*
 * Synthetic training proxy for measuring the snapshot path: a compute-bound bf16 GEMM that stands
 * in for the forward and backward passes (the phase in which, per the paper's observation on
 * immutability, parameters and optimizer state are only read), an element-wise Adam step that
 * stands in for the update phase that mutates all of them, seeded state generators, and a plain
 * device copy that measures the HBM copy ceiling. Measurement harness only: the checkpoint engine
 * (ckpt.h) does not depend on it.
 *
 * Plain C ABI; every `dev_` pointer is a device address on the current HIP device; `stream` is a
 * hipStream_t passed as void*. Returns 0 on success, -1 on a bad argument, -4 on a HIP error.
 * All kernels are deterministic (no atomics): same inputs, same bits.
 *
 * The random numbers are counter based so that a CPU implementation can reproduce them:
 *   mix(x):  z = x + 0x9E3779B97F4A7C15; z = (z ^ z>>30) * 0xBF58476D1CE4E5B9;
 *            z = (z ^ z>>27) * 0x94D049BB133111EB; return z ^ z>>31          (64-bit, wrapping)
 *   r(seed, tensor, tag, i) = mix( mix(seed ^ mix(tensor * 4 + tag)) ^ mix(i) )
 *   u_hi = ((r >> 40) + 0.5) / 2^24,  u_lo = ((r & 0xFFFFFF) + 0.5) / 2^24
 *   normal(seed, tensor, tag, i) = sqrt(-2 ln u_hi) * cos(2 pi u_lo)           (Box-Muller)
 */
#ifndef DSLLM_CKPT_PROXY_H
#define DSLLM_CKPT_PROXY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = A[M,K] * B[N,K]^T. A, B, C row-major bf16; accumulation in f32 on the matrix cores;
 * C rounded to bf16 (nearest even). M and N multiples of 128, K a multiple of 64. */
int proxy_gemm_bf16(const void *dev_a, const void *dev_b, void *dev_c, int32_t m, int32_t n, int32_t k, void *stream);

/* Fills the four state tensors of parameter tensor `tensor`: master = 0.02 * normal(tag 0),
 * p_bf16 = bf16(master), m = 0.02 * normal(tag 1), v = (0.001 * normal(tag 2))^2. */
int proxy_fill_state(void *dev_p_bf16, void *dev_master, void *dev_m, void *dev_v, uint64_t numel, uint64_t seed,
                     uint64_t tensor, void *stream);

/* One Adam step, step number `step` >= 1, on elements [0, numel):
 *   g = 0.001 * (2 * (r(seed + step, tensor, 3, i) >> 40) / 2^24 - 1)
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   master -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps);  p_bf16 = bf16(master)
 * in f32 arithmetic. */
int proxy_adam_step(void *dev_p_bf16, void *dev_master, void *dev_m, void *dev_v, uint64_t numel, uint64_t seed,
                    uint64_t tensor, uint64_t step, float lr, float beta1, float beta2, float eps, void *stream);

/* 32-bit words of a flat buffer: fill w[i] = low 32 bits of r(seed, 0, 0, i); mutate
 * w[i] = w[i] * 1664525 + 1013904223 + step (wrapping). The update stand-in for shards that are
 * carved out of flat buffers. */
int proxy_fill_words(void *dev_words, uint64_t n_words, uint64_t seed, void *stream);
int proxy_mutate_words(void *dev_words, uint64_t n_words, uint64_t step, void *stream);

/* dst[0..nbytes) = src[0..nbytes), both 16-byte aligned, nbytes a multiple of 16: the contiguous
 * copy whose bandwidth is the practical ceiling for the pack kernel. */
int proxy_devcopy(void *dev_dst, const void *dev_src, uint64_t nbytes, void *stream);

/* ---- device memory, copies, events: thin wrappers so that a harness needs no other GPU package ----
 * All return 0 on success, -1 on a bad argument, -4 on a HIP error. Copies marked blocking return
 * when the bytes have arrived; host pointers of the blocking copies may be pageable. */
int proxy_device_alloc(uint64_t nbytes, void **dev_out);              /* hipMalloc */
int proxy_device_free(void *dev);
int proxy_host_alloc_pinned(uint64_t nbytes, void **host_out);        /* hipHostMalloc, pages touched */
int proxy_host_free_pinned(void *host);
int proxy_copy_h2d(void *dev_dst, const void *host_src, uint64_t nbytes);                 /* blocking */
int proxy_copy_d2h(void *host_dst, const void *dev_src, uint64_t nbytes);                 /* blocking */
int proxy_copy_d2d_async(void *dev_dst, const void *dev_src, uint64_t nbytes, void *stream);
int proxy_copy_pinned_async(void *dst, const void *src, uint64_t nbytes, int32_t to_host, void *stream);
int proxy_device_fill_async(void *dev, int32_t byte, uint64_t nbytes, void *stream);      /* hipMemsetAsync */
int proxy_stream_synchronize(void *stream);
int proxy_device_synchronize(void);
int proxy_event_create(void **event_out);                             /* timing enabled */
int proxy_event_destroy(void *event);
int proxy_event_record(void *event, void *stream);
int proxy_event_synchronize(void *event);
int proxy_event_elapsed_ms(void *start, void *stop, float *ms_out);
int proxy_device_info(char *name_buf, uint64_t name_cap, int32_t *cu_count, uint64_t *total_mem, uint64_t *free_mem,
                      int32_t *runtime_version);

/* A plain non-blocking HIP stream of default priority (hipStreamCreateWithFlags), returned as void*.
 * The harness takes its compute stream from here instead of a framework's stream pool: every HIP
 * stream is mapped onto one of a few hardware queues, and work of two streams that share a queue
 * runs in submission order, so the compute stream must not share a hardware queue with the
 * library's pack and copy streams. Creating the few streams that are really used, one after the
 * other, gives each a queue of its own. */
int proxy_stream_create(void **stream_out);
int proxy_stream_destroy(void *stream);

#ifdef __cplusplus
}
#endif
#endif
