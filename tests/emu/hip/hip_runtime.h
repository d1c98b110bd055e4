// Stand-in for <hip/hip_runtime.h> that lets the library's sources be compiled for the HOST:
//  * the pack/scatter kernel source runs thread by thread (AddressSanitizer then checks every
//    address the kernels compute against exactly sized buffers), and
//  * the engine (streams, events, asynchronous copies, kernel launches) runs against a small model of
//    the HIP execution model: every stream is a thread that executes its queue in order, events carry
//    a record generation, a stream-wait captures the generation at the time of the call. Under
//    ThreadSanitizer a missing dependency between streams (say a copy that does not wait for the
//    pack kernel) shows up as a data race on the buffers involved.
// Test infrastructure; only what the library uses.
#pragma once
#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <atomic>
#include <functional>
#include <mutex>
#include <thread>

#include <unistd.h>

// File writes of the engine go through a function the test program owns, so that a test can make one
// particular write fail, hold it back, or end the process in the middle of a flush. (unistd.h is included
// above, so its own declaration of pwrite is already past when the name is redirected.)
ssize_t emu_pwrite(int fd, const void *buf, size_t n, off_t off);
#define pwrite emu_pwrite

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
// one "thread" runs at a time per launch, and launches of different streams may run at the same time: LDS of the
// model belongs to the host thread that runs the launch (only kernels whose lanes read back what they wrote themselves)
#define __shared__ static thread_local
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x

typedef int hipError_t;
static const hipError_t hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorNotSupported = 801;
inline hipError_t hipGetLastError() { return hipSuccess; }
inline const char *hipGetErrorString(hipError_t e) { return e == hipSuccess ? "no error" : "emulated error"; }

// the descriptor is identical in every lane of a wavefront, so the first lane's value is the lane's own;
// like the real builtin this returns a SIGNED int (a careless widening sign-extends, as on the GPU)
#define __builtin_amdgcn_readfirstlane(x) int(x)
// v_alignbyte_b32: low 32 bits of ({hi,lo} >> 8*(shift & 3))
static inline uint32_t emu_alignbyte(uint32_t hi, uint32_t lo, uint32_t shift) {
    return uint32_t(((uint64_t(hi) << 32) | lo) >> (8 * (shift & 3)));
}
#define __builtin_amdgcn_alignbyte(hi, lo, s) emu_alignbyte(hi, lo, s)

// ---------------------------------------------------------------- streams and events

struct EmuStream {
    std::mutex m;
    std::condition_variable cv;
    std::deque<std::function<void()>> q;
    uint64_t enqueued = 0, done = 0;
    bool stop = false;
    std::thread th;
    EmuStream() {
        th = std::thread([this] {
            for (;;) {
                std::function<void()> f;
                {
                    std::unique_lock<std::mutex> lk(m);
                    cv.wait(lk, [&] { return stop || !q.empty(); });
                    if (q.empty()) return;
                    f = std::move(q.front());
                    q.pop_front();
                }
                f();
                {
                    std::lock_guard<std::mutex> lk(m);
                    done++;
                }
                cv.notify_all();
            }
        });
    }
    void push(std::function<void()> f) {
        {
            std::lock_guard<std::mutex> lk(m);
            q.push_back(std::move(f));
            enqueued++;
        }
        cv.notify_all();
    }
    void drain() {
        std::unique_lock<std::mutex> lk(m);
        const uint64_t target = enqueued;
        cv.wait(lk, [&] { return done >= target; });
    }
    ~EmuStream() {
        drain();
        {
            std::lock_guard<std::mutex> lk(m);
            stop = true;
        }
        cv.notify_all();
        th.join();
    }
};
typedef EmuStream *hipStream_t;

struct EmuEvent {
    std::mutex m;
    std::condition_variable cv;
    uint64_t recorded = 0, completed = 0;
    std::chrono::steady_clock::time_point when;
};
typedef EmuEvent *hipEvent_t;

enum { hipStreamNonBlocking = 1, hipEventDefault = 0, hipEventBlockingSync = 1, hipEventDisableTiming = 2, hipHostMallocDefault = 0 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
enum hipMemoryType { hipMemoryTypeHost = 1, hipMemoryTypeDevice = 2 };
struct hipPointerAttribute_t { hipMemoryType type; int device; };
typedef void *hipDeviceptr_t;

// the null stream of the model executes immediately in the calling thread
// a test may watch what is enqueued where (called with the stream of every submission, before it is queued)
inline std::atomic<void (*)(hipStream_t)> g_emu_submit_hook{nullptr};
inline void emu_submit(hipStream_t s, std::function<void()> f) {
    if (auto hook = g_emu_submit_hook.load()) hook(s);
    if (s) s->push(std::move(f)); else f();
}

inline hipError_t hipSetDevice(int) { return hipSuccess; }
inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
template <class T> inline hipError_t hipGetSymbolAddress(void **p, T &symbol) { *p = &symbol; return hipSuccess; }   // the model has one "device"
inline hipError_t hipGetDeviceCount(int *n) { *n = 1; return hipSuccess; }
inline hipError_t hipMalloc(void **p, size_t n) { *p = aligned_alloc(256, (n + 255) / 256 * 256); return *p ? hipSuccess : hipErrorOutOfMemory; }
inline hipError_t hipFree(void *p) { free(p); return hipSuccess; }
inline hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = aligned_alloc(4096, (n + 4095) / 4096 * 4096); return *p ? hipSuccess : hipErrorOutOfMemory; }
inline hipError_t hipHostFree(void *p) { free(p); return hipSuccess; }
inline hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return hipSuccess; }
inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t st) {
    emu_submit(st, [=] { memcpy(d, s, n); });
    return hipSuccess;
}
inline hipError_t hipPointerGetAttributes(hipPointerAttribute_t *a, const void *) { a->type = hipMemoryTypeDevice; a->device = 0; return hipSuccess; }
inline hipError_t hipMemGetAddressRange(hipDeviceptr_t *, size_t *, hipDeviceptr_t) { return hipErrorNotSupported; }

inline hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = new EmuStream; return hipSuccess; }
inline hipError_t hipStreamDestroy(hipStream_t s) { delete s; return hipSuccess; }
inline hipError_t hipStreamSynchronize(hipStream_t s) { if (s) s->drain(); return hipSuccess; }
inline hipError_t hipStreamQuery(hipStream_t s) {
    if (!s) return hipSuccess;
    std::lock_guard<std::mutex> lk(s->m);
    return s->done >= s->enqueued ? hipSuccess : 600;   // hipErrorNotReady
}

inline hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = new EmuEvent; return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t *e) { return hipEventCreateWithFlags(e, 0); }
inline hipError_t hipEventDestroy(hipEvent_t e) { delete e; return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
    uint64_t gen;
    {
        std::lock_guard<std::mutex> lk(e->m);
        gen = ++e->recorded;
    }
    emu_submit(s, [e, gen] {
        std::lock_guard<std::mutex> lk(e->m);     // notify under the lock: a waiter may destroy the event right after
        if (gen > e->completed) { e->completed = gen; e->when = std::chrono::steady_clock::now(); }
        e->cv.notify_all();
    });
    return hipSuccess;
}
inline hipError_t hipEventSynchronize(hipEvent_t e) {
    std::unique_lock<std::mutex> lk(e->m);
    const uint64_t gen = e->recorded;       // never recorded: returns at once, like the real call
    e->cv.wait(lk, [&] { return e->completed >= gen; });
    return hipSuccess;
}
static const hipError_t hipErrorNotReady = 600;
inline hipError_t hipEventQuery(hipEvent_t e) {
    std::lock_guard<std::mutex> lk(e->m);
    return e->completed >= e->recorded ? hipSuccess : hipErrorNotReady;
}
inline hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
    uint64_t gen;
    {
        std::lock_guard<std::mutex> lk(e->m);
        gen = e->recorded;                  // the wait is for the record that exists NOW
    }
    if (gen == 0) return hipSuccess;
    emu_submit(s, [e, gen] {
        std::unique_lock<std::mutex> lk(e->m);
        e->cv.wait(lk, [&] { return e->completed >= gen; });
    });
    return hipSuccess;
}
inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t a, hipEvent_t b) {
    std::lock_guard<std::mutex> la(a->m);
    std::chrono::steady_clock::time_point ta = a->when;
    std::chrono::steady_clock::time_point tb;
    if (a == b) tb = ta; else { std::lock_guard<std::mutex> lb(b->m); tb = b->when; }
    *ms = std::chrono::duration<float, std::milli>(tb - ta).count();
    return hipSuccess;
}

// ---------------------------------------------------------------- kernel launches

template <class F>
static inline void emu_run_grid(dim3 grid, dim3 block, F body) {
    gridDim = grid;
    blockDim = block;
    for (unsigned b = 0; b < grid.x; b++)
        for (unsigned t = 0; t < block.x; t++) {
            blockIdx = dim3(b);
            threadIdx = dim3(t);
            body();
        }
}
// kernels without barriers or cross-lane traffic can be run one thread after the other; the launch is
// queued on the stream like any other operation (arguments captured by value)
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    emu_submit(stream, [=] { emu_run_grid(grid, block, [&] { kernel(__VA_ARGS__); }); })
// the launch that also fills a start and a stop event: here the events are recorded around the launch
#define hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, start_ev, stop_ev, flags, ...)          \
    do {                                                                                                  \
        if (start_ev) (void)hipEventRecord(start_ev, stream);                                             \
        hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                              \
        if (stop_ev) (void)hipEventRecord(stop_ev, stream);                                               \
    } while (0)
