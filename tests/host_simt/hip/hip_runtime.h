// Runs the library's HIP kernels on the HOST, for test builds under AddressSanitizer only.
// Every workgroup of a launch is executed by a pool of host threads, one per lane, with
// __syncthreads() as a real barrier and __shared__ arrays as statics, so the kernels' own index
// arithmetic (global offsets, LDS indices, the workgroup-to-tile mapping, the launch shapes)
// is checked access by access against the exact extents of malloc'ed buffers.  The rest of the
// runtime (streams, events, pinned memory) comes from the stand-in in tests/fake_hip.
// Test infrastructure: the product is never built against this header.
#pragma once
#include "../../fake_hip/hip/hip_runtime.h"

#include <pthread.h>

#include <algorithm>
#include <cstdint>
#include <functional>
#include <thread>
#include <vector>

struct dim3 {
    uint32_t x, y, z;
    dim3(uint32_t x_ = 1, uint32_t y_ = 1, uint32_t z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct uint3_ { uint32_t x, y, z; };
extern thread_local uint3_ threadIdx;
extern uint3_ blockIdx, blockDim, gridDim;

#define __global__
#define __device__
#define __forceinline__ inline
#define __shared__ static
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))
#define __builtin_amdgcn_s_setprio(level) ((void)0)  // wave priority means nothing on the host
#define __builtin_amdgcn_readfirstlane(x) (x)
static inline uint32_t atomicAdd(uint32_t *p, uint32_t v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
using std::min;
static inline uint32_t __umulhi(uint32_t a, uint32_t b) { return uint32_t((uint64_t(a) * b) >> 32); }

namespace host_simt {
// A pool of host threads, one per lane of a workgroup of `n` lanes; the workgroups of a launch
// run one after another on it (they share the statics that stand for LDS).
struct Pool {
    pthread_barrier_t start, done, sync;
    std::vector<std::thread> lanes;
    std::function<void()> job;
    bool quit = false;
    explicit Pool(uint32_t n) {
        pthread_barrier_init(&start, nullptr, n + 1);
        pthread_barrier_init(&done, nullptr, n + 1);
        pthread_barrier_init(&sync, nullptr, n);
        for (uint32_t t = 0; t < n; ++t)
            lanes.emplace_back([this, t] {
                for (;;) {
                    pthread_barrier_wait(&start);
                    if (quit) return;
                    threadIdx = {t, 0, 0};
                    job();
                    pthread_barrier_wait(&done);
                }
            });
    }
    ~Pool() {
        quit = true;
        pthread_barrier_wait(&start);
        for (std::thread &l : lanes) l.join();
        pthread_barrier_destroy(&start);
        pthread_barrier_destroy(&done);
        pthread_barrier_destroy(&sync);
    }
    void run_block(const std::function<void()> &f) {
        job = f;
        pthread_barrier_wait(&start);
        pthread_barrier_wait(&done);
    }
};
Pool &pool(uint32_t lanes);
extern pthread_barrier_t *current_sync;
extern long launches, blocks_run;
inline void launch(dim3 grid, dim3 block, const std::function<void()> &body) {
    ++launches;
    gridDim = {grid.x, 1, 1};
    blockDim = {block.x, 1, 1};
    Pool &p = pool(block.x);
    current_sync = &p.sync;
    for (uint32_t b = 0; b < grid.x; ++b) {
        blockIdx = {b, 0, 0};
        p.run_block(body);
        ++blocks_run;
    }
}
}  // namespace host_simt

// every lane of the workgroup must reach it, as on the device (a lane that returned early would hang here)
#define __syncthreads() pthread_barrier_wait(host_simt::current_sync)
#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    host_simt::launch(grid, block, [=] { kernel(__VA_ARGS__); })

enum { hipDeviceAttributeMultiprocessorCount = 1 };
inline hipError_t hipGetDevice(int *d) { *d = 0; return hipSuccess; }
inline hipError_t hipDeviceGetAttribute(int *v, int, int) { *v = 4; return hipSuccess; }
template <typename T> inline hipError_t hipGetSymbolAddress(void **p, T *symbol) { *p = const_cast<void *>(static_cast<const void *>(symbol)); return hipSuccess; }
inline hipError_t hipMalloc(void **p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
inline hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
