/*
 * A stand-in for <hip/hip_runtime.h> that runs HIP kernels on host threads, one thread per
 * GPU thread, one workgroup at a time.  It exists so that the decode kernels' own source
 * can be compiled for the host and run under AddressSanitizer, UBSan and ThreadSanitizer
 * (tests/test_kernel_cpu_build.py): "device" memory is host memory, so every access a
 * kernel makes outside a buffer is reported, and LDS is ordinary static memory, so every
 * unsynchronised pair of accesses is.  Only what those kernels and their host code use is
 * here.  Test infrastructure; nothing in the library includes it.
 */
#ifndef L3_KERNEL_CPU_HIP_RUNTIME_H
#define L3_KERNEL_CPU_HIP_RUNTIME_H

#include <pthread.h>
#include <stdint.h>

#include <cstdlib>
#include <cstring>
#include <functional>
#include <map>
#include <thread>
#include <vector>

/* ---- language ------------------------------------------------------------- */

#define __global__
#define __device__
#define __host__
#define __shared__ static          /* one workgroup runs at a time */
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};

namespace l3cpu {

constexpr int kWave = 64;

/* what the threads of the workgroup that is running share */
struct Workgroup {
    unsigned threads = 0;
    pthread_barrier_t all;
    pthread_barrier_t wave[16];
    uint32_t exchange[16][2][kWave];   /* [wave][parity][lane]: values handed between lanes */
};
inline Workgroup*& workgroup() {
    static Workgroup* wg = nullptr;
    return wg;
}
inline dim3& grid_dim() {
    static dim3 d;
    return d;
}
inline dim3& block_dim() {
    static dim3 d;
    return d;
}
inline thread_local dim3 t_thread_idx, t_block_idx;
inline thread_local unsigned t_parity = 0;

inline unsigned lane() { return t_thread_idx.x % kWave; }
inline unsigned wave() { return t_thread_idx.x / kWave; }

inline void wave_barrier() { pthread_barrier_wait(&workgroup()->wave[wave()]); }
inline void workgroup_barrier() { pthread_barrier_wait(&workgroup()->all); }

/* every lane of the wave hands a value in and gets the wave's 64 values to read: the
 * lanes of a wave run in lockstep on the GPU, here they meet at a barrier.  Two sets of
 * slots in turn: a lane that is one exchange ahead writes the other set. */
inline const uint32_t* exchange(uint32_t v) {
    Workgroup* wg = workgroup();
    const unsigned p = t_parity++ & 1u;
    wg->exchange[wave()][p][lane()] = v;
    wave_barrier();
    return wg->exchange[wave()][p];
}

/* Runs `body` once per thread of every workgroup of the grid. */
inline void launch(dim3 grid, dim3 block, const std::function<void()>& body) {
    const unsigned threads = block.x * block.y * block.z;
    if (threads % kWave != 0 || threads / kWave > 16 || block.y != 1 || block.z != 1) std::abort();
    grid_dim() = grid;
    block_dim() = block;
    for (unsigned bz = 0; bz < grid.z; ++bz)
        for (unsigned by = 0; by < grid.y; ++by)
            for (unsigned bx = 0; bx < grid.x; ++bx) {
                Workgroup wg;
                wg.threads = threads;
                pthread_barrier_init(&wg.all, nullptr, threads);
                for (unsigned w = 0; w < threads / kWave; ++w) pthread_barrier_init(&wg.wave[w], nullptr, kWave);
                workgroup() = &wg;
                std::vector<std::thread> pool;
                pool.reserve(threads);
                for (unsigned t = 0; t < threads; ++t)
                    pool.emplace_back([&, t] {
                        t_thread_idx = dim3(t, 0, 0);
                        t_block_idx = dim3(bx, by, bz);
                        t_parity = 0;
                        body();
                    });
                for (auto& th : pool) th.join();
                for (unsigned w = 0; w < threads / kWave; ++w) pthread_barrier_destroy(&wg.wave[w]);
                pthread_barrier_destroy(&wg.all);
                workgroup() = nullptr;
            }
}

/* kernels launched through hipLaunchKernel (a function address and an array of argument
 * addresses) are registered with a function that unpacks the arguments */
inline std::map<const void*, std::function<void(void**)>>& registry() {
    static std::map<const void*, std::function<void(void**)>> r;
    return r;
}
/* every block of "device" memory that is alive: address -> bytes (what hipMalloc and
 * hipHostMalloc gave out, device symbols that were asked for, and what the harness adds) */
inline std::map<const void*, size_t>& regions() {
    static std::map<const void*, size_t> r;
    return r;
}
inline const void* symbol(const void* p, size_t n) {
    regions()[p] = n;
    return p;
}
/* called ahead of every hipLaunchKernel, if set (the harness can record the launch) */
inline std::function<void(const void*, dim3, dim3, void**)>& launch_observer() {
    static std::function<void(const void*, dim3, dim3, void**)> f;
    return f;
}

}  // namespace l3cpu

#define threadIdx (l3cpu::t_thread_idx)
#define blockIdx (l3cpu::t_block_idx)
#define blockDim (l3cpu::block_dim())
#define gridDim (l3cpu::grid_dim())

inline void __syncthreads() { l3cpu::workgroup_barrier(); }

inline uint32_t atomicOr(uint32_t* p, uint32_t v) { return __atomic_fetch_or(p, v, __ATOMIC_RELAXED); }
inline float __fdiv_rn(float a, float b) { return a / b; }
inline float __fsub_rn(float a, float b) { return a - b; }
inline uint32_t __float_as_uint(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}
inline uint32_t min(uint32_t a, uint32_t b) { return a < b ? a : b; }
inline uint32_t max(uint32_t a, uint32_t b) { return a > b ? a : b; }

/* ---- runtime -------------------------------------------------------------- */

typedef int hipError_t;
constexpr hipError_t hipSuccess = 0;
typedef struct l3cpu_stream* hipStream_t;
typedef struct l3cpu_event* hipEvent_t;
constexpr unsigned hipEventDisableTiming = 2, hipHostMallocDefault = 0;

inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipSetDevice(int) { return hipSuccess; }
inline hipError_t hipGetDeviceCount(int* n) { *n = 1; return hipSuccess; }
enum hipDeviceAttribute_t { hipDeviceAttributeMultiprocessorCount = 63 };
inline hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 1; return hipSuccess; }   /* one CU: launches of more than 8 workgroups have early rounds */
inline hipError_t hipMalloc(void** p, size_t n) {
    *p = std::malloc(n ? n : 1);
    if (*p) l3cpu::regions()[*p] = n;
    return *p ? hipSuccess : 2;
}
inline hipError_t hipFree(void* p) {
    l3cpu::regions().erase(p);
    std::free(p);
    return hipSuccess;
}
inline hipError_t hipHostMalloc(void** p, size_t n, unsigned) { return hipMalloc(p, n); }
inline hipError_t hipHostFree(void* p) { return hipFree(p); }
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
    *e = reinterpret_cast<hipEvent_t>(std::malloc(1));
    return hipSuccess;
}
inline hipError_t hipEventDestroy(hipEvent_t e) { std::free(e); return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }   /* launches are synchronous */
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
#define HIP_SYMBOL(x) l3cpu::symbol(&(x), sizeof(x))
inline hipError_t hipGetSymbolAddress(void** p, const void* symbol) {
    *p = const_cast<void*>(symbol);
    return hipSuccess;
}
inline hipError_t hipLaunchKernel(const void* kernel, dim3 grid, dim3 block, void** args, size_t, hipStream_t) {
    auto it = l3cpu::registry().find(kernel);
    if (it == l3cpu::registry().end()) return 98;
    if (l3cpu::launch_observer()) l3cpu::launch_observer()(kernel, grid, block, args);
    void** a = args;
    auto call = it->second;
    l3cpu::launch(grid, block, [call, a] { call(a); });
    return hipSuccess;
}
#define hipLaunchKernelGGL(kernel, grid, block, shared_bytes, stream, ...) \
    l3cpu::launch((grid), (block), [&] { kernel(__VA_ARGS__); })

#endif
