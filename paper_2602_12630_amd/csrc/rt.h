/*
 * Thin runtime layer under the library: device memory, copies, kernel launch.
 *
 * The product build (hipcc, gfx950) maps these onto HIP: every kernel is a
 * functor `F` with `void operator()(uint32_t lane) const` launched as
 * `kernel<F, BLOCK>` over `n` lanes on the context's stream.
 *
 * With -DTC_HOST_EMU the same functors are executed lane by lane on the host.
 * That build exists only so that the CPU test-suite and a debugger can walk
 * the library's host logic (sorting passes, level loops, buffer sizes) without
 * a GPU.  The Python binding never loads it; the product library has no CPU
 * path.
 */
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>

namespace tc {
namespace rt {
/* every allocation or release of device or pinned host memory that the library asks the runtime for */
inline std::atomic<uint64_t>& alloc_calls() {
    static std::atomic<uint64_t> n{0};
    return n;
}
}  // namespace rt
}  // namespace tc

#if defined(TC_HOST_EMU)

namespace tc {
namespace rt {
typedef void* stream_t;
inline int dev_malloc(void** p, size_t n) { ++alloc_calls(); *p = malloc(n ? n : 1); return *p ? 0 : 2; }
inline int dev_free(void* p) { ++alloc_calls(); free(p); return 0; }
inline int host_pinned_malloc(void** p, size_t n) { ++alloc_calls(); *p = malloc(n ? n : 1); return *p ? 0 : 2; }
inline int host_pinned_free(void* p) { ++alloc_calls(); free(p); return 0; }
inline int memcpy_h2d(void* d, const void* s, size_t n, stream_t) { memcpy(d, s, n); return 0; }
inline int memcpy_d2h(void* d, const void* s, size_t n, stream_t) { memcpy(d, s, n); return 0; }
inline int memcpy_d2d(void* d, const void* s, size_t n, stream_t) { memmove(d, s, n); return 0; }
inline int memset_async(void* d, int v, size_t n, stream_t) { memset(d, v, n); return 0; }
inline int stream_sync(stream_t) { return 0; }
inline int set_device(int) { return 0; }
typedef void* event_t;
inline int event_create(event_t* e) { *e = nullptr; return 0; }
inline int event_record(event_t, stream_t) { return 0; }
inline int event_elapsed_ms(event_t, event_t, float* ms) { *ms = 0.0f; return 0; }
inline void event_destroy(event_t) {}
inline int last_error() { return 0; }
inline const char* error_string(int) { return "host emulation"; }
template <int BLOCK, class F>
inline int launch(uint64_t n, stream_t, const F& f) {
    for (uint64_t t = 0; t < n; ++t) f((uint32_t)t);
    return 0;
}
template <int BLOCK, int WAVES, class F>
inline int launch_waves(uint64_t n, stream_t st, const F& f) {
    return launch<BLOCK>(n, st, f);
}
}  // namespace rt
inline uint32_t atomic_add_u32(uint32_t* p, uint32_t v) { uint32_t o = *p; *p += v; return o; }
inline uint32_t atomic_and_u32(uint32_t* p, uint32_t v) { uint32_t o = *p; *p &= v; return o; }
inline uint32_t atomic_max_u32(uint32_t* p, uint32_t v) { uint32_t o = *p; if (v > o) *p = v; return o; }
}  // namespace tc

#else

#include <hip/hip_runtime.h>

namespace tc {

template <class F, int BLOCK>
__global__ __launch_bounds__(BLOCK) void kernel(const F f, uint32_t n) {
    uint32_t t = blockIdx.x * BLOCK + threadIdx.x;
    if (t < n) f(t);
}

/* the same with the register budget of exactly WAVES waves per SIMD: a kernel that is one long stretch of
 * straight-line arithmetic, where the compiler's own choice trades registers for spills */
template <class F, int BLOCK, int WAVES>
__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES))) void kernel_waves(const F f, uint32_t n) {
    uint32_t t = blockIdx.x * BLOCK + threadIdx.x;
    if (t < n) f(t);
}

namespace rt {
typedef hipStream_t stream_t;
inline int dev_malloc(void** p, size_t n) { ++alloc_calls(); return (int)hipMalloc(p, n ? n : 1); }
inline int dev_free(void* p) { ++alloc_calls(); return (int)hipFree(p); }
inline int host_pinned_malloc(void** p, size_t n) { ++alloc_calls(); return (int)hipHostMalloc(p, n ? n : 1, hipHostMallocDefault); }
inline int host_pinned_free(void* p) { ++alloc_calls(); return (int)hipHostFree(p); }
inline int memcpy_h2d(void* d, const void* s, size_t n, stream_t st) { return (int)hipMemcpyAsync(d, s, n, hipMemcpyHostToDevice, st); }
inline int memcpy_d2h(void* d, const void* s, size_t n, stream_t st) { return (int)hipMemcpyAsync(d, s, n, hipMemcpyDeviceToHost, st); }
inline int memcpy_d2d(void* d, const void* s, size_t n, stream_t st) { return (int)hipMemcpyAsync(d, s, n, hipMemcpyDeviceToDevice, st); }
inline int memset_async(void* d, int v, size_t n, stream_t st) { return (int)hipMemsetAsync(d, v, n, st); }
inline int stream_sync(stream_t st) { return (int)hipStreamSynchronize(st); }
inline int set_device(int dev) { return (int)hipSetDevice(dev); }
typedef hipEvent_t event_t;
inline int event_create(event_t* e) { return (int)hipEventCreate(e); }
inline int event_record(event_t e, stream_t st) { return (int)hipEventRecord(e, st); }
inline int event_elapsed_ms(event_t a, event_t b, float* ms) {
    int e = (int)hipEventSynchronize(b);
    return e ? e : (int)hipEventElapsedTime(ms, a, b);
}
inline void event_destroy(event_t e) { (void)hipEventDestroy(e); }
inline int last_error() { return (int)hipGetLastError(); }
inline const char* error_string(int e) { return hipGetErrorString((hipError_t)e); }
template <int BLOCK, class F>
inline int launch(uint64_t n, stream_t st, const F& f) {
    if (n == 0) return 0;
    if (n > 0xFFFFFFFFull) return (int)hipErrorInvalidValue;
    uint32_t blocks = (uint32_t)((n + BLOCK - 1) / BLOCK);
    hipLaunchKernelGGL((kernel<F, BLOCK>), dim3(blocks), dim3(BLOCK), 0, st, f, (uint32_t)n);
    return (int)hipGetLastError();
}
template <int BLOCK, int WAVES, class F>
inline int launch_waves(uint64_t n, stream_t st, const F& f) {
    if (n == 0) return 0;
    if (n > 0xFFFFFFFFull) return (int)hipErrorInvalidValue;
    uint32_t blocks = (uint32_t)((n + BLOCK - 1) / BLOCK);
    hipLaunchKernelGGL((kernel_waves<F, BLOCK, WAVES>), dim3(blocks), dim3(BLOCK), 0, st, f, (uint32_t)n);
    return (int)hipGetLastError();
}
}  // namespace rt
__device__ __forceinline__ uint32_t atomic_add_u32(uint32_t* p, uint32_t v) { return atomicAdd(p, v); }
__device__ __forceinline__ uint32_t atomic_and_u32(uint32_t* p, uint32_t v) { return atomicAnd(p, v); }
__device__ __forceinline__ uint32_t atomic_max_u32(uint32_t* p, uint32_t v) { return atomicMax(p, v); }
}  // namespace tc

#endif

#if defined(__HIPCC__)
#define TC_DEV __device__ __forceinline__
#else
#define TC_DEV inline
#endif
