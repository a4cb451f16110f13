// Bench-only shared object (libwht_copybench.so), not part of the layer's C ABI: a plain streaming
// copy with the access pattern of the layer's kernels (16 bytes per lane, non-temporal both ways)
// and an empty kernel.  The benchmark uses the copy as the bandwidth a streaming kernel reaches on
// this GPU and, at the decode shapes, both as the latency floor of a call; the profiling helper
// uses the copy as a known-size reference for the profiler's HBM byte counters.  Also timing events
// without the system-scope fence, for timing single launches inside a series of launches.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    for (size_t base = ((size_t)blockIdx.x * blockDim.x) * 4 + threadIdx.x; base < nvec; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (base + k * 256 < nvec) v[k] = __builtin_nontemporal_load(src + base + k * 256);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (base + k * 256 < nvec) __builtin_nontemporal_store(v[k], dst + base + k * 256);
    }
}

__global__ void empty_kernel() {}

// One launch of a kernel that does nothing: the per-call floor of the launch path on `stream`.
extern "C" int wht_bench_empty(void* stream) {
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Shader clock now: counts of the shader-clock counter and of the constant 100 MHz counter over a
// short spin, written to out[0], out[1] (device memory, two uint64).  MHz = 100 * out[0] / out[1].
__global__ void clock_probe_kernel(unsigned long long* out) {
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    float v = (float)threadIdx.x;
    for (int i = 0; i < 2000; ++i) v = v * 1.0001f + 0.5f;
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    if (threadIdx.x == 0) { out[0] = c1 - c0 + (v == 12345.678f); out[1] = r1 - r0; }
}
extern "C" int wht_bench_clock_probe(void* out, void* stream) {
    if (!out) return 1;
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       static_cast<unsigned long long*>(out));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// dst[i] = src[i] for `bytes` bytes (a multiple of 16); device pointers, 16-byte aligned, not
// overlapping; enqueued on `stream`.  Returns 0, or 1 for bad arguments, 2 if the launch failed.
extern "C" int wht_bench_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || bytes % 16 != 0 || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return 1;
    if (bytes == 0) return 0;
    const size_t nvec = bytes / 16;
    const size_t want = (nvec + 1023) / 1024;
    const size_t cap = (size_t)256 * 64;                 // 256 CUs
    const int grid = (int)(want < cap ? want : cap);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), nvec);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Timing events created with hipEventDisableSystemFence.  An event record is work on the stream: with
// the default flags two records with nothing between them complete 4.5 us apart and a pair around
// every launch adds 8 us per launch to a series of kernels; without the system-scope fence the
// figures are 3.3 us and 4.6 us, and the interval around a 100 us kernel reads 0.9 us more than the
// kernel takes (default: 2.8 us).  Measured on MI355X.
extern "C" void* wht_bench_event_create(void) {
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
    return e;
}
extern "C" int wht_bench_event_record(void* event, void* stream) {
    return hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)) == hipSuccess ? 0 : 2;
}
// Milliseconds from `start` to `stop` (both recorded and complete), negative on error.
extern "C" float wht_bench_event_elapsed_ms(void* start, void* stop) {
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, static_cast<hipEvent_t>(start), static_cast<hipEvent_t>(stop)) != hipSuccess) return -1.0f;
    return ms;
}
extern "C" int wht_bench_event_destroy(void* event) {
    return hipEventDestroy(static_cast<hipEvent_t>(event)) == hipSuccess ? 0 : 2;
}
