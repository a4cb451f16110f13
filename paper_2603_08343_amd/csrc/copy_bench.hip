// Bench-only shared object (libwht_copybench.so), not part of the layer's C ABI: a plain streaming
// copy with the access pattern of the layer's kernels (16 bytes per lane, non-temporal both ways).
// The benchmark uses it as the bandwidth a streaming kernel reaches on this GPU, and the profiling
// helper as a known-size reference for the profiler's HBM byte counters.
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
