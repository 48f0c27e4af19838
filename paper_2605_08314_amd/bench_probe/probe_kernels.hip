// Measurement helpers of the benchmark -- NOT part of liblowrank.so and of no use to a caller of the library: a kernel
// that only streams a buffer (what a pure read of the size of a decode call achieves on the box: the practical ceiling
// next to the 8 TB/s nominal figure) and a plain copy (the kernel of known traffic against which the rocprofv3
// FETCH_SIZE / WRITE_SIZE counters are scaled).  Built into libbenchprobe.so, loaded by bench.py only.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

__global__ void __launch_bounds__(256) k_probe_read(const uint4* __restrict__ p, size_t n, uint32_t* sink) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 7 * stride < n; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n; i += stride) { const uint4 v = p[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9e3779b9u) sink[0] = acc;      // keeps the loads alive; practically never true
}

__global__ void __launch_bounds__(256) k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

extern "C" {

// src: device, 16-byte aligned, bytes a multiple of 16; sink: device word (practically never written).  0 on success.
int benchprobe_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || (((uintptr_t)src) & 15u) || (bytes & 15u)) return -1;
    if (bytes == 0) return 0;
    hipLaunchKernelGGL(k_probe_read, dim3(512), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

int benchprobe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!src || !dst || ((((uintptr_t)src) | ((uintptr_t)dst)) & 15u) || (bytes & 15u)) return -1;
    if (bytes == 0) return 0;
    hipLaunchKernelGGL(k_probe_copy, dim3(1024), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
