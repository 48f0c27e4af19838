// Measurement helpers behind lowrank_probe_read / lowrank_probe_copy: a plain streaming read and a
// plain copy.  The benchmark uses the read to report what a kernel that does nothing but stream a
// buffer of the same size achieves on the box (the practical ceiling next to the 8 TB/s nominal
// figure); the copy is the kernel of known traffic against which the rocprofv3 FETCH_SIZE / WRITE_SIZE
// counters are scaled.
#include "lr_common.hpp"

namespace lr {

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

}  // namespace lr

using namespace lr;

extern "C" {

int lowrank_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink) { set_error("NULL operand"); return LR_ERR_NULL; }
    if ((((uintptr_t)src) & 15u) || (bytes & 15u)) { set_error("probe buffers must be 16-byte multiples"); return LR_ERR_ALIGN; }
    if (bytes == 0) return LR_OK;
    hipLaunchKernelGGL(k_probe_read, dim3(512), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16, (uint32_t*)sink);
    return launch_status("probe read");
}

int lowrank_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!src || !dst) { set_error("NULL operand"); return LR_ERR_NULL; }
    if ((((uintptr_t)src | (uintptr_t)dst) & 15u) || (bytes & 15u)) { set_error("probe buffers must be 16-byte multiples"); return LR_ERR_ALIGN; }
    if (bytes == 0) return LR_OK;
    hipLaunchKernelGGL(k_probe_copy, dim3(1024), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
    return launch_status("probe copy");
}

}  // extern "C"
