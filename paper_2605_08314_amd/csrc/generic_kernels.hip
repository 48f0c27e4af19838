// Generic kernels: one thread per output element, plain loops.  They accept any shape and any
// alignment in both element types and are the fallback under the tuned decode / prefill
// kernels.  fp32 calls accumulate in fp64, bf16 calls in fp32.
#include "lr_common.hpp"
#include "decode.hpp"

namespace lr {

template <class IO, class TIn>
__global__ void __launch_bounds__(256)
k_gen_stage1(const TIn* __restrict__ x, const typename IO::T* __restrict__ U, float* __restrict__ t,
             int64_t ldt, int64_t M, int64_t K, int64_t R) {
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= R) return;
    for (int64_t m = blockIdx.y; m < M; m += gridDim.y) {
        typename IO::Acc acc = 0;
        const TIn* xr = x + m * K;
        for (int64_t k = 0; k < K; ++k) {
            float xv;
            if constexpr (sizeof(TIn) == 4) xv = (float)xr[k]; else xv = bf16_to_f32((bf16_t)xr[k]);
            acc += (typename IO::Acc)xv * (typename IO::Acc)IO::ld(U + k * R + j);
        }
        t[m * ldt + j] = (float)acc;
    }
}

template <class IO>
__global__ void __launch_bounds__(256)
k_gen_stage2(const float* __restrict__ t, int64_t ldt, const typename IO::T* __restrict__ V,
             const typename IO::T* __restrict__ bias, typename IO::T* __restrict__ y,
             int64_t M, int64_t r, int64_t N, CacheDst cd) {
    const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    for (int64_t m = blockIdx.y; m < M; m += gridDim.y) {
        typename IO::Acc acc = 0;
        const float* tr = t + m * ldt;
        for (int64_t j = 0; j < r; ++j)
            acc += (typename IO::Acc)tr[j] * (typename IO::Acc)IO::ld(V + j * N + n);
        if (bias) acc += (typename IO::Acc)IO::ld(bias + n);
        const typename IO::T o = IO::cvt((float)acc);
        if (y) y[m * N + n] = o;
        if (cd.cache) {
            const int64_t b = m / cd.T, s = m % cd.T;
            const int64_t p = (int64_t)cd.pos[b] + s;
            if (p >= 0 && p < cd.S_max)
                ((typename IO::T*)cd.cache)[(b * cd.S_max + p) * N + n] = o;
        }
    }
}

template <class IO>
__global__ void __launch_bounds__(256)
k_gen_gateup(const float* __restrict__ t, int64_t ldt, const typename IO::T* __restrict__ V_g,
             const typename IO::T* __restrict__ V_u, const typename IO::T* __restrict__ b_g,
             const typename IO::T* __restrict__ b_u, float* __restrict__ h,
             int64_t M, int64_t r_g, int64_t r_u, int64_t ffn) {
    const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (f >= ffn) return;
    for (int64_t m = blockIdx.y; m < M; m += gridDim.y) {
        typename IO::Acc g = 0, u = 0;
        const float* tr = t + m * ldt;
        for (int64_t j = 0; j < r_g; ++j) g += (typename IO::Acc)tr[j] * (typename IO::Acc)IO::ld(V_g + j * ffn + f);
        for (int64_t j = 0; j < r_u; ++j) u += (typename IO::Acc)tr[r_g + j] * (typename IO::Acc)IO::ld(V_u + j * ffn + f);
        if (b_g) g += (typename IO::Acc)IO::ld(b_g + f);
        if (b_u) u += (typename IO::Acc)IO::ld(b_u + f);
        h[m * ffn + f] = silu_f32((float)g) * (float)u;
    }
}

__global__ void __launch_bounds__(256)
k_pack_copy(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst,
            int64_t rows, int64_t src_row_bytes, int64_t dst_row_bytes, int64_t dst_col_bytes) {
    const int64_t total = rows * src_row_bytes;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t k = i / src_row_bytes, c = i % src_row_bytes;
        dst[k * dst_row_bytes + dst_col_bytes + c] = src[i];
    }
}

__global__ void __launch_bounds__(256) k_fill_zero(uint32_t* p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

static inline dim3 grid2(int64_t cols, int64_t rows) {
    return dim3((unsigned)((cols + 255) / 256), (unsigned)(rows < 4096 ? (rows < 1 ? 1 : rows) : 4096), 1);
}

int generic_stage1(const void* x, bool x_is_f32, const void* U, float* t, int64_t ldt,
                   int64_t M, int64_t K, int64_t R, int dtype, hipStream_t s) {
    if (M <= 0 || R <= 0) return LR_OK;
    dim3 g = grid2(R, M);
    if (dtype == LR_F32)
        hipLaunchKernelGGL((k_gen_stage1<IoF32, float>), g, dim3(256), 0, s, (const float*)x, (const float*)U, t, ldt, M, K, R);
    else if (x_is_f32)
        hipLaunchKernelGGL((k_gen_stage1<IoBF16, float>), g, dim3(256), 0, s, (const float*)x, (const bf16_t*)U, t, ldt, M, K, R);
    else
        hipLaunchKernelGGL((k_gen_stage1<IoBF16, bf16_t>), g, dim3(256), 0, s, (const bf16_t*)x, (const bf16_t*)U, t, ldt, M, K, R);
    return launch_status("generic stage 1");
}

int generic_stage2(const float* t, int64_t ldt, const void* V, const void* bias, void* y,
                   int64_t M, int64_t r, int64_t N, CacheDst cd, int dtype, hipStream_t s) {
    if (M <= 0 || N <= 0) return LR_OK;
    dim3 g = grid2(N, M);
    if (dtype == LR_F32)
        hipLaunchKernelGGL((k_gen_stage2<IoF32>), g, dim3(256), 0, s, t, ldt, (const float*)V, (const float*)bias, (float*)y, M, r, N, cd);
    else
        hipLaunchKernelGGL((k_gen_stage2<IoBF16>), g, dim3(256), 0, s, t, ldt, (const bf16_t*)V, (const bf16_t*)bias, (bf16_t*)y, M, r, N, cd);
    return launch_status("generic stage 2");
}

int generic_gateup(const float* t, int64_t ldt, const void* V_g, const void* V_u, const void* b_g,
                   const void* b_u, float* h, int64_t M, int64_t r_g, int64_t r_u, int64_t ffn,
                   int dtype, hipStream_t s) {
    if (M <= 0 || ffn <= 0) return LR_OK;
    dim3 g = grid2(ffn, M);
    if (dtype == LR_F32)
        hipLaunchKernelGGL((k_gen_gateup<IoF32>), g, dim3(256), 0, s, t, ldt, (const float*)V_g, (const float*)V_u,
                           (const float*)b_g, (const float*)b_u, h, M, r_g, r_u, ffn);
    else
        hipLaunchKernelGGL((k_gen_gateup<IoBF16>), g, dim3(256), 0, s, t, ldt, (const bf16_t*)V_g, (const bf16_t*)V_u,
                           (const bf16_t*)b_g, (const bf16_t*)b_u, h, M, r_g, r_u, ffn);
    return launch_status("generic gate/up");
}

int generic_pack_concat(const void* const* U_list, const int64_t* r_list, int n, int64_t d_in,
                        int elem_bytes, void* packed, hipStream_t s) {
    int64_t R = 0;
    for (int i = 0; i < n; ++i) R += r_list[i];
    int64_t col = 0;
    for (int i = 0; i < n; ++i) {
        const int64_t bytes = d_in * r_list[i] * elem_bytes;
        if (bytes > 0) {
            int64_t blocks = (bytes + 255) / 256;
            if (blocks > 8192) blocks = 8192;
            hipLaunchKernelGGL(k_pack_copy, dim3((unsigned)blocks), dim3(256), 0, s, (const unsigned char*)U_list[i],
                               (unsigned char*)packed, d_in, r_list[i] * elem_bytes, R * elem_bytes, col * elem_bytes);
            int st = launch_status("pack concat");
            if (st != LR_OK) return st;
        }
        col += r_list[i];
    }
    return LR_OK;
}

// 64-column panels of a row-major bf16 matrix [K, N]: element (k, n) goes to ((n / 64) * K + k) * 64 + n % 64.
// One thread per 16-byte unit (8 columns); a panel row is 128 bytes, so reads and writes are whole 128-byte segments.
__global__ void __launch_bounds__(256) k_pack_panels(const uint4* __restrict__ W, uint4* __restrict__ P, int64_t K, int64_t N) {
    const int64_t units_per_row = N / 8, total = K * units_per_row;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t k = i / units_per_row, u = i - k * units_per_row;      // unit u of row k
        const int64_t panel = u >> 3, pu = u & 7;
        P[(panel * K + k) * 8 + pu] = W[i];
    }
}

int generic_pack_panels(const void* W, int64_t K, int64_t N, void* panels, hipStream_t s) {
    const int64_t total = K * (N / 8);
    if (total <= 0) return LR_OK;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_pack_panels, dim3((unsigned)blocks), dim3(256), 0, s, (const uint4*)W, (uint4*)panels, K, N);
    return launch_status("pack panels");
}

// Check-and-prepare for launches that keep state in the workspace without being a fused decode kernel (the prefill product
// that shares K, lowrank_workspace_init): ONE small launch.  When the control block carries the ready word (every call but
// the first) the single workgroup leaves at once; otherwise it zeroes the control block, the flags and the accumulator areas
// (8 MiB by 1024 threads: some tens of microseconds, once) and then writes the word.  Nothing is copied back, nothing waits.
__global__ void __launch_bounds__(1024) k_ws_prepare(char* ws) {
    Ctrl* c = reinterpret_cast<Ctrl*>(ws);
    if (__hip_atomic_load(&c->magic, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == kCtrlReady) return;
    uint2* head = reinterpret_cast<uint2*>(ws) + 1;                               // behind the magic word
    const size_t n_head = (kHeaderBytes + kSkFlagBytes) / 8 - 1;
    uint4* acc = reinterpret_cast<uint4*>(ws + kHeaderBytes + kSkFlagBytes + kDecPartBytes);
    const size_t n_acc = 2 * kAccBytes / 16;
    for (size_t i = threadIdx.x; i < n_head; i += 1024) head[i] = make_uint2(0u, 0u);
    for (size_t i = threadIdx.x; i < n_acc; i += 1024) acc[i] = make_uint4(0u, 0u, 0u, 0u);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");                             // the zeroes are in memory before the word says so
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(&c->magic, kCtrlReady, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

int ws_prepare(void* ws, hipStream_t s) {
    hipLaunchKernelGGL(k_ws_prepare, dim3(1), dim3(1024), 0, s, (char*)ws);
    return launch_status("workspace preparation");
}

template <class IO>
__global__ void __launch_bounds__(256) k_gen_round(const float* __restrict__ src, typename IO::T* __restrict__ dst, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = IO::cvt(src[i]);
}

// dst[i] = src[i] rounded to dtype (nearest-even)
int generic_round(const float* src, void* dst, int64_t n, int dtype, hipStream_t s) {
    if (n <= 0) return LR_OK;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (dtype == LR_F32) hipLaunchKernelGGL((k_gen_round<IoF32>), dim3((unsigned)blocks), dim3(256), 0, s, src, (float*)dst, n);
    else hipLaunchKernelGGL((k_gen_round<IoBF16>), dim3((unsigned)blocks), dim3(256), 0, s, src, (bf16_t*)dst, n);
    return launch_status("generic round");
}

int fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return LR_OK;
    size_t words = bytes / 4;   // callers pass multiples of 4
    size_t blocks = (words + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)blocks), dim3(256), 0, s, (uint32_t*)p, words);
    return launch_status("fill");
}

}  // namespace lr
