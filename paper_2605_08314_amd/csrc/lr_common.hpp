// Shared declarations of the HIP library: error reporting, element-type traits, workspace
// layout and the launcher prototypes of the kernel families.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "lowrank.h"

namespace lr {

// ---- host-side error reporting (thread-local message behind lowrank_last_error) -------------
void set_error(const char* fmt, ...);
int launch_status(const char* what);   // hipGetLastError -> LR_OK / LR_ERR_LAUNCH

// ---- element types ---------------------------------------------------------------------------
typedef uint16_t bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round-to-nearest-even fp32 -> bf16; NaN stays NaN (quiet), infinities are preserved.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

struct IoF32 {
    typedef float T;
    typedef double Acc;     // generic fp32 path accumulates in fp64 so that long reductions keep 1e-5
    static constexpr int dtype = LR_F32;
    __device__ static __forceinline__ float ld(const T* p) { return *p; }
    __device__ static __forceinline__ T cvt(float v) { return v; }
};
struct IoBF16 {
    typedef bf16_t T;
    typedef float Acc;
    static constexpr int dtype = LR_BF16;
    __device__ static __forceinline__ float ld(const T* p) { return bf16_to_f32(*p); }
    __device__ static __forceinline__ T cvt(float v) { return f32_to_bf16(v); }
};

__device__ __forceinline__ float silu_f32(float z) {
    // z * sigmoid(z); __expf(-z) overflows to +inf for z < -88 and the quotient is then -0, the
    // correctly rounded limit.
    return z / (1.0f + __expf(-z));
}

// The same for results that are rounded to bf16 right away: hardware exp2 and reciprocal (1 ulp each)
// instead of the IEEE division sequence -- 5 instructions per element.  exp2 overflows to +inf for
// z < -128 and rcp(inf) = 0, so the limit is again -0.
__device__ __forceinline__ float silu_bf16out(float z) {
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z * -1.4426950408889634f));
}

// ---- dense KV-cache scatter description (device copy of lr_kv_target, one cache) -------------
struct CacheDst {
    void* cache;            // NULL: no scatter
    const int32_t* pos;     // device int32[B]
    int64_t S_max;
    int64_t T;              // tokens per sequence
};

// ---- workspace layout --------------------------------------------------------------------------
// [0, kHeaderBytes)   control block (epoch, error flag, barrier counters), zero when prepared
// then fp32 areas, each 256-byte aligned, carved by the entry points.
constexpr size_t kHeaderBytes = 16384;
__host__ __device__ inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Dims { int64_t M, d_in, r, d_out; };

// ---- generic (any shape, any alignment, both dtypes) -----------------------------------------
// t[M, R] (fp32, leading dim ldt) = x[M, K] * U[K, R]; x element type = dtype, or fp32 if x_is_f32.
int generic_stage1(const void* x, bool x_is_f32, const void* U, float* t, int64_t ldt,
                   int64_t M, int64_t K, int64_t R, int dtype, hipStream_t s);
// y[M, N] = t[M, r] * V[r, N] + bias, rounded to dtype; y may be NULL; optional cache scatter.
int generic_stage2(const float* t, int64_t ldt, const void* V, const void* bias, void* y,
                   int64_t M, int64_t r, int64_t N, CacheDst cd, int dtype, hipStream_t s);
// h[M, ffn] (fp32) = SiLU(tg*V_g + b_g) .* (tu*V_u + b_u); tg = t[:, :r_g], tu = t[:, r_g:].
int generic_gateup(const float* t, int64_t ldt, const void* V_g, const void* V_u, const void* b_g,
                   const void* b_u, float* h, int64_t M, int64_t r_g, int64_t r_u, int64_t ffn,
                   int dtype, hipStream_t s);
int generic_pack_concat(const void* const* U_list, const int64_t* r_list, int n, int64_t d_in,
                        int elem_bytes, void* packed, hipStream_t s);
int generic_pack_panels(const void* W, int64_t K, int64_t N, void* panels, hipStream_t s);   // bf16 [K, N] -> 64-column panels
int fill_zero(void* p, size_t bytes, hipStream_t s);
int generic_round(const float* src, void* dst, int64_t n, int dtype, hipStream_t s);

}  // namespace lr
