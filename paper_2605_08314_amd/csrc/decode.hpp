// Decode-phase launch descriptors shared by the host planner and the kernels.
#pragma once
#include "lr_common.hpp"

namespace lr {

enum { EPI_ATOMIC = 0, EPI_STORE = 1, EPI_GATEUP = 2 };
constexpr int kMaxProb = 8;

// One skinny product handled inside a stage: C[M, N] (+)= A[M, K] * W[K, N] (W row-major, ld = N).
struct DProb {
    const bf16_t* W;  const void* A;  int K;  int lda;      // first matrix and its activation rows
    const bf16_t* W2; const void* A2; int K2; int lda2;     // second matrix (EPI_GATEUP: up branch)
    int N;
    float* C; int ldc;                                      // EPI_ATOMIC: fp32 accumulator
    bf16_t* Y;                                              // EPI_STORE / EPI_GATEUP: bf16 output [M, N] (nullable for STORE)
    const bf16_t* bias; const bf16_t* bias2;
    void* cache; const int32_t* pos; int S_max; int T;      // EPI_STORE: optional dense-cache scatter
    int tiles_n;      // column tiles (N / NC)
    int KS;           // rows of W per tile (multiple of 32); tiles along K = ceil(K / KS)
    int tile_begin;   // first tile index of this product inside the stage
};

struct DStage {
    DProb p[kMaxProb];
    int nprob;
    int M;
    int total_tiles;
};

// Launch one stage: cpl = bf16 columns per lane (4 or 8), a_f32 = activations are fp32 (rank-space
// accumulators) rather than bf16, epi = EPI_*.
int decode_launch_stage(const DStage& st, int cpl, bool a_f32, int epi, hipStream_t s);

// Host planners (decode_plan.hip).  They assume decode_shape_ok(...) held for every product.
bool decode_shape_ok(int64_t M, int64_t K, int64_t N);
int decode_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                  int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, hipStream_t s);
int decode_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
               void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
               const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
               void* ws, hipStream_t s);
int decode_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
               const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
               int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
               void* ws, hipStream_t s);

}  // namespace lr
