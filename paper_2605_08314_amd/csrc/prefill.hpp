// Prefill-phase launch descriptors (hundreds to thousands of token rows, bf16, MFMA-bound).
#pragma once
#include "lr_common.hpp"

namespace lr {

enum { PEPI_STORE = 0, PEPI_GATEUP = 1, PEPI_PARTIAL = 2 };     // PARTIAL: fp32 partial sums of a K chunk to P.Cf (no bias, no cache)
constexpr int kMaxPProb = 16;

// One dense product C[M, N] = A[M, K] * B[K, N] (+ epilogue); A, B, C row-major bf16.
struct PProb {
    const bf16_t* A;  int lda;  const bf16_t* B;  int K;    // B has leading dimension N
    const bf16_t* A2; int lda2; const bf16_t* B2; int K2;   // PEPI_GATEUP: the up-branch product
    int N;
    bf16_t* C; int ldc;                                     // nullable for STORE when only the cache is wanted
    float* Cf;                                              // PEPI_PARTIAL: fp32 output [M, ldc]
    const bf16_t* bias; const bf16_t* bias2;
    void* cache; const int32_t* pos; int S_max; int T;      // optional dense-cache scatter of the rows of C
};

struct PArgs {
    PProb p[kMaxPProb];
    int nprob;
    int M;
    int tiles_m;        // ceil(M / BM)
    int tiles_n_max;    // max over problems of ceil(N / BN)
    int group_m;        // tile rows per L2 group of the tile order
    unsigned long long* trace;   // timeline buffer of trace builds, else NULL
    // products whose K range is shared between workgroups: flags, fp32 partial-tile slots, error word
    uint32_t* sk_flags; float* sk_slots; uint32_t* err;
    int sk;             // 1: the launch walks k-step ranges, not tiles
    int sk_nk;          // k-steps (of 32) per tile in that case
    uint32_t sk_spin_limit;   // polls after which the holder of a shared tile stops waiting for a partial sum
};

bool prefill_shape_ok(int64_t M, int64_t K, int64_t N);
int prefill_launch(const PArgs& a, int epi, hipStream_t s);
void prefill_plan_query(int64_t M, int64_t K, int64_t N, int n, bool gateup, int* bm, int* bn, int* share_k);

int prefill_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                   int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, size_t ws_bytes, hipStream_t s);
int prefill_rank_project(const void* x, const void* U, void* t, int64_t M, int64_t d_in, int64_t r,
                         void* ws, size_t ws_bytes, hipStream_t s);
int prefill_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
                void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
                const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
                void* ws, size_t ws_bytes, hipStream_t s);
int prefill_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
                const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
                int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
                void* ws, size_t ws_bytes, hipStream_t s);

}  // namespace lr
