// Decode attention over the dense KV cache (host-side declarations).
#pragma once
#include "lr_common.hpp"

namespace lr {

constexpr int kAttnMaxSplit = 32;     // workgroups that may share the cached positions of one (row, head)

// Workspace: header | rotated queries (8 bytes per element) | partial results of the shares.
struct AttnLayout {
    void* q_rot;                 // [M, H*E]: fp32 (fast path) or fp64 (generic path)
    float* part;                 // [M*H, kAttnMaxSplit, E + 2]: {max, sum, weighted V[E]}
};
size_t attn_ws_bytes(int64_t M, int64_t d, int64_t H);
AttnLayout attn_layout(void* ws, int64_t M, int64_t d, int64_t H);

// true: the MFMA-free fast kernel applies (bf16, head_dim 64 / 128 / 256, 16-byte aligned pointers)
bool attn_fast_ok(int dtype, int64_t E, bool aligned);

int attn_decode(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base, int dtype,
                bool fast, void* ws, hipStream_t s);

// Prefill attention (attention_prefill.hip): bf16, head_dim 128, 16-byte aligned operands.
bool attn_prefill_ok(int dtype, int64_t E, bool aligned);
// q != NULL: dense queries; q == NULL: factorized queries q = tq vq (+ bq), tq [M, r_q], vq [r_q, H * 128], r_q a multiple of 64
int attn_prefill(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base, hipStream_t s,
                 const void* tq = nullptr, const void* vq = nullptr, const void* bq = nullptr, int64_t r_q = 0);

}  // namespace lr
