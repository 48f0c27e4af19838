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
    float* part;      // EPI_ATOMIC with bf16 finalisation: fp32 partial tiles, one slot of 16*MB x NC floats per tile of the stage
    int ldy;          // EPI_ATOMIC with bf16 finalisation: row stride of Y (the bf16 copy of the accumulator)
    int ctile_begin;  // EPI_ATOMIC with bf16 finalisation: index of this product's first column-tile counter
    int tiles_n;      // column tiles (N / NC)
    int KS;           // rows of W per tile (multiple of 32); tiles along K = ceil(K / KS)
    int tile_begin;   // first tile index of this product inside the stage
};

template <int NP> struct DStageT { DProb p[NP]; int nprob, M, total_tiles; };
typedef DStageT<kMaxProb> DStage;

// Control block at the start of every workspace (zero when prepared).  A stage barrier is kSlots
// counters on separate 128-byte lines: workgroup w adds 1 to slot w % kSlots, a waiting wave reads
// all slots with one load instruction.  One hot counter for 256 workgroups costs several
// microseconds per barrier on this chip; sixteen cool ones cost about one.
constexpr int kBarriers = 3;
constexpr int kSlots = 16;
constexpr int kSlotStride = 32;   // uint32 words between slots (128 bytes)
constexpr int kTileCounters = 256;
struct Ctrl {
    uint32_t epoch;                     // number of fused calls completed on this workspace
    uint32_t error;                     // nonzero: a bounded device-side wait gave up
    uint32_t dirty[2];                  // floats of accumulator area p that are not zero
    uint32_t pad[28];
    uint32_t cnt[2][kBarriers][kSlots * kSlotStride];   // [epoch parity][barrier][slot]
    uint32_t tcnt[2][kTileCounters];                    // arrivals per accumulator column tile (bf16 finalisation)
};
static_assert(sizeof(Ctrl) <= kHeaderBytes, "control block must fit the workspace header");

// Tail of a workspace that may serve a prefill call (more than 32 token rows): flags and fp32 partial
// tiles of products whose K range is shared between workgroups (256 slots of one 256 x 256 tile, or
// 512 of 128 x 128).  Zero when prepared; every call leaves the flags zero.
constexpr size_t kSkFlagBytes = 4096;
constexpr size_t kSkSlotBytes = (size_t)256 * 256 * 256 * 4;
constexpr size_t kSkBytes = kSkFlagBytes + kSkSlotBytes;
// Tail of a decode workspace for 9..32 token rows: fp32 partial tiles of the split-K stages (one slot per
// workgroup tile; the last K-slice of a column tile to arrive adds them up in slice order and writes bf16).
constexpr size_t kDecPartBytes = (size_t)8 << 20;
// More token rows than this may use split-K partial tiles in slots + bf16 finalisation instead of atomics (the packed MLP
// does from 9 rows on, the two-stage calls from 25: measured cross-over points), so the workspace has the tail for them.
constexpr int kT16Rows = 8;
inline size_t sk_tail_bytes(int64_t M) { return M > 32 ? kSkBytes : (M > kT16Rows ? kDecPartBytes : 0); }

// Where the parts of a workspace of `ws_bytes` bytes for M token rows sit:
// header | acc area 0 | acc area 1 | staging | tail (decode partial tiles for 8 < M <= 32, shared-K area for M > 32).
struct WsLayout {
    Ctrl* ctrl; char* acc0; size_t acc_bytes; char* staging; size_t staging_bytes;
    uint32_t* sk_flags; float* sk_slots;       // prefill tail (M > 32), else NULL
    float* dec_part;                           // decode partial tiles (8 < M <= 32), else NULL
};
inline WsLayout ws_layout(void* ws, size_t ws_bytes, int64_t M) {
    WsLayout L;
    const size_t tail = sk_tail_bytes(M);
    const size_t body = ws_bytes - tail;
    L.ctrl = (Ctrl*)ws;
    L.acc_bytes = ((body - kHeaderBytes) / 4) & ~(size_t)255;
    L.acc0 = (char*)ws + kHeaderBytes;
    L.staging = L.acc0 + 2 * L.acc_bytes;
    L.staging_bytes = body - kHeaderBytes - 2 * L.acc_bytes;
    char* t = (char*)ws + (body & ~(size_t)255);
    L.sk_flags = M > 32 ? (uint32_t*)t : nullptr;
    L.sk_slots = M > 32 ? (float*)(t + kSkFlagBytes) : nullptr;
    L.dec_part = (M > kT16Rows && M <= 32) ? (float*)t : nullptr;
    return L;
}

struct FusedCommon {
    Ctrl* ctrl;
    char* acc0;              // accumulator area 0; area 1 = acc0 + acc_bytes
    size_t acc_bytes;
    uint32_t dirty_floats;   // floats of the accumulator area this call adds into
    uint32_t reserved;
    unsigned long long* trace;   // timeline buffer of trace builds, else NULL
};
template <int NP> struct Fused2Args { FusedCommon fc; DStageT<NP> s1, s2; };
struct FusedMlpArgs { FusedCommon fc; DStageT<1> a, b, c, d; };

// Fused launches (all stages in one kernel, `grid` resident workgroups of nw = 4 or 8 waves).  cpl* = columns per lane
// of each stage.  Return LR_ERR_UNSUPPORTED if the grid would not be fully resident.
int decode_launch_fused2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int cpl1, int cpl2,
                         int grid, int nw, bool t16, hipStream_t s);
int decode_launch_fused_mlp(const FusedMlpArgs& fa, int cpl_a, int cpl_c, int cpl_d, int grid, int nw, bool t16, hipStream_t s);
extern unsigned long long* g_trace_buffer;   // host copy of the trace pointer (NULL unless a trace build set it)
int decode_resident_grid();   // workgroups that are certainly co-resident (number of CUs), cached

// Launch one stage: cpl = bf16 columns per lane (4 or 8), a_f32 = activations are fp32 (rank-space
// accumulators) rather than bf16, epi = EPI_*.
int decode_launch_stage(const DStage& st, int cpl, bool a_f32, int epi, hipStream_t s);

// Host planners (decode_plan.hip).  They assume decode_shape_ok(...) held for every product.
bool decode_shape_ok(int64_t M, int64_t K, int64_t N);
int decode_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                  int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, size_t ws_bytes, hipStream_t s);
int decode_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
               void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
               const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
               void* ws, size_t ws_bytes, hipStream_t s);
int decode_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
               const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
               int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
               void* ws, size_t ws_bytes, hipStream_t s);

}  // namespace lr
