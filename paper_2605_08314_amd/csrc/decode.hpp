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
    int wstride;      // elements between consecutive rows of W (and W2) as stored: N, or 64 for the panel layout
    int64_t wtile, wtile2;   // elements between consecutive column tiles of W / W2: the tile width, or K * 64 (K2 * 64) for panels
};

template <int NP> struct DStageT { DProb p[NP]; int nprob, M, total_tiles; };
typedef DStageT<kMaxProb> DStage;

// Control block at the start of every workspace.  A stage barrier is kSlots counters on separate 128-byte lines:
// workgroup w adds 1 to slot w % kSlots, a waiting wave reads all slots with one load instruction.  One hot counter
// for 256 workgroups costs several microseconds per barrier on this chip; sixteen cool ones cost about one.
//
// `magic` says whether the block is valid.  A workspace may arrive with any contents (fresh allocation): the first
// kernel that needs the block and does not find kCtrlReady there prepares it itself (one wave wins a compare-and-swap
// to kCtrlBusy, zeroes the block, the shared-K flags and both accumulator areas, and publishes kCtrlReady; everyone
// else waits for that), so no host-side initialisation is required and a graph replay never depends on one.
constexpr int kBarriers = 3;
constexpr int kSlots = 16;
constexpr int kSlotStride = 32;   // uint32 words between slots (128 bytes)
constexpr int kTileCounters = 256;
constexpr uint64_t kCtrlReady = 0x6c72776b73703031ull;
constexpr uint64_t kCtrlBusy = 0x6c72776b73703030ull;
struct Ctrl {
    uint64_t magic;                     // kCtrlReady: everything below and the accumulator areas are in their between-calls state
    uint32_t epoch;                     // number of fused calls completed on this workspace
    uint32_t error;                     // nonzero: a bounded device-side wait gave up; stays set until the workspace is prepared again
    uint32_t dirty[2];                  // floats of accumulator area p that are not zero
    uint32_t pad[26];
    uint32_t cnt[2][kBarriers][kSlots * kSlotStride];   // [epoch parity][barrier][slot]
    uint32_t tcnt[2][kTileCounters];                    // arrivals per accumulator column tile (bf16 finalisation)
};
static_assert(sizeof(Ctrl) <= kHeaderBytes, "control block must fit the workspace header");

// Workspace layout.  Everything that carries state from one call to the next sits at a FIXED offset, whatever the
// call's shape or row count, so calls of any kind may follow each other on one workspace:
//   [0, 16 KiB)            control block
//   [16 KiB, 20 KiB)       flags of prefill products whose K range is shared between workgroups (zero between calls)
//   then 8 MiB             fp32 partial tiles of decode split-K stages with bf16 finalisation (scratch)
//   then 2 x 4 MiB         accumulator areas 0 and 1 of the fused decode kernels (zero between calls up to `dirty`)
//   then                   staging: scratch of the call (rank-space rows, hidden rows), sized by the call
//   last 64 MiB            only when the call has more than 32 rows: fp32 partial tiles of shared-K prefill products
constexpr size_t kSkFlagBytes = 4096;
constexpr size_t kSkSlotBytes = (size_t)256 * 256 * 256 * 4;
constexpr size_t kDecPartBytes = (size_t)8 << 20;
constexpr size_t kAccBytes = (size_t)4 << 20;
constexpr size_t kFrontBytes = kHeaderBytes + kSkFlagBytes + kDecPartBytes + 2 * kAccBytes;
// More token rows than this may use split-K partial tiles in slots + bf16 finalisation instead of atomics (the packed MLP
// does from 25 rows on: measured cross-over point; the two-stage calls keep the atomics).
constexpr int kT16Rows = 24;
inline size_t sk_tail_bytes(int64_t M) { return M > 32 ? kSkSlotBytes : 0; }

struct WsLayout {
    Ctrl* ctrl; uint32_t* sk_flags; float* dec_part;
    char* acc0; size_t acc_bytes;              // area 1 = acc0 + acc_bytes
    char* staging; size_t staging_bytes;
    float* sk_slots;                           // calls with more than 32 rows, else NULL
};
inline WsLayout ws_layout(void* ws, size_t ws_bytes, int64_t M) {
    WsLayout L;
    char* b = (char*)ws;
    L.ctrl = (Ctrl*)b;
    L.sk_flags = (uint32_t*)(b + kHeaderBytes);
    L.dec_part = (float*)(b + kHeaderBytes + kSkFlagBytes);
    L.acc0 = b + kHeaderBytes + kSkFlagBytes + kDecPartBytes;
    L.acc_bytes = kAccBytes;
    L.staging = b + kFrontBytes;
    const size_t tail = sk_tail_bytes(M);
    const size_t end = (ws_bytes - tail) & ~(size_t)255;
    L.staging_bytes = end - kFrontBytes;
    L.sk_slots = tail ? (float*)(b + end) : nullptr;
    return L;
}

struct FusedCommon {
    Ctrl* ctrl;
    char* acc0;              // accumulator area 0; area 1 = acc0 + acc_bytes
    size_t acc_bytes;
    uint32_t dirty_floats;   // floats of the accumulator area this call adds into
    uint32_t spin_limit;     // polls after which a device-wide wait gives up
    unsigned long long* trace;   // timeline buffer of trace builds, else NULL
};
template <int NP> struct Fused2Args { FusedCommon fc; DStageT<NP> s1, s2; };
struct FusedMlpArgs { FusedCommon fc; DStageT<1> a, b, c, d; };

// Fused launches (all stages in one kernel, `grid` resident workgroups of 8 waves).  cpl* = columns per lane
// of each stage.  Return LR_ERR_UNSUPPORTED if the grid would not be fully resident.
int decode_launch_fused2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int cpl1, int cpl2, int grid, hipStream_t s);
int decode_launch_fused_mlp(const FusedMlpArgs& fa, int cpl_a, int cpl_c, int cpl_d, int grid, bool t16, hipStream_t s);
extern unsigned long long* g_trace_buffer;   // host copy of the trace pointer (NULL unless a trace build set it)
bool decode_grid_is_resident(const void* kernel, int threads, int grid);   // occupancy of this very kernel x compute units >= grid
int decode_resident_grid();   // workgroups that are certainly co-resident (number of CUs), cached; 0 when the device is shared
// Process-wide settings behind lowrank_configure.
extern bool g_device_shared;        // other work may occupy CUs: no launch may rely on all of its workgroups being resident
extern uint32_t g_wait_limit;       // polls after which a device-side wait gives up
int ws_prepare(void* ws, hipStream_t s);   // enqueue the check-and-prepare launches (calls that run no fused decode kernel)

// Launch one stage: cpl = bf16 columns per lane (4 or 8), a_f32 = activations are fp32 (rank-space
// accumulators) rather than bf16, epi = EPI_*.
int decode_launch_stage(const DStage& st, int cpl, bool a_f32, int epi, hipStream_t s);

// Host planners (decode_plan.hip).  They assume decode_shape_ok(...) held for every product.  panels: the factors are stored
// as 64-column panels (lowrank_pack_panels) instead of row-major.
bool decode_shape_ok(int64_t M, int64_t K, int64_t N);
int decode_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                  int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, size_t ws_bytes, hipStream_t s, bool panels);
// the same with nothing but an fp32 area t[M * r] as scratch: one launch per stage
int decode_linear_scratch(const void* x, const void* U, const void* V, const void* bias, void* y,
                          int64_t M, int64_t d_in, int64_t r, int64_t d_out, float* t, hipStream_t s);
int decode_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
               void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
               const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
               void* ws, size_t ws_bytes, hipStream_t s, bool panels);
int decode_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
               const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
               int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
               void* ws, size_t ws_bytes, hipStream_t s, bool panels);

}  // namespace lr
