// C-ABI entry points of liblowrank.so: argument validation, plan selection (host integer
// logic only) and launches.  See include/lowrank.h for the contract of every function.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include "lr_common.hpp"
#include "decode.hpp"
#include "prefill.hpp"
#include "attention.hpp"

namespace lr {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return LR_OK;
    set_error("%s: HIP launch failed: %s", what, hipGetErrorString(e));
    return LR_ERR_LAUNCH;
}

static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

static int check_common(int dtype, int phase, int64_t M, void* ws, size_t ws_bytes, size_t need, bool allow_panels = false) {
    if (dtype != LR_F32 && dtype != LR_BF16 && !(allow_panels && dtype == LR_BF16_PANELS)) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (phase != LR_PHASE_DECODE && phase != LR_PHASE_PREFILL && phase != LR_PHASE_AUTO) {
        set_error("unknown phase %d", phase); return LR_ERR_PHASE; }
    if (M > 0) {
        if (!ws) { set_error("workspace is NULL"); return LR_ERR_WORKSPACE; }
        if (((uintptr_t)ws) & 255u) { set_error("workspace must be 256-byte aligned"); return LR_ERR_ALIGN; }
        if (ws_bytes < need) { set_error("workspace too small: %zu bytes given, %zu needed", ws_bytes, need); return LR_ERR_WORKSPACE; }
    }
    return LR_OK;
}

static inline int resolve_phase(int phase, int64_t M) {
    if (phase == LR_PHASE_AUTO) return M <= 32 ? LR_PHASE_DECODE : LR_PHASE_PREFILL;
    return phase;
}

enum Plan { PLAN_GENERIC = 0, PLAN_DECODE = 1, PLAN_PREFILL = 2 };

// LR_BF16_PANELS: bf16 data whose factor operands are stored as 64-column panels; only the decode kernels read that layout.
static int panels_need_decode(Plan plan) {
    if (plan == PLAN_DECODE) return LR_OK;
    set_error("factors in panel layout (LR_BF16_PANELS) are read by the decode kernels only: up to 32 rows, decode phase, "
              "16-byte aligned operands, every d_in and r a multiple of 32, every r and d_out a multiple of 64");
    return LR_ERR_UNSUPPORTED;
}
static const char* const kPlanNames[] = {"generic", "decode_mfma", "prefill_mfma"};


// The tuned kernels are bf16-only and need 16-byte aligned operands; decode additionally needs
// M <= 32.  A DECODE request with more rows, or a PREFILL request, goes to the prefill kernels
// when the shape allows, else to the generic ones.
static Plan pick_plan(int dtype, int phase, int64_t M, bool decode_ok, bool prefill_ok, bool aligned) {
    if (dtype != LR_BF16 || !aligned) return PLAN_GENERIC;
    if (resolve_phase(phase, M) == LR_PHASE_DECODE && decode_ok) return PLAN_DECODE;
    if (prefill_ok) return PLAN_PREFILL;
    return PLAN_GENERIC;
}

static size_t ws_bytes_for(int op, int64_t M, int64_t r_total, int64_t d_out) {
    // fixed front (control block, flags, partial-tile area, two accumulator areas: see ws_layout) | staging | shared-K tail.
    // Staging holds the rank-space rows [M, r_total] and, for the MLP, the hidden rows [M, ffn], as fp32 (the widest
    // any kernel family keeps them).
    size_t staging = align256((size_t)M * (size_t)r_total * 4) + 256;
    if (op == LR_OP_PACKED_MLP) staging += align256((size_t)M * (size_t)d_out * 4) + 256;
    return kFrontBytes + staging + sk_tail_bytes(M);
}

}  // namespace lr

using namespace lr;

// ---- scratch of lowrank_linear_noalloc: lives in the library image, one copy per device, never freed ----------
constexpr size_t kStaticScratchBytes = (size_t)512 << 10;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};        // device address of `scratch` on each device, once looked up

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
static int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { set_error("cannot identify the current device"); return LR_ERR_LAUNCH; }
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { set_error("static scratch: hipGetSymbolAddress failed: %s", hipGetErrorString(e)); return LR_ERR_LAUNCH; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LR_OK;
}

#ifdef LR_TRACE
extern "C" int lowrank_debug_trace(void* buf) { lr::g_trace_buffer = (unsigned long long*)buf; return 0; }
#endif

extern "C" {

const char* lowrank_last_error(void) { return g_err; }
const char* lowrank_version(void) { return "lowrank-mi355x 0.1 (gfx950)"; }

size_t lowrank_workspace_bytes(int op, int64_t M, int64_t d_in, int64_t r_total, int64_t d_out,
                               int dtype, int phase) {
    if (op < LR_OP_LINEAR || op > LR_OP_DECODE_ATTENTION) return 0;
    if (M < 0 || d_in < 0 || r_total < 0 || d_out < 0) return 0;
    if (dtype != LR_F32 && dtype != LR_BF16 && dtype != LR_BF16_PANELS) return 0;
    if (phase < LR_PHASE_DECODE || phase > LR_PHASE_AUTO) return 0;
    if (op == LR_OP_DECODE_ATTENTION) return (r_total > 0 && d_in % r_total == 0) ? attn_ws_bytes(M, d_in, r_total) : 0;
    return ws_bytes_for(op, M, r_total, d_out);
}

int lowrank_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace) { set_error("workspace is NULL"); return LR_ERR_NULL; }
    if (((uintptr_t)workspace) & 255u) { set_error("workspace must be 256-byte aligned"); return LR_ERR_ALIGN; }
    if (workspace_bytes < kFrontBytes) { set_error("workspace too small: %zu bytes given, every workspace has at least %zu", workspace_bytes, (size_t)kFrontBytes); return LR_ERR_WORKSPACE; }
    // zero-fill the part that carries state (the ready word included), then let the preparation launches mark it ready
    int st = fill_zero(workspace, kHeaderBytes + kSkFlagBytes, (hipStream_t)stream);
    if (st != LR_OK) return st;
    return ws_prepare(workspace, (hipStream_t)stream);
}

int lowrank_workspace_status(const void* workspace, void* stream) {
    if (!workspace) { set_error("workspace is NULL"); return LR_ERR_NULL; }
    Ctrl c;
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(&c, workspace, 128, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        set_error("workspace status: copy failed: %s", hipGetErrorString(hipGetLastError()));
        return LR_ERR_LAUNCH;
    }
    if (c.magic == kCtrlReady && c.error != 0) {
        set_error("a device-side wait between stages gave up; the results of that call are NaN and the workspace must be prepared again (lowrank_workspace_init)");
        return LR_ERR_LAUNCH;
    }
    return LR_OK;
}

int lowrank_configure(int option, int64_t value) {
    switch (option) {
        case LR_CFG_DEVICE_SHARED: g_device_shared = value != 0; return LR_OK;
        case LR_CFG_WAIT_LIMIT:
            if (value < 0 || value > (int64_t)0x7fffffff) { set_error("wait limit out of range"); return LR_ERR_SHAPE; }
            g_wait_limit = (uint32_t)value; return LR_OK;
        default: set_error("unknown option %d", option); return LR_ERR_UNSUPPORTED;
    }
}

const char* lowrank_plan_name(int op, int64_t M, int64_t d_in, int64_t r_total, int64_t d_out,
                              int dtype, int phase, int aligned) {
    if (phase < LR_PHASE_DECODE || phase > LR_PHASE_AUTO || M < 1) return kPlanNames[PLAN_GENERIC];
    bool dec, pre;
    if (op == LR_OP_PACKED_MLP) {   // every rank taken as r_total / 3
        const int64_t r = r_total / 3;
        dec = (r_total % 3 == 0) && decode_shape_ok(M, d_in, 2 * r) && decode_shape_ok(M, r, d_out) &&
              decode_shape_ok(M, d_out, r) && decode_shape_ok(M, r, d_in);
        pre = (r_total % 3 == 0) && prefill_shape_ok(M, d_in, 2 * r) && prefill_shape_ok(M, r, d_out) &&
              prefill_shape_ok(M, d_out, r) && prefill_shape_ok(M, r, d_in);
    } else {                        // QKV: the sums stand for projections that each satisfy the rule
        dec = decode_shape_ok(M, d_in, r_total) && decode_shape_ok(M, r_total, d_out);
        pre = prefill_shape_ok(M, d_in, r_total) && prefill_shape_ok(M, r_total, d_out);
    }
    if (dtype == LR_BF16_PANELS) {      // panels run the decode kernels or nothing
        const Plan p = pick_plan(LR_BF16, phase, M, dec, pre, aligned != 0);
        return p == PLAN_DECODE ? kPlanNames[PLAN_DECODE] : "unsupported";
    }
    return kPlanNames[pick_plan(dtype, phase, M, dec, pre, aligned != 0)];
}

int lowrank_prefill_tile(int64_t M, int64_t K, int64_t N, int n_products, int gate_up,
                         int* tile_m, int* tile_n, int* share_k) {
    if (!tile_m || !tile_n || !share_k) { set_error("NULL result pointer"); return LR_ERR_NULL; }
    if (n_products < 1 || n_products > 8) { set_error("n_products must be 1..8"); return LR_ERR_SHAPE; }
    if (!prefill_shape_ok(M, K, N)) { set_error("shape outside the matrix-core prefill rule (K %% 64, N %% 128)"); return LR_ERR_UNSUPPORTED; }
    prefill_plan_query(M, K, N, n_products, gate_up != 0, tile_m, tile_n, share_k);
    return LR_OK;
}

int lowrank_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                   int64_t M, int64_t d_in, int64_t r, int64_t d_out, int dtype, int phase,
                   void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || d_in < 0 || r < 0 || d_out < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    int st = check_common(dtype, phase, M, workspace, workspace_bytes, ws_bytes_for(LR_OP_LINEAR, M, r, d_out), true);
    if (st != LR_OK) return st;
    const bool panels = dtype == LR_BF16_PANELS;
    if (panels) dtype = LR_BF16;
    if (M == 0 || d_out == 0) return LR_OK;
    if (!y || (d_in > 0 && !x) || (r > 0 && d_in > 0 && !U) || (r > 0 && !V)) { set_error("NULL operand"); return LR_ERR_NULL; }
    hipStream_t s = (hipStream_t)stream;
    const bool al = aligned16(x) && aligned16(U) && aligned16(V) && aligned16(y) && aligned16(bias);
    const Plan plan = pick_plan(dtype, phase, M, decode_shape_ok(M, d_in, r) && decode_shape_ok(M, r, d_out),
                                prefill_shape_ok(M, d_in, r) && prefill_shape_ok(M, r, d_out), al);
    if (panels && (st = panels_need_decode(plan)) != LR_OK) return st;
    if (plan == PLAN_DECODE) return decode_linear(x, U, V, bias, y, M, d_in, r, d_out, workspace, workspace_bytes, s, panels);
    if (plan == PLAN_PREFILL) return prefill_linear(x, U, V, bias, y, M, d_in, r, d_out, workspace, workspace_bytes, s);
    float* t = (float*)ws_layout(workspace, workspace_bytes, M).staging;
    CacheDst none = {nullptr, nullptr, 0, 1};
    st = generic_stage1(x, false, U, t, r, M, d_in, r, dtype, s);
    if (st != LR_OK) return st;
    return generic_stage2(t, r, V, bias, y, M, r, d_out, none, dtype, s);
}

int lowrank_linear_noalloc(const void* x, const void* U, const void* V, const void* bias, void* y,
                           int64_t M, int64_t d_in, int64_t r, int64_t d_out, int dtype, void* stream) {
    if (M < 0 || d_in < 0 || r < 0 || d_out < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    if (dtype != LR_F32 && dtype != LR_BF16) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (M == 0 || d_out == 0) return LR_OK;
    if (!y || (d_in > 0 && !x) || (r > 0 && d_in > 0 && !U) || (r > 0 && !V)) { set_error("NULL operand"); return LR_ERR_NULL; }
    if (M >= ((int64_t)1 << 31) / 4 || r >= ((int64_t)1 << 31) / 4 || (size_t)M * (size_t)r * 4 > kStaticScratchBytes) {
        set_error("lowrank_linear_noalloc: M * r = %lld exceeds the %zu floats of the built-in scratch (use lowrank_linear with a workspace)",
                  (long long)(M * r), kStaticScratchBytes / 4);
        return LR_ERR_WORKSPACE;
    }
    void* sp = nullptr;
    int st = static_scratch(&sp);
    if (st != LR_OK) return st;
    float* t = (float*)sp;
    hipStream_t s = (hipStream_t)stream;
    const bool al = aligned16(x) && aligned16(U) && aligned16(V) && aligned16(y) && aligned16(bias);
    if (dtype == LR_BF16 && al && M <= 32 && decode_shape_ok(M, d_in, r) && decode_shape_ok(M, r, d_out))
        return decode_linear_scratch(x, U, V, bias, y, M, d_in, r, d_out, t, s);
    CacheDst none = {nullptr, nullptr, 0, 1};
    st = generic_stage1(x, false, U, t, r, M, d_in, r, dtype, s);
    if (st != LR_OK) return st;
    return generic_stage2(t, r, V, bias, y, M, r, d_out, none, dtype, s);
}

int lowrank_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
                void* const* out, const int64_t* r, const int64_t* d_out, int n_proj,
                int64_t M, int64_t d_in, const lr_kv_target* kv, int dtype, int phase,
                void* workspace, size_t workspace_bytes, void* stream) {
    if (n_proj < 1 || n_proj > 8) { set_error("n_proj must be 1..8"); return LR_ERR_SHAPE; }
    if (!U || !V || !out || !r || !d_out) { set_error("NULL host array"); return LR_ERR_NULL; }
    if (M < 0 || d_in < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    int64_t r_sum = 0, n_sum = 0;
    for (int i = 0; i < n_proj; ++i) {
        if (r[i] < 0 || d_out[i] < 0) { set_error("negative size in projection %d", i); return LR_ERR_SHAPE; }
        r_sum += r[i]; n_sum += d_out[i];
    }
    int st = check_common(dtype, phase, M, workspace, workspace_bytes, ws_bytes_for(LR_OP_QKV, M, r_sum, n_sum), true);
    if (st != LR_OK) return st;
    const bool panels = dtype == LR_BF16_PANELS;
    if (panels) dtype = LR_BF16;
    // shared bases: projection i reuses the stage-1 product of the first j < i with U[j] == U[i]
    int base_of[8]; int64_t t_off[8]; int64_t R = 0;
    for (int i = 0; i < n_proj; ++i) {
        base_of[i] = i;
        for (int j = 0; j < i; ++j)
            if (U[j] == U[i] && U[i] != nullptr) {
                if (r[j] != r[i]) { set_error("projections %d and %d share U but differ in rank", j, i); return LR_ERR_SHAPE; }
                base_of[i] = j; break;
            }
        if (base_of[i] == i) { t_off[i] = R; R += r[i]; } else t_off[i] = t_off[base_of[i]];
    }
    if (kv) {
        if (kv->k_index < 0 || kv->k_index >= n_proj || kv->v_index < 0 || kv->v_index >= n_proj) {
            set_error("k_index / v_index out of range"); return LR_ERR_SHAPE; }
        if (kv->B < 0 || kv->tokens_per_seq < 1 || kv->B * kv->tokens_per_seq != M) {
            set_error("kv: B * tokens_per_seq must equal M"); return LR_ERR_SHAPE; }
        if (kv->S_max < kv->tokens_per_seq || kv->n_heads < 1 || kv->head_dim < 1) {
            set_error("kv: bad cache shape"); return LR_ERR_SHAPE; }
        if (kv->S_max >= (1ll << 30) || kv->B >= (1ll << 30) || kv->B * kv->S_max >= (1ll << 31)) {   // cache rows are indexed with 32-bit integers
            set_error("kv: B * S_max must be below 2^31"); return LR_ERR_SHAPE; }
        const int64_t w = kv->n_heads * kv->head_dim;
        if (d_out[kv->k_index] != w || d_out[kv->v_index] != w) {
            set_error("kv: d_out of K and V must equal n_heads * head_dim"); return LR_ERR_SHAPE; }
        if (M > 0 && (!kv->pos || !kv->k_cache || !kv->v_cache)) { set_error("kv: NULL cache or pos"); return LR_ERR_NULL; }
    }
    if (M == 0) return LR_OK;
    for (int i = 0; i < n_proj; ++i) {
        const bool to_cache = kv && (i == kv->k_index || i == kv->v_index);
        if (d_out[i] == 0) continue;
        if (!out[i] && !to_cache) { set_error("projection %d has no destination", i); return LR_ERR_NULL; }
        if ((r[i] > 0 && d_in > 0 && !U[i]) || (r[i] > 0 && !V[i])) { set_error("NULL factor in projection %d", i); return LR_ERR_NULL; }
    }
    if (d_in > 0 && !x) { set_error("x is NULL"); return LR_ERR_NULL; }
    hipStream_t s = (hipStream_t)stream;
    bool al = aligned16(x), dec = true, pre = true;
    for (int i = 0; i < n_proj; ++i) {
        al = al && aligned16(U[i]) && aligned16(V[i]) && aligned16(out[i]) && aligned16(bias ? bias[i] : nullptr);
        dec = dec && decode_shape_ok(M, d_in, r[i]) && decode_shape_ok(M, r[i], d_out[i]);
        pre = pre && prefill_shape_ok(M, d_in, r[i]) && prefill_shape_ok(M, r[i], d_out[i]);
    }
    if (kv) al = al && aligned16(kv->k_cache) && aligned16(kv->v_cache);
    const Plan plan = pick_plan(dtype, phase, M, dec, pre, al);
    if (panels && (st = panels_need_decode(plan)) != LR_OK) return st;
    if (plan == PLAN_DECODE)
        return decode_qkv(x, U, V, bias, out, r, d_out, n_proj, base_of, t_off, R, M, d_in, kv, workspace, workspace_bytes, s, panels);
    if (plan == PLAN_PREFILL)
        return prefill_qkv(x, U, V, bias, out, r, d_out, n_proj, base_of, t_off, R, M, d_in, kv, workspace, workspace_bytes, s);
    float* t = (float*)ws_layout(workspace, workspace_bytes, M).staging;
    const int64_t ldt = R > 0 ? R : 1;
    for (int i = 0; i < n_proj; ++i)
        if (base_of[i] == i) {
            st = generic_stage1(x, false, U[i], t + t_off[i], ldt, M, d_in, r[i], dtype, s);
            if (st != LR_OK) return st;
        }
    for (int i = 0; i < n_proj; ++i) {
        CacheDst cd = {nullptr, nullptr, 0, 1};
        if (kv && i == kv->k_index) cd = {kv->k_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        if (kv && i == kv->v_index) cd = {kv->v_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        st = generic_stage2(t + t_off[i], ldt, V[i], bias ? bias[i] : nullptr, out[i], M, r[i], d_out[i], cd, dtype, s);
        if (st != LR_OK) return st;
    }
    return LR_OK;
}

int lowrank_packed_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u,
                       const void* U_d, const void* V_d, const void* b_g, const void* b_u, const void* b_d,
                       void* out, int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
                       int dtype, int phase, void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || d < 0 || ffn < 0 || r_g < 0 || r_u < 0 || r_d < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    const int64_t r_total = r_g + r_u + r_d;
    int st = check_common(dtype, phase, M, workspace, workspace_bytes, ws_bytes_for(LR_OP_PACKED_MLP, M, r_total, ffn), true);
    if (st != LR_OK) return st;
    const bool panels = dtype == LR_BF16_PANELS;
    if (panels) dtype = LR_BF16;
    if (M == 0 || d == 0) return LR_OK;
    if (!x || !out) { set_error("NULL operand"); return LR_ERR_NULL; }
    if ((r_g + r_u > 0 && !U_gu) || (r_g > 0 && ffn > 0 && !V_g) || (r_u > 0 && ffn > 0 && !V_u) ||
        (r_d > 0 && ffn > 0 && !U_d) || (r_d > 0 && !V_d)) { set_error("NULL factor"); return LR_ERR_NULL; }
    hipStream_t s = (hipStream_t)stream;
    const bool al = aligned16(x) && aligned16(U_gu) && aligned16(V_g) && aligned16(V_u) && aligned16(U_d) &&
                    aligned16(V_d) && aligned16(b_g) && aligned16(b_u) && aligned16(b_d) && aligned16(out);
    const bool dec = decode_shape_ok(M, d, r_g) && decode_shape_ok(M, d, r_u) && decode_shape_ok(M, r_g, ffn) &&
                     decode_shape_ok(M, r_u, ffn) && decode_shape_ok(M, ffn, r_d) && decode_shape_ok(M, r_d, d);
    const bool pre = prefill_shape_ok(M, d, r_g + r_u) && prefill_shape_ok(M, r_g, ffn) && prefill_shape_ok(M, r_u, ffn) &&
                     prefill_shape_ok(M, ffn, r_d) && prefill_shape_ok(M, r_d, d);
    const Plan plan = pick_plan(dtype, phase, M, dec, pre, al);
    if (panels && (st = panels_need_decode(plan)) != LR_OK) return st;
    if (plan == PLAN_DECODE)
        return decode_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g, b_u, b_d, out, M, d, ffn, r_g, r_u, r_d, workspace, workspace_bytes, s, panels);
    if (plan == PLAN_PREFILL)
        return prefill_mlp(x, U_gu, V_g, V_u, U_d, V_d, b_g, b_u, b_d, out, M, d, ffn, r_g, r_u, r_d, workspace, workspace_bytes, s);
    char* base = ws_layout(workspace, workspace_bytes, M).staging;
    float* t = (float*)base;                                   // [M, r_g + r_u + r_d]
    float* h = (float*)(base + align256((size_t)M * (size_t)r_total * 4));       // [M, ffn]
    const int64_t ldt = r_total > 0 ? r_total : 1;
    CacheDst none = {nullptr, nullptr, 0, 1};
    st = generic_stage1(x, false, U_gu, t, ldt, M, d, r_g + r_u, dtype, s);
    if (st != LR_OK) return st;
    st = generic_gateup(t, ldt, V_g, V_u, b_g, b_u, h, M, r_g, r_u, ffn, dtype, s);
    if (st != LR_OK) return st;
    st = generic_stage1(h, true, U_d, t + (r_g + r_u), ldt, M, ffn, r_d, dtype, s);
    if (st != LR_OK) return st;
    return generic_stage2(t + (r_g + r_u), ldt, V_d, b_d, out, M, r_d, d, none, dtype, s);
}

int lowrank_decode_attention(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base,
                             int dtype, void* workspace, size_t workspace_bytes, void* stream) {
    if (dtype != LR_F32 && dtype != LR_BF16) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (!kv) { set_error("kv is NULL"); return LR_ERR_NULL; }
    if (kv->B < 0 || kv->tokens_per_seq < 1 || kv->S_max < kv->tokens_per_seq || kv->n_heads < 1 || kv->head_dim < 1) {
        set_error("kv: bad cache shape"); return LR_ERR_SHAPE; }
    if ((kv->head_dim & 1) || kv->head_dim > 1024) { set_error("head_dim must be even and at most 1024"); return LR_ERR_UNSUPPORTED; }
    const int64_t M = kv->B * kv->tokens_per_seq, H = kv->n_heads, E = kv->head_dim;
    if (M >= (1ll << 24) || H * E >= (1ll << 24) || kv->S_max >= (1ll << 30)) { set_error("size out of range"); return LR_ERR_SHAPE; }
    if (M == 0) return LR_OK;
    if (!q || !out || !kv->k_cache || !kv->v_cache || !kv->pos) { set_error("NULL operand"); return LR_ERR_NULL; }
    if (!workspace) { set_error("workspace is NULL"); return LR_ERR_WORKSPACE; }
    if (((uintptr_t)workspace) & 255u) { set_error("workspace must be 256-byte aligned"); return LR_ERR_ALIGN; }
    const size_t need = attn_ws_bytes(M, H * E, H);
    if (workspace_bytes < need) { set_error("workspace too small: %zu bytes given, %zu needed", workspace_bytes, need); return LR_ERR_WORKSPACE; }
    const bool al = aligned16(q) && aligned16(out) && aligned16(kv->k_cache) && aligned16(kv->v_cache);
    return attn_decode(q, kv, out, scale, rope_base, dtype, attn_fast_ok(dtype, E, al), workspace, (hipStream_t)stream);
}

int lowrank_prefill_attention(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base,
                              int dtype, void* stream) {
    if (dtype != LR_F32 && dtype != LR_BF16) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (!kv) { set_error("kv is NULL"); return LR_ERR_NULL; }
    if (kv->B < 0 || kv->tokens_per_seq < 1 || kv->S_max < kv->tokens_per_seq || kv->n_heads < 1 || kv->head_dim < 1) {
        set_error("kv: bad cache shape"); return LR_ERR_SHAPE; }
    const int64_t M = kv->B * kv->tokens_per_seq, H = kv->n_heads, E = kv->head_dim;
    if (M >= (1ll << 24) || H * E >= (1ll << 24) || kv->S_max >= (1ll << 30)) { set_error("size out of range"); return LR_ERR_SHAPE; }
    if (M == 0) return LR_OK;
    if (!q || !out || !kv->k_cache || !kv->v_cache || !kv->pos) { set_error("NULL operand"); return LR_ERR_NULL; }
    const bool al = aligned16(q) && aligned16(out) && aligned16(kv->k_cache) && aligned16(kv->v_cache);
    if (!attn_prefill_ok(dtype, E, al)) {
        set_error("prefill attention: needs bf16, head_dim 128 and 16-byte aligned operands (use lowrank_decode_attention)");
        return LR_ERR_UNSUPPORTED;
    }
    return attn_prefill(q, kv, out, scale, rope_base, (hipStream_t)stream);
}

int lowrank_prefill_factorized_attention(const void* t_q, const void* V_q, const void* b_q, int64_t r_q, const lr_kv_target* kv,
                                         void* out, float scale, float rope_base, int dtype, void* stream) {
    if (dtype != LR_F32 && dtype != LR_BF16) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (!kv) { set_error("kv is NULL"); return LR_ERR_NULL; }
    if (kv->B < 0 || kv->tokens_per_seq < 1 || kv->S_max < kv->tokens_per_seq || kv->n_heads < 1 || kv->head_dim < 1 || r_q < 0) {
        set_error("kv: bad cache shape"); return LR_ERR_SHAPE; }
    const int64_t M = kv->B * kv->tokens_per_seq, H = kv->n_heads, E = kv->head_dim;
    if (M >= (1ll << 24) || H * E >= (1ll << 24) || kv->S_max >= (1ll << 30) || r_q >= (1ll << 20)) { set_error("size out of range"); return LR_ERR_SHAPE; }
    if (M == 0) return LR_OK;
    if (!t_q || !V_q || !out || !kv->k_cache || !kv->v_cache || !kv->pos) { set_error("NULL operand"); return LR_ERR_NULL; }
    const bool al = aligned16(t_q) && aligned16(V_q) && aligned16(b_q) && aligned16(out) && aligned16(kv->k_cache) && aligned16(kv->v_cache);
    if (!attn_prefill_ok(dtype, E, al) || r_q < 64 || r_q % 64 != 0) {
        set_error("factorized prefill attention: needs bf16, head_dim 128, a rank that is a multiple of 64 and 16-byte aligned operands "
                  "(otherwise reconstruct q with lowrank_linear and use lowrank_prefill_attention / lowrank_decode_attention)");
        return LR_ERR_UNSUPPORTED;
    }
    return attn_prefill(nullptr, kv, out, scale, rope_base, (hipStream_t)stream, t_q, V_q, b_q, r_q);
}

int lowrank_rank_project(const void* x, const void* U, void* t, int64_t M, int64_t d_in, int64_t r, int dtype,
                         void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || d_in < 0 || r < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    int st = check_common(dtype, LR_PHASE_AUTO, M, workspace, workspace_bytes, ws_bytes_for(LR_OP_LINEAR, M, r, 0));
    if (st != LR_OK) return st;
    if (M == 0 || r == 0) return LR_OK;
    if (!t || (d_in > 0 && (!x || !U))) { set_error("NULL operand"); return LR_ERR_NULL; }
    hipStream_t s = (hipStream_t)stream;
    const bool al = aligned16(x) && aligned16(U) && aligned16(t);
    if (dtype == LR_BF16 && al && prefill_shape_ok(M, d_in, r)) return prefill_rank_project(x, U, t, M, d_in, r, workspace, workspace_bytes, s);
    float* t32 = (float*)ws_layout(workspace, workspace_bytes, M).staging;
    st = generic_stage1(x, false, U, t32, r, M, d_in, r, dtype, s);
    if (st != LR_OK) return st;
    return generic_round(t32, t, M * r, dtype, s);
}

int lowrank_pack_concat(const void* const* U_list, const int64_t* r_list, int n, int64_t d_in,
                        int dtype, void* U_packed, void* stream) {
    if (n < 1 || n > 8) { set_error("n must be 1..8"); return LR_ERR_SHAPE; }
    if (!U_list || !r_list) { set_error("NULL host array"); return LR_ERR_NULL; }
    if (dtype != LR_F32 && dtype != LR_BF16) { set_error("unknown dtype %d", dtype); return LR_ERR_DTYPE; }
    if (d_in < 0) { set_error("negative size"); return LR_ERR_SHAPE; }
    int64_t R = 0;
    for (int i = 0; i < n; ++i) {
        if (r_list[i] < 0) { set_error("negative rank"); return LR_ERR_SHAPE; }
        if (r_list[i] > 0 && d_in > 0 && !U_list[i]) { set_error("NULL factor %d", i); return LR_ERR_NULL; }
        R += r_list[i];
    }
    if (R * d_in > 0 && !U_packed) { set_error("U_packed is NULL"); return LR_ERR_NULL; }
    return generic_pack_concat(U_list, r_list, n, d_in, dtype == LR_F32 ? 4 : 2, U_packed, (hipStream_t)stream);
}

int lowrank_pack_panels(const void* W, int64_t K, int64_t N, void* W_panels, int dtype, void* stream) {
    if (dtype != LR_BF16) { set_error("lowrank_pack_panels: bf16 only"); return LR_ERR_DTYPE; }
    if (K < 0 || N < 0 || (N % 64) != 0) { set_error("lowrank_pack_panels: N must be a multiple of 64 (and sizes non-negative)"); return LR_ERR_SHAPE; }
    if (K * N == 0) return LR_OK;
    if (!W || !W_panels) { set_error("NULL operand"); return LR_ERR_NULL; }
    if (W == W_panels) { set_error("lowrank_pack_panels: not in place"); return LR_ERR_SHAPE; }
    if (!aligned16(W) || !aligned16(W_panels)) { set_error("lowrank_pack_panels: operands must be 16-byte aligned"); return LR_ERR_ALIGN; }
    return generic_pack_panels(W, K, N, W_panels, (hipStream_t)stream);
}

}  // extern "C"
