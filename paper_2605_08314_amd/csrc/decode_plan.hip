// Host-side planning of the decode phase: how each stage is cut into workgroup tiles and whether
// the call runs as one fused launch.  Integer logic only; every function enqueues kernels on the
// caller's stream and returns.
#include <stdlib.h>
#include <string.h>
#include "decode.hpp"

namespace lr {

unsigned long long* g_trace_buffer = nullptr;

bool g_device_shared = false;
uint32_t g_wait_limit = 1u << 20;

// Fast-path shape rule: rows ride on one or two 16-row MFMA blocks, K in 32-row blocks, N in
// 64-column tiles.
bool decode_shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && M <= 32 && K >= 32 && (K % 32) == 0 && N >= 64 && (N % 64) == 0 &&
           K < (1 << 24) && N < (1 << 24);
}

// Columns per lane of every stage: 4 = 64-column tiles with 8-byte loads.  (128-column tiles with 16-byte loads
// were measured slower: fewer, fatter tiles.)
constexpr int kCpl = 4;
// Tiles of a split-K stage that runs as a launch of its own (device shared with other work, or accumulators too big).
constexpr int kUnfusedTiles = 512;

// Split-K stage: rows of W per tile so that the stage has about `want_tiles` tiles.  Multiples of
// 32 rows, at least 128 (one block per wave); at least 256 for more than 8 token rows, which keeps
// the fp32 atomics (tiles_k * M * N) small against the weight bytes.
static int pick_ks(int64_t K, int64_t tiles_n_total, int64_t M, int64_t want_tiles) {
    int64_t tk = want_tiles / (tiles_n_total > 0 ? tiles_n_total : 1);
    if (tk < 1) tk = 1;
    int64_t ks = (K + tk - 1) / tk;
    ks = ((ks + 31) / 32) * 32;
    const int64_t floor_ks = M > 8 ? 256 : 128;
    if (ks < floor_ks) ks = floor_ks;
    if (ks > K) ks = K;
    return (int)ks;
}

static void zero_prob(DProb& p) { memset(&p, 0, sizeof(p)); p.T = 1; }
// Where the factor of every product of a stage lives: row-major [K, N] as stored in a checkpoint, or 64-column panels
// (lowrank_pack_panels: element (k, n) at ((n / 64) * K + k) * 64 + n % 64), in which a tile is one contiguous run.
static void set_wlayout(DStage& st, int nc, bool panels) {
    for (int i = 0; i < st.nprob; ++i) {
        DProb& p = st.p[i];
        if (panels) { p.wstride = nc; p.wtile = (int64_t)p.K * nc; p.wtile2 = (int64_t)p.K2 * nc; }
        else { p.wstride = p.N; p.wtile = nc; p.wtile2 = nc; }
    }
}

struct SplitK { const void* W; int64_t N; float* C; bf16_t* T16; float* part; };   // T16: bf16 copy of C made by the last K-slice (or NULL)
struct Final { const void* T; int64_t r; const void* V; int64_t N; const void* bias; void* Y; CacheDst cd; };   // T: fp32 or bf16 rank-space rows

// t[M, ldc] += A[M, K] * W_i[K, N_i] for several weight matrices sharing A, split along K.
static void build_splitk(DStage& st, const void* A, int64_t lda, int64_t M, int64_t K, const SplitK* items, int n,
                         int64_t ldc, int64_t want_tiles, int cpl, int* ctile_next, bool panels) {
    st.nprob = n; st.M = (int)M;
    int64_t n_all = 0;
    for (int i = 0; i < n; ++i) n_all += items[i].N;
    const int nc = 16 * cpl;
    const int ks = pick_ks(K, n_all / nc, M, want_tiles);
    const int tk = (int)((K + ks - 1) / ks);
    int tile = 0;
    for (int i = 0; i < n; ++i) {
        DProb& p = st.p[i]; zero_prob(p);
        p.W = (const bf16_t*)items[i].W; p.A = A; p.K = (int)K; p.lda = (int)lda; p.N = (int)items[i].N;
        p.C = items[i].C; p.ldc = (int)ldc; p.tiles_n = (int)(items[i].N / nc); p.KS = ks; p.tile_begin = tile;
        p.Y = items[i].T16; p.part = items[i].part; p.ldy = (int)ldc; p.ctile_begin = *ctile_next; *ctile_next += p.tiles_n;
        tile += p.tiles_n * tk;
    }
    st.total_tiles = tile;
    set_wlayout(st, nc, panels);
}

// y_i[M, N_i] = t_i[M, r_i] * V_i[r_i, N_i] + bias_i: full K per tile, the epilogue writes bf16.
static int build_final(DStage& st, const Final* items, int n, int64_t ldt, int64_t M, bool panels) {
    st.nprob = n; st.M = (int)M;
    const int cpl = 4;   // 64-column tiles: full K per tile, so narrow tiles are the only source of parallelism
    const int nc = 16 * cpl;
    int tile = 0;
    for (int i = 0; i < n; ++i) {
        DProb& p = st.p[i]; zero_prob(p);
        p.W = (const bf16_t*)items[i].V; p.A = items[i].T; p.K = (int)items[i].r; p.lda = (int)ldt; p.N = (int)items[i].N;
        p.Y = (bf16_t*)items[i].Y; p.bias = (const bf16_t*)items[i].bias;
        p.cache = items[i].cd.cache; p.pos = items[i].cd.pos; p.S_max = (int)items[i].cd.S_max; p.T = (int)items[i].cd.T;
        p.tiles_n = (int)(items[i].N / nc); p.KS = (int)items[i].r; p.tile_begin = tile;
        tile += p.tiles_n;
    }
    st.total_tiles = tile;
    set_wlayout(st, nc, panels);
    return cpl;
}

// One launch per call unless the device is shared with other work (lowrank_configure) or the device query fails.  The grid is one
// workgroup per ~96 KB of factor bytes, between 64 and the number of CUs: a stage barrier costs more
// the more workgroups take part, and a 6 MB call (one O projection) gains nothing from 256 of them
// (measured: 8.1 us at 64 workgroups, 9.8 us at 256), while 18 MB and more want the whole chip.
static int fused_grid(size_t factor_bytes) {
    const int cus = decode_resident_grid();
    if (cus <= 0) return 0;
    size_t g = factor_bytes / (96u << 10);
    if (g < 64) g = 64;
    if (g > (size_t)cus) g = (size_t)cus;
    return (int)g;
}

// More than `min_rows` token rows: split-K accumulators are finalised to bf16 once (see decode_tile) instead of
// every consumer workgroup converting all of t.  Measured (atomics / finalisation, us): packed MLP 27.3 / 31.2 at 8 rows,
// 30.1 / 32.6 at 16, 33.7 / 34.5 at 20, 34.9 / 34.95 at 24, 36.15 / 36.05 at 28, 37.2 / 36.9 at 32; QKV (R = 1152) 11.9 / 13.9
// at 16, 12.8 / 14.4 at 20, 13.95 / 15.2 at 32; O projection (R = 384) 12.0 / 12.5 at 25, 12.5 / 13.0 at 32.  (Before the
// atomics went out as one per thread on consecutive floats the cross-over points were 8 and 17 rows.)
static bool use_t16(int64_t M, int64_t col_tiles, int min_rows) {
    return M > min_rows && M > kT16Rows && col_tiles <= kTileCounters;
}

// t_only != NULL: the call has no workspace, only this fp32 area of M * R floats for the rank-space rows; it then runs as
// one launch per stage (no control block, no cross-workgroup waits).
static int run_two_stage(const void* x, int64_t d_in, int64_t M, const SplitK* sk_in, int nb, const Final* fin_in,
                         int nf, int64_t R, void* ws, size_t ws_bytes, hipStream_t s, bool panels, float* t_only = nullptr) {
    WsLayout L;
    if (t_only) { memset(&L, 0, sizeof(L)); L.staging = (char*)t_only; }
    else L = ws_layout(ws, ws_bytes, M);
    size_t factor_bytes = 0;
    for (int i = 0; i < nb; ++i) factor_bytes += (size_t)d_in * sk_in[i].N * 2;
    for (int i = 0; i < nf; ++i) factor_bytes += (size_t)fin_in[i].r * fin_in[i].N * 2;
    const int G = t_only ? 0 : fused_grid(factor_bytes);
    const bool fused = G > 0 && (size_t)M * R * 4 <= L.acc_bytes;
    const int c1 = kCpl;
    // two-stage calls add their split-K partial sums with atomics at every row count (see the measurements above); the bf16
    // finalisation is the packed MLP's, whose split-K stages are followed by the widest consumers
    float* tbase = fused ? (float*)L.acc0 : (float*)L.staging;
    SplitK sk[kMaxProb]; Final fin[kMaxProb];
    DStage s1, s2;
    // the callers pass the column offset of each product inside t as the pointer value of C / T
    for (int i = 0; i < nb; ++i) {
        const size_t off = (size_t)(uintptr_t)sk_in[i].C;
        sk[i] = sk_in[i]; sk[i].C = tbase + off; sk[i].T16 = nullptr; sk[i].part = nullptr;
    }
    for (int i = 0; i < nf; ++i) {
        const size_t off = (size_t)(uintptr_t)fin_in[i].T;
        fin[i] = fin_in[i]; fin[i].T = (const void*)(tbase + off);
    }
    int ctile = 0;
    build_splitk(s1, x, d_in, M, d_in, sk, nb, R, fused ? G : kUnfusedTiles, c1, &ctile, panels);
    const int c2 = build_final(s2, fin, nf, R, M, panels);
    if (fused) {
        FusedCommon fc = {L.ctrl, L.acc0, L.acc_bytes, (uint32_t)(M * R), g_wait_limit, g_trace_buffer};
        return decode_launch_fused2(fc, s1, s2, c1, c2, G, s);
    }
    int st = fill_zero(tbase, (size_t)M * R * 4, s);
    if (st != LR_OK) return st;
    st = decode_launch_stage(s1, c1, false, EPI_ATOMIC, s);
    if (st != LR_OK) return st;
    return decode_launch_stage(s2, c2, true, EPI_STORE, s);
}

int decode_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                  int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, size_t ws_bytes, hipStream_t s, bool panels) {
    SplitK sk = {U, r, (float*)0, nullptr, nullptr};
    Final f = {(const void*)0, r, V, d_out, bias, y, {nullptr, nullptr, 0, 1}};
    return run_two_stage(x, d_in, M, &sk, 1, &f, 1, r, ws, ws_bytes, s, panels);
}

int decode_linear_scratch(const void* x, const void* U, const void* V, const void* bias, void* y,
                          int64_t M, int64_t d_in, int64_t r, int64_t d_out, float* t, hipStream_t s) {
    SplitK sk = {U, r, (float*)0, nullptr, nullptr};
    Final f = {(const void*)0, r, V, d_out, bias, y, {nullptr, nullptr, 0, 1}};
    return run_two_stage(x, d_in, M, &sk, 1, &f, 1, r, nullptr, 0, s, false, t);
}

int decode_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
               void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
               const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
               void* ws, size_t ws_bytes, hipStream_t s, bool panels) {
    SplitK sk[kMaxProb]; int nb = 0;
    for (int i = 0; i < n_proj; ++i)
        if (base_of[i] == i) sk[nb++] = SplitK{U[i], r[i], (float*)(uintptr_t)t_off[i], nullptr, nullptr};
    Final f[kMaxProb];
    for (int i = 0; i < n_proj; ++i) {
        CacheDst cd = {nullptr, nullptr, 0, 1};
        if (kv && i == kv->k_index) cd = CacheDst{kv->k_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        if (kv && i == kv->v_index) cd = CacheDst{kv->v_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        f[i] = Final{(const void*)(uintptr_t)t_off[i], r[i], V[i], d_out[i], bias ? bias[i] : nullptr, out[i], cd};
    }
    return run_two_stage(x, d_in, M, sk, nb, f, n_proj, R, ws, ws_bytes, s, panels);
}

int decode_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
               const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
               int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
               void* ws, size_t ws_bytes, hipStream_t s, bool panels) {
    const int64_t r_gu = r_g + r_u, r_all = r_gu + r_d;
    const WsLayout L = ws_layout(ws, ws_bytes, M);
    const int G = fused_grid(((size_t)d * r_gu + (size_t)(r_g + r_u) * ffn + (size_t)ffn * r_d + (size_t)r_d * d) * 2);
    const bool fused = G > 0 && (size_t)M * r_all * 4 <= L.acc_bytes;
    // rank-space accumulators t[M, r_g + r_u + r_d] (fp32), the bf16 hidden rows h[M, ffn] and, for more
    // than 24 token rows in a fused launch, the bf16 copy t16 of t
    float* t = fused ? (float*)L.acc0 : (float*)L.staging;
    bf16_t* h = fused ? (bf16_t*)L.staging : (bf16_t*)(L.staging + align256((size_t)M * r_all * 4));
    bf16_t* t16 = (bf16_t*)(L.staging + align256((size_t)M * ffn * 2));
    const int64_t want = fused ? G : kUnfusedTiles;
    DStage sa, sb, sc, sd;
    const int ca = kCpl, cc = ca;   // both split-K stages share one tile width
    const size_t slot = (size_t)(M > 16 ? 32 : 16) * 16 * ca * 4;      // bytes of one partial tile
    bool use16 = fused && use_t16(M, (r_gu + r_d) / (16 * ca), 24);
    SplitK a, c;
    for (int attempt = 0; attempt < 2; ++attempt) {
        int ctile = 0;
        a = SplitK{U_gu, r_gu, t, use16 ? t16 : nullptr, use16 ? L.dec_part : nullptr};
        build_splitk(sa, x, d, M, d, &a, 1, r_all, want, ca, &ctile, panels);
        c = SplitK{U_d, r_d, t + r_gu, use16 ? t16 + r_gu : nullptr, use16 ? L.dec_part : nullptr};   // the two split-K stages take turns in the same slots
        build_splitk(sc, h, ffn, M, ffn, &c, 1, r_all, want, cc, &ctile, panels);
        const int most = sa.total_tiles > sc.total_tiles ? sa.total_tiles : sc.total_tiles;
        if (!use16 || (size_t)most * slot <= kDecPartBytes) break;
        use16 = false;
    }
    {   // gate/up: both products of a 64-column tile in one workgroup, full K
        sb.nprob = 1; sb.M = (int)M;
        DProb& p = sb.p[0]; zero_prob(p);
        p.W = (const bf16_t*)V_g; p.K = (int)r_g; p.lda = (int)r_all;
        p.W2 = (const bf16_t*)V_u; p.K2 = (int)r_u; p.lda2 = (int)r_all;
        if (use16) { p.A = t16; p.A2 = t16 + r_g; } else { p.A = t; p.A2 = t + r_g; }
        p.N = (int)ffn; p.Y = h; p.bias = (const bf16_t*)b_g; p.bias2 = (const bf16_t*)b_u;
        p.tiles_n = (int)(ffn / 64); p.KS = (int)r_g; p.tile_begin = 0;
        sb.total_tiles = p.tiles_n;
        set_wlayout(sb, 64, panels);
    }
    Final f = {use16 ? (const void*)(t16 + r_gu) : (const void*)(t + r_gu), r_d, V_d, d, b_d, out, {nullptr, nullptr, 0, 1}};
    const int cd = build_final(sd, &f, 1, r_all, M, panels);
    if (fused) {
        FusedMlpArgs fa;
        fa.fc = FusedCommon{L.ctrl, L.acc0, L.acc_bytes, use16 ? 0u : (uint32_t)(M * r_all), g_wait_limit, g_trace_buffer};
        const DStage* src[4] = {&sa, &sb, &sc, &sd};
        DStageT<1>* dst[4] = {&fa.a, &fa.b, &fa.c, &fa.d};
        for (int i = 0; i < 4; ++i) { dst[i]->p[0] = src[i]->p[0]; dst[i]->nprob = 1; dst[i]->M = (int)M; dst[i]->total_tiles = src[i]->total_tiles; }
        return decode_launch_fused_mlp(fa, ca, cc, cd, G, use16, s);
    }
    int st = fill_zero(t, (size_t)M * r_all * 4, s);
    if (st != LR_OK) return st;
    st = decode_launch_stage(sa, ca, false, EPI_ATOMIC, s);
    if (st != LR_OK) return st;
    st = decode_launch_stage(sb, 4, true, EPI_GATEUP, s);
    if (st != LR_OK) return st;
    st = decode_launch_stage(sc, cc, false, EPI_ATOMIC, s);
    if (st != LR_OK) return st;
    return decode_launch_stage(sd, cd, true, EPI_STORE, s);
}

}  // namespace lr
