// Host-side planning of the decode phase: how each stage is cut into workgroup tiles.
// Integer logic only; every function enqueues kernels on the caller's stream and returns.
#include <stdlib.h>
#include <string.h>
#include "decode.hpp"

namespace lr {

static int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

// Fast-path shape rule: rows ride on one or two 16-row MFMA blocks, K in 32-row blocks, N in
// 64-column tiles.
bool decode_shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && M <= 32 && K >= 32 && (K % 32) == 0 && N >= 64 && (N % 64) == 0 &&
           K < (1 << 24) && N < (1 << 24);
}

static int pick_cpl(int64_t N) {
    const int forced = env_int("LOWRANK_DECODE_CPL", 0);
    if ((forced == 4) || (forced == 8 && N % 128 == 0)) return forced;
    return 4;
}

// Split-K stage: rows per tile so that the stage has about `want` tiles; multiples of 128 rows
// (one 32-row block per wave), larger slices for more token rows to keep the number of fp32
// atomics (tiles_k * M * N) small against the weight bytes.
static int pick_ks(int64_t K, int64_t tiles_n_total, int64_t M) {
    const int forced = env_int("LOWRANK_DECODE_KS", 0);
    if (forced >= 32 && forced % 32 == 0) return forced;
    const int64_t want = env_int("LOWRANK_DECODE_TILES", 512);
    int64_t tk = (want + tiles_n_total - 1) / tiles_n_total;
    if (tk < 1) tk = 1;
    int64_t ks = (K + tk - 1) / tk;
    ks = ((ks + 127) / 128) * 128;
    const int64_t floor_ks = M > 8 ? 256 : 128;
    if (ks < floor_ks) ks = floor_ks;
    if (ks > K) ks = ((K + 31) / 32) * 32;
    return (int)ks;
}

static void zero_prob(DProb& p) { memset(&p, 0, sizeof(p)); p.T = 1; }

// t[M, ldc] += A[M, K] * W[K, N] for several (A shared) weight matrices, split along K.
struct SplitK { const void* W; int64_t N; float* C; };

static int stage_splitk(const void* A, bool a_f32, int64_t lda, int64_t M, int64_t K, const SplitK* items, int n,
                        int64_t ldc, hipStream_t s) {
    DStage st; st.nprob = n; st.M = (int)M;
    int64_t n_all = 0; bool all128 = true;
    for (int i = 0; i < n; ++i) { n_all += items[i].N; all128 = all128 && (items[i].N % 128 == 0); }
    const int cpl = all128 ? pick_cpl(128) : 4;
    const int nc = 16 * cpl;
    const int ks = pick_ks(K, n_all / nc, M);
    const int tk = (int)((K + ks - 1) / ks);
    int tile = 0;
    for (int i = 0; i < n; ++i) {
        DProb& p = st.p[i]; zero_prob(p);
        p.W = (const bf16_t*)items[i].W; p.A = A; p.K = (int)K; p.lda = (int)lda; p.N = (int)items[i].N;
        p.C = items[i].C; p.ldc = (int)ldc; p.tiles_n = (int)(items[i].N / nc); p.KS = ks; p.tile_begin = tile;
        tile += p.tiles_n * tk;
    }
    st.total_tiles = tile;
    return decode_launch_stage(st, cpl, a_f32, EPI_ATOMIC, s);
}

struct Final { const float* T; int64_t r; const void* V; int64_t N; const void* bias; void* Y; CacheDst cd; };

// y_i[M, N_i] = t_i[M, r_i] * V_i[r_i, N_i] + bias_i, full K per tile, epilogue writes bf16.
static int stage_final(const Final* items, int n, int64_t ldt, int64_t M, hipStream_t s) {
    DStage st; st.nprob = n; st.M = (int)M;
    bool all128 = true;
    for (int i = 0; i < n; ++i) all128 = all128 && (items[i].N % 128 == 0);
    const int cpl = all128 ? pick_cpl(128) : 4;
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
    return decode_launch_stage(st, cpl, true, EPI_STORE, s);
}

int decode_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                  int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, hipStream_t s) {
    float* t = (float*)((char*)ws + kHeaderBytes);
    int st = fill_zero(t, (size_t)M * r * 4, s);
    if (st != LR_OK) return st;
    SplitK sk = {U, r, t};
    st = stage_splitk(x, false, d_in, M, d_in, &sk, 1, r, s);
    if (st != LR_OK) return st;
    Final f = {t, r, V, d_out, bias, y, {nullptr, nullptr, 0, 1}};
    return stage_final(&f, 1, r, M, s);
}

int decode_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
               void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
               const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
               void* ws, hipStream_t s) {
    float* t = (float*)((char*)ws + kHeaderBytes);
    int st = fill_zero(t, (size_t)M * R * 4, s);
    if (st != LR_OK) return st;
    SplitK sk[kMaxProb]; int nb = 0;
    for (int i = 0; i < n_proj; ++i)
        if (base_of[i] == i) sk[nb++] = SplitK{U[i], r[i], t + t_off[i]};
    st = stage_splitk(x, false, d_in, M, d_in, sk, nb, R, s);
    if (st != LR_OK) return st;
    Final f[kMaxProb];
    for (int i = 0; i < n_proj; ++i) {
        CacheDst cd = {nullptr, nullptr, 0, 1};
        if (kv && i == kv->k_index) cd = CacheDst{kv->k_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        if (kv && i == kv->v_index) cd = CacheDst{kv->v_cache, kv->pos, kv->S_max, kv->tokens_per_seq};
        f[i] = Final{t + t_off[i], r[i], V[i], d_out[i], bias ? bias[i] : nullptr, out[i], cd};
    }
    return stage_final(f, n_proj, R, M, s);
}

int decode_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
               const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
               int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
               void* ws, hipStream_t s) {
    const int64_t r_gu = r_g + r_u, r_all = r_gu + r_d;
    char* base = (char*)ws + kHeaderBytes;
    float* t = (float*)base;                                              // [M, r_g + r_u + r_d] fp32
    bf16_t* h = (bf16_t*)(base + 2 * align256((size_t)M * (size_t)r_all * 4));   // [M, ffn] bf16
    int st = fill_zero(t, (size_t)M * r_all * 4, s);
    if (st != LR_OK) return st;
    // stage A: t_gu = x U_gu
    SplitK a = {U_gu, r_gu, t};
    st = stage_splitk(x, false, d, M, d, &a, 1, r_all, s);
    if (st != LR_OK) return st;
    // stage B: h = SiLU(t_g V_g + b_g) * (t_u V_u + b_u)
    {
        DStage sg; sg.nprob = 1; sg.M = (int)M;
        DProb& p = sg.p[0]; zero_prob(p);
        p.W = (const bf16_t*)V_g; p.A = t; p.K = (int)r_g; p.lda = (int)r_all;
        p.W2 = (const bf16_t*)V_u; p.A2 = t + r_g; p.K2 = (int)r_u; p.lda2 = (int)r_all;
        p.N = (int)ffn; p.Y = h; p.bias = (const bf16_t*)b_g; p.bias2 = (const bf16_t*)b_u;
        p.tiles_n = (int)(ffn / 64); p.KS = (int)r_g; p.tile_begin = 0;
        sg.total_tiles = p.tiles_n;
        st = decode_launch_stage(sg, 4, true, EPI_GATEUP, s);
        if (st != LR_OK) return st;
    }
    // stage C: t_d = h U_d
    SplitK c = {U_d, r_d, t + r_gu};
    st = stage_splitk(h, false, ffn, M, ffn, &c, 1, r_all, s);
    if (st != LR_OK) return st;
    // stage D: out = t_d V_d + b_d
    Final f = {t + r_gu, r_d, V_d, d, b_d, out, {nullptr, nullptr, 0, 1}};
    return stage_final(&f, 1, r_all, M, s);
}

}  // namespace lr
