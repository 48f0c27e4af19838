// Host-side planning of the prefill phase: each entry point is a short chain of GEMM launches whose
// rank-space intermediate T (and, for the MLP, the hidden rows H) are bf16 matrices in the staging
// part of the workspace.  Integer logic only.
#include <string.h>
#include "decode.hpp"
#include "prefill.hpp"

namespace lr {

static void zero_pprob(PProb& p) { memset(&p, 0, sizeof(p)); p.T = 1; }
static void init_pargs(PArgs& a, int64_t M, const WsLayout& L) {
    memset(&a, 0, sizeof(a));
    a.M = (int)M;
    a.sk_flags = L.sk_flags; a.sk_slots = L.sk_slots; a.err = &L.ctrl->error;
}

int prefill_qkv(const void* x, const void* const* U, const void* const* V, const void* const* bias,
                void* const* out, const int64_t* r, const int64_t* d_out, int n_proj, const int* base_of,
                const int64_t* t_off, int64_t R, int64_t M, int64_t d_in, const lr_kv_target* kv,
                void* ws, size_t ws_bytes, hipStream_t s) {
    const WsLayout L = ws_layout(ws, ws_bytes, M);
    bf16_t* T = (bf16_t*)L.staging;                 // [M, R] bf16
    PArgs a1; init_pargs(a1, M, L);
    for (int i = 0; i < n_proj; ++i) {
        if (base_of[i] != i) continue;
        PProb& p = a1.p[a1.nprob++]; zero_pprob(p);
        p.A = (const bf16_t*)x; p.lda = (int)d_in; p.B = (const bf16_t*)U[i]; p.K = (int)d_in; p.N = (int)r[i];
        p.C = T + t_off[i]; p.ldc = (int)R;
        if (p.N / 128 > a1.tiles_n_max) a1.tiles_n_max = p.N / 128;
    }
    int st = prefill_launch(a1, PEPI_STORE, s);
    if (st != LR_OK) return st;
    PArgs a2; init_pargs(a2, M, L); a2.nprob = n_proj;
    for (int i = 0; i < n_proj; ++i) {
        PProb& p = a2.p[i]; zero_pprob(p);
        p.A = T + t_off[i]; p.lda = (int)R; p.B = (const bf16_t*)V[i]; p.K = (int)r[i]; p.N = (int)d_out[i];
        p.C = (bf16_t*)out[i]; p.ldc = (int)d_out[i]; p.bias = (const bf16_t*)(bias ? bias[i] : nullptr);
        if (kv && (i == kv->k_index || i == kv->v_index)) {
            p.cache = (i == kv->k_index) ? kv->k_cache : kv->v_cache;
            p.pos = kv->pos; p.S_max = (int)kv->S_max; p.T = (int)kv->tokens_per_seq;
        }
        if (p.N / 128 > a2.tiles_n_max) a2.tiles_n_max = p.N / 128;
    }
    return prefill_launch(a2, PEPI_STORE, s);
}

// t[M, r] = x U as one dense product, rounded to bf16 (the rank-space rows handed to the factorized attention kernel)
int prefill_rank_project(const void* x, const void* U, void* t, int64_t M, int64_t d_in, int64_t r,
                         void* ws, size_t ws_bytes, hipStream_t s) {
    const WsLayout L = ws_layout(ws, ws_bytes, M);
    PArgs a; init_pargs(a, M, L); a.nprob = 1;
    PProb& p = a.p[0]; zero_pprob(p);
    p.A = (const bf16_t*)x; p.lda = (int)d_in; p.B = (const bf16_t*)U; p.K = (int)d_in; p.N = (int)r;
    p.C = (bf16_t*)t; p.ldc = (int)r;
    a.tiles_n_max = p.N / 128;
    return prefill_launch(a, PEPI_STORE, s);
}

int prefill_linear(const void* x, const void* U, const void* V, const void* bias, void* y,
                   int64_t M, int64_t d_in, int64_t r, int64_t d_out, void* ws, size_t ws_bytes, hipStream_t s) {
    const void* Us[1] = {U}; const void* Vs[1] = {V}; const void* bs[1] = {bias}; void* outs[1] = {y};
    const int64_t rs[1] = {r}, ns[1] = {d_out}, toff[1] = {0};
    const int base_of[1] = {0};
    return prefill_qkv(x, Us, Vs, bs, outs, rs, ns, 1, base_of, toff, r, M, d_in, nullptr, ws, ws_bytes, s);
}

int prefill_mlp(const void* x, const void* U_gu, const void* V_g, const void* V_u, const void* U_d,
                const void* V_d, const void* b_g, const void* b_u, const void* b_d, void* out,
                int64_t M, int64_t d, int64_t ffn, int64_t r_g, int64_t r_u, int64_t r_d,
                void* ws, size_t ws_bytes, hipStream_t s) {
    const int64_t r_gu = r_g + r_u, r_all = r_gu + r_d;
    const WsLayout L = ws_layout(ws, ws_bytes, M);
    bf16_t* T = (bf16_t*)L.staging;                                         // [M, r_g + r_u + r_d] bf16
    bf16_t* H = (bf16_t*)(L.staging + align256((size_t)M * r_all * 2));     // [M, ffn] bf16
    PArgs a; init_pargs(a, M, L); a.nprob = 1;
    {   // T_gu = x U_gu
        PProb& p = a.p[0]; zero_pprob(p);
        p.A = (const bf16_t*)x; p.lda = (int)d; p.B = (const bf16_t*)U_gu; p.K = (int)d; p.N = (int)r_gu; p.C = T; p.ldc = (int)r_all;
        a.tiles_n_max = p.N / 128;
        int st = prefill_launch(a, PEPI_STORE, s);
        if (st != LR_OK) return st;
    }
    {   // H = SiLU(T_g V_g + b_g) * (T_u V_u + b_u)
        PProb& p = a.p[0]; zero_pprob(p);
        p.A = T; p.lda = (int)r_all; p.B = (const bf16_t*)V_g; p.K = (int)r_g;
        p.A2 = T + r_g; p.lda2 = (int)r_all; p.B2 = (const bf16_t*)V_u; p.K2 = (int)r_u;
        p.N = (int)ffn; p.C = H; p.ldc = (int)ffn; p.bias = (const bf16_t*)b_g; p.bias2 = (const bf16_t*)b_u;
        a.tiles_n_max = p.N / 128;
        int st = prefill_launch(a, PEPI_GATEUP, s);
        if (st != LR_OK) return st;
    }
    {   // T_d = H U_d
        PProb& p = a.p[0]; zero_pprob(p);
        p.A = H; p.lda = (int)ffn; p.B = (const bf16_t*)U_d; p.K = (int)ffn; p.N = (int)r_d; p.C = T + r_gu; p.ldc = (int)r_all;
        a.tiles_n_max = p.N / 128;
        int st = prefill_launch(a, PEPI_STORE, s);
        if (st != LR_OK) return st;
    }
    {   // out = T_d V_d + b_d
        PProb& p = a.p[0]; zero_pprob(p);
        p.A = T + r_gu; p.lda = (int)r_all; p.B = (const bf16_t*)V_d; p.K = (int)r_d; p.N = (int)d; p.C = (bf16_t*)out; p.ldc = (int)d;
        p.bias = (const bf16_t*)b_d;
        a.tiles_n_max = p.N / 128;
        return prefill_launch(a, PEPI_STORE, s);
    }
}

}  // namespace lr
