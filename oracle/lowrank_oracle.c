/*
 * lowrank_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain fp64 CPU definition of what the factorized-linear hot path computes.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the HIP library.
 *
 * The paper (Section 3.1, "Unified runtime across checkpoint families") states
 * that every compressed linear layer is held as a pair of factors and is
 * "executed exactly" (Section 3.1, MLP paragraph): at run time there is no
 * approximation, so the result has a plain definition and the oracle is that
 * definition written out:
 *
 *     t[m, j] = sum_k x[m, k] * U[k, j]          k ascending
 *     y[m, n] = sum_j t[m, j] * V[j, n] + b[n]   j ascending
 *
 * All arrays are row-major, contiguous, IEEE binary64; nothing is rounded
 * between the two stages.  Rows of x are independent, so the outer loop over m
 * may run under OpenMP; that is the only parallelism.  There is no blocking,
 * fusion or re-association.
 *
 * The last two functions (rotary embedding, attention over the dense cache) define
 * the step that reads the cache this path writes (Section 3.1, decode attention).
 *
 * Every function below is pinned by tests/test_oracle_pins.py (brute force on
 * integer inputs, dense reconstruction, full-rank SVD recovery, closed forms,
 * invariants); nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* t[0..r) = xrow[0..d_in) * U[d_in, r]; each t[j] is accumulated for k = 0, 1, ... in order. */
static void row_times_matrix(const double *xrow, const double *W, double *out, int64_t K, int64_t N)
{
    for (int64_t n = 0; n < N; ++n) out[n] = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        const double a = xrow[k];
        const double *wrow = W + (size_t)k * (size_t)N;
        for (int64_t n = 0; n < N; ++n) out[n] += a * wrow[n];
    }
}

/*
 * Factorized linear layer (Section 3.1: a compressed linear is a factor pair).
 * y[M, d_out] = (x[M, d_in] * U[d_in, r]) * V[r, d_out] (+ bias[d_out] when bias != NULL).
 * r == 0 gives y = bias (or 0).  Returns 0, or -1 if scratch memory cannot be had.
 */
int lr_oracle_linear(const double *x, const double *U, const double *V, const double *bias,
                     double *y, int64_t M, int64_t d_in, int64_t r, int64_t d_out)
{
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *t = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        if (!t) { failed = 1; continue; }
        row_times_matrix(x + (size_t)m * (size_t)d_in, U, t, d_in, r);
        double *yrow = y + (size_t)m * (size_t)d_out;
        row_times_matrix(t, V, yrow, r, d_out);
        if (bias) for (int64_t n = 0; n < d_out; ++n) yrow[n] += bias[n];
        free(t);
    }
    return failed ? -1 : 0;
}

/*
 * Second stage only: y[M, d_out] = t[M, r] * V[r, d_out] (+ bias).  Used for the
 * shared-basis form (Section 3.1: a basis shared by grouped layers is "reused once"):
 * t = x * U_shared is formed once by lr_oracle_stage1 and fed to every V_i.
 */
int lr_oracle_stage1(const double *x, const double *U, double *t, int64_t M, int64_t d_in, int64_t r)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        row_times_matrix(x + (size_t)m * (size_t)d_in, U, t + (size_t)m * (size_t)r, d_in, r);
    return 0;
}

int lr_oracle_stage2(const double *t, const double *V, const double *bias, double *y,
                     int64_t M, int64_t r, int64_t d_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *yrow = y + (size_t)m * (size_t)d_out;
        row_times_matrix(t + (size_t)m * (size_t)r, V, yrow, r, d_out);
        if (bias) for (int64_t n = 0; n < d_out; ++n) yrow[n] += bias[n];
    }
    return 0;
}

/*
 * Dense KV-cache write (Section 3.1, attention paragraph: the current tokens' K and V
 * are reconstructed once and stored in a standard dense cache laid out
 * [batch, position, head, head_dim]).  Row (b*T + s) of `proj` ([B*T, n_heads*head_dim])
 * goes to cache[b, pos[b] + s, h, e] with column c = h*head_dim + e.  Pure index work.
 * Returns -2 if a position falls outside [0, S_max).
 */
int lr_oracle_cache_write(const double *proj, double *cache, const int32_t *pos,
                          int64_t B, int64_t T, int64_t S_max, int64_t n_heads, int64_t head_dim)
{
    const int64_t width = n_heads * head_dim;
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t s = 0; s < T; ++s) {
            const int64_t p = (int64_t)pos[b] + s;
            if (p < 0 || p >= S_max) return -2;
            const double *src = proj + (size_t)(b * T + s) * (size_t)width;
            for (int64_t h = 0; h < n_heads; ++h)
                for (int64_t e = 0; e < head_dim; ++e)
                    cache[(((size_t)b * (size_t)S_max + (size_t)p) * (size_t)n_heads + (size_t)h)
                              * (size_t)head_dim + (size_t)e] = src[h * head_dim + e];
        }
    }
    return 0;
}

/* SiLU(z) = z * sigmoid(z) = z / (1 + exp(-z)). */
static double silu(double z) { return z / (1.0 + exp(-z)); }

/*
 * Packed MLP (Section 3.1, MLP paragraph): the gate and up input-side factors are
 * concatenated offline into U_gu[d, r_g + r_u] (gate columns first); online there is one
 * wide projection whose result is split; output-side reconstruction and the down
 * projection are unchanged:
 *
 *   t_gu = x * U_gu;  g = t_gu[:, :r_g] * V_g + b_g;  u = t_gu[:, r_g:] * V_u + b_u;
 *   h = SiLU(g) .* u;  t_d = h * U_d;  out = t_d * V_d + b_d.
 *
 * x[M,d]  U_gu[d,r_g+r_u]  V_g[r_g,ffn]  V_u[r_u,ffn]  U_d[ffn,r_d]  V_d[r_d,d]  out[M,d].
 */
int lr_oracle_packed_mlp(const double *x, const double *U_gu, const double *V_g, const double *V_u,
                         const double *U_d, const double *V_d,
                         const double *b_g, const double *b_u, const double *b_d,
                         double *out, int64_t M, int64_t d, int64_t ffn,
                         int64_t r_g, int64_t r_u, int64_t r_d)
{
    int failed = 0;
    const int64_t r_gu = r_g + r_u;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *t_gu = (double *)malloc(sizeof(double) * (size_t)(r_gu > 0 ? r_gu : 1));
        double *g = (double *)malloc(sizeof(double) * (size_t)(ffn > 0 ? ffn : 1));
        double *u = (double *)malloc(sizeof(double) * (size_t)(ffn > 0 ? ffn : 1));
        double *t_d = (double *)malloc(sizeof(double) * (size_t)(r_d > 0 ? r_d : 1));
        if (!t_gu || !g || !u || !t_d) { failed = 1; free(t_gu); free(g); free(u); free(t_d); continue; }
        row_times_matrix(x + (size_t)m * (size_t)d, U_gu, t_gu, d, r_gu);
        row_times_matrix(t_gu, V_g, g, r_g, ffn);
        row_times_matrix(t_gu + r_g, V_u, u, r_u, ffn);
        for (int64_t f = 0; f < ffn; ++f) {
            const double gv = g[f] + (b_g ? b_g[f] : 0.0);
            const double uv = u[f] + (b_u ? b_u[f] : 0.0);
            g[f] = silu(gv) * uv;                       /* h, stored over g */
        }
        row_times_matrix(g, U_d, t_d, ffn, r_d);
        double *orow = out + (size_t)m * (size_t)d;
        row_times_matrix(t_d, V_d, orow, r_d, d);
        if (b_d) for (int64_t n = 0; n < d; ++n) orow[n] += b_d[n];
        free(t_gu); free(g); free(u); free(t_d);
    }
    return failed ? -1 : 0;
}

/*
 * Offline prepack (Section 3.1, MLP paragraph and Figure 3): concatenate n input-side
 * factors U_i[d_in, r_i] along the rank axis into packed[d_in, sum r_i].  Works on raw
 * elements of `elem_bytes` bytes each: index work only, so the result is bit-exact.
 */
int lr_oracle_pack_concat(const void *const *U_list, const int64_t *r_list, int n, int64_t d_in,
                          int64_t elem_bytes, void *packed)
{
    int64_t R = 0;
    for (int i = 0; i < n; ++i) R += r_list[i];
    int64_t col0 = 0;
    for (int i = 0; i < n; ++i) {
        const unsigned char *src = (const unsigned char *)U_list[i];
        for (int64_t k = 0; k < d_in; ++k)
            memcpy((unsigned char *)packed + ((size_t)k * (size_t)R + (size_t)col0) * (size_t)elem_bytes,
                   src + (size_t)k * (size_t)r_list[i] * (size_t)elem_bytes,
                   (size_t)r_list[i] * (size_t)elem_bytes);
        col0 += r_list[i];
    }
    return 0;
}

/*
 * Rotary position embedding in the "rotate-half" pairing that LLaMA checkpoints in the common
 * exchange format use (the paper's aligned baseline "applies external RoPE", Section 4; the paper
 * does not write the formula -- this is the standard one): for head dimension E, pair
 * (i, i + E/2), i < E/2, is rotated by the angle p * base^(-2i/E):
 *     y[i]       = x[i] * cos(a) - x[i + E/2] * sin(a)
 *     y[i + E/2] = x[i + E/2] * cos(a) + x[i] * sin(a)
 * x, y: [rows, H * E] (column h * E + e); p[rows]: position of each row.  y may equal x.
 */
int lr_oracle_rope(const double *x, double *y, const int64_t *p, int64_t rows, int64_t H, int64_t E, double base)
{
    if (E % 2 != 0) return -2;
    const int64_t half = E / 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t h = 0; h < H; ++h) {
            const double *xi = x + ((size_t)r * (size_t)H + (size_t)h) * (size_t)E;
            double *yi = y + ((size_t)r * (size_t)H + (size_t)h) * (size_t)E;
            for (int64_t i = 0; i < half; ++i) {
                const double a = (double)p[r] * pow(base, -2.0 * (double)i / (double)E);
                const double c = cos(a), sn = sin(a);
                const double lo = xi[i], hi = xi[i + half];
                yi[i] = lo * c - hi * sn;
                yi[i + half] = hi * c + lo * sn;
            }
        }
    return 0;
}

/*
 * Decode attention over the dense KV cache (Section 3.1, decode-attention paragraph: the present
 * token's q/k/v are reconstructed once, the past is read from a standard dense cache
 * [batch, position, head, head_dim]; Section 4: RoPE is applied to q and k).
 *
 * q[B*T, H*E]: the queries of T new tokens per sequence; row b*T+s sits at position pos[b]+s.
 * k_cache, v_cache[B, S_max, H, E]: rows pos[b] .. pos[b]+T-1 already hold the new tokens' raw k and v.
 * If rope_base > 0, first the T new k rows of every sequence are rotated IN PLACE (the cache then
 * holds rotated keys, as it does for all earlier positions) and the queries are rotated (not in
 * place).  Then, for every row and head, with n = pos[b]+s+1 visible positions (causal):
 *     score[j] = scale * sum_e q[e] * K[b, j, h, e],  j < n
 *     w[j]     = exp(score[j] - max_j score) / sum_j exp(score[j] - max_j score)
 *     out[e]   = sum_j w[j] * V[b, j, h, e]
 * Returns 0; -1 if a position falls outside [0, S_max); -2 for odd E with RoPE.
 */
int lr_oracle_decode_attention(const double *q, double *k_cache, const double *v_cache, const int32_t *pos,
                               double *out, int64_t B, int64_t T, int64_t S_max, int64_t H, int64_t E,
                               double scale, double rope_base)
{
    const int64_t d = H * E;
    for (int64_t b = 0; b < B; ++b)
        if (pos[b] < 0 || (int64_t)pos[b] + T > S_max) return -1;
    double *qr = (double *)malloc(sizeof(double) * (size_t)(B * T > 0 ? B * T : 1) * (size_t)(d > 0 ? d : 1));
    if (!qr) return -3;
    if (rope_base > 0.0) {
        if (E % 2 != 0) { free(qr); return -2; }
        for (int64_t b = 0; b < B; ++b)
            for (int64_t s = 0; s < T; ++s) {
                const int64_t p = (int64_t)pos[b] + s;
                double *krow = k_cache + ((size_t)b * (size_t)S_max + (size_t)p) * (size_t)d;
                lr_oracle_rope(krow, krow, &p, 1, H, E, rope_base);
                lr_oracle_rope(q + (size_t)(b * T + s) * (size_t)d, qr + (size_t)(b * T + s) * (size_t)d, &p, 1, H, E, rope_base);
            }
    } else {
        memcpy(qr, q, sizeof(double) * (size_t)(B * T) * (size_t)d);
    }
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < B * T; ++r) {
        const int64_t b = r / T, s = r - b * T;
        const int64_t n = (int64_t)pos[b] + s + 1;
        double *w = (double *)malloc(sizeof(double) * (size_t)n);
        if (!w) { failed = 1; continue; }
        for (int64_t h = 0; h < H; ++h) {
            const double *qh = qr + (size_t)r * (size_t)d + (size_t)h * (size_t)E;
            double mx = -INFINITY;
            for (int64_t j = 0; j < n; ++j) {
                const double *kj = k_cache + (((size_t)b * (size_t)S_max + (size_t)j) * (size_t)H + (size_t)h) * (size_t)E;
                double sc = 0.0;
                for (int64_t e = 0; e < E; ++e) sc += qh[e] * kj[e];
                w[j] = sc * scale;
                if (w[j] > mx) mx = w[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j < n; ++j) { w[j] = exp(w[j] - mx); den += w[j]; }
            double *oh = out + (size_t)r * (size_t)d + (size_t)h * (size_t)E;
            for (int64_t e = 0; e < E; ++e) oh[e] = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                const double *vj = v_cache + (((size_t)b * (size_t)S_max + (size_t)j) * (size_t)H + (size_t)h) * (size_t)E;
                const double wj = w[j] / den;
                for (int64_t e = 0; e < E; ++e) oh[e] += wj * vj[e];
            }
        }
        free(w);
    }
    free(qr);
    return failed ? -3 : 0;
}

int lr_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
