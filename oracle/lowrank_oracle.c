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
