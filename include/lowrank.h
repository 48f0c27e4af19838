/*
 * lowrank.h -- C ABI of liblowrank.so: the factorized linear layer y = (x U) V of an
 * SVD-compressed transformer on one AMD MI355X (gfx950), in a decode form (1..32 token
 * rows, bound by streaming the factors from HBM) and a prefill form (hundreds to thousands
 * of rows, bound by bf16 MFMA throughput).
 *
 * The operations are those of the paper's Section 3.1 ("FlashSVD v1.5 Design"):
 *   - every compressed linear layer is a pair of factors ("common native factorized
 *     representation", first paragraph);
 *   - attention reconstructs dense q/k/v for the current tokens only and stores K and V in a
 *     standard dense cache (second paragraph);
 *   - the MLP packs the gate and up input-side factors into one operand, runs one wide
 *     projection, splits the rank activations, and leaves output-side reconstruction and the
 *     down projection unchanged (third paragraph, Figure 3);
 *   - a basis shared by grouped layers stays physically shared and is used once (first
 *     paragraph);
 *   - prefill and decode run phase-specific kernels (abstract, Section 3).
 *
 * Conventions common to every entry point
 *   Layout     All matrices are row-major and contiguous: x[M, d_in], U[d_in, r], V[r, d_out],
 *              bias[d_out], y[M, d_out].  W ~ U V is [d_in, d_out] (row-vector convention).
 *   dtype      One element type per call (lr_dtype) for x, U, V, bias, outputs and caches.
 *              Accumulation is fp32 or wider; the output is rounded once (nearest-even).
 *   Pointers   Device pointers unless marked "host".  Inputs are never written.  Outputs must
 *              not alias inputs.  The caller owns every buffer; the library allocates and frees
 *              no device memory, never synchronises the stream and never changes the current
 *              device.  All work is enqueued on `stream` (a hipStream_t, NULL = default stream).
 *   Workspace  Caller-provided device scratch of at least lowrank_workspace_bytes(...) bytes,
 *              256-byte aligned.  Its contents on entry may be anything: the first call that finds no
 *              valid control block at its start prepares the workspace itself, on `stream`, without
 *              host synchronisation (lowrank_workspace_init does the same ahead of time and is
 *              optional).  Between calls the library keeps state in the first 16 MiB + 20 KiB; the
 *              rest is scratch whose contents are undefined after a call.  One workspace may serve
 *              calls of any entry point, phase, shape and row count for which it is large enough.
 *              Two calls that share a workspace must be ordered on one stream; calls overlapping in
 *              time on one workspace race.
 *   Residency  Decode calls (up to 32 rows) normally run as ONE launch whose workgroups (one per
 *              compute unit) hand intermediates to each other through device-wide counters, and the
 *              prefill product with the longest K shares tiles between workgroups the same way.  Both
 *              need every workgroup of the launch resident at the same time, which holds when nothing
 *              else occupies compute units while the call runs: no kernel of another stream, process
 *              or graph branch.  A caller that cannot guarantee this says so once with
 *              lowrank_configure(LR_CFG_DEVICE_SHARED, 1); calls then use one launch per stage and no
 *              cross-workgroup waits.  If the guarantee is broken anyway, the waits are bounded: a
 *              workgroup that gives up writes NaN as its part of the result and raises the error word
 *              of the workspace, every later call on that workspace returns NaN results until it is
 *              prepared again (lowrank_workspace_init), and lowrank_workspace_status reports it.
 *   Errors     Return value is an lr_status: 0 on success, negative on error.  On a validation
 *              error nothing is launched.  lowrank_last_error() gives a thread-local message.
 *              No C++ exception crosses this boundary.
 *   Sizes      Any M, d_in, r, d_out >= 0 is legal.  M == 0 is a no-op.  r == 0 gives
 *              y = bias (or zeros).  The fast kernels need bf16 and 16-byte aligned pointers;
 *              decode (up to 32 rows): every d_in and r a multiple of 32, every r and d_out a multiple
 *              of 64; prefill: every d_in and r a multiple of 64, every r and d_out a multiple of 128.
 *              Anything else takes a slower generic kernel with the same results to rounding.
 */
#ifndef LOWRANK_H
#define LOWRANK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Element type of a call.  LR_BF16_PANELS is bf16 whose FACTOR operands (every U, V, U_gu, V_g, V_u, U_d, V_d argument) are
 * stored as 64-column panels (lowrank_pack_panels) instead of row-major; x, biases, outputs and caches are as with LR_BF16.
 * Only lowrank_linear, lowrank_qkv and lowrank_packed_mlp accept it, and only where they run the decode kernels (decode
 * phase, up to 32 rows, fast-path shapes, aligned operands); any other such call returns LR_ERR_UNSUPPORTED and launches
 * nothing.  Results are those of the same call on row-major factors, bit for bit in the same launch shape.
 */
typedef enum { LR_F32 = 0, LR_BF16 = 1, LR_BF16_PANELS = 2 } lr_dtype;

/* Phase of serving (paper: "phase-specific kernels").  AUTO picks DECODE when M <= 32. */
typedef enum { LR_PHASE_DECODE = 0, LR_PHASE_PREFILL = 1, LR_PHASE_AUTO = 2 } lr_phase;

typedef enum {
    LR_OK = 0,
    LR_ERR_NULL = -1,        /* a required pointer is NULL */
    LR_ERR_SHAPE = -2,       /* negative or inconsistent sizes */
    LR_ERR_DTYPE = -3,       /* unknown lr_dtype */
    LR_ERR_ALIGN = -4,       /* workspace not 256-byte aligned */
    LR_ERR_PHASE = -5,       /* unknown lr_phase */
    LR_ERR_WORKSPACE = -6,   /* workspace missing or too small */
    LR_ERR_LAUNCH = -7,      /* the HIP runtime refused a launch (message has the HIP error) */
    LR_ERR_UNSUPPORTED = -8  /* combination not available */
} lr_status;

typedef enum { LR_OP_LINEAR = 0, LR_OP_QKV = 1, LR_OP_PACKED_MLP = 2, LR_OP_DECODE_ATTENTION = 3 } lr_op;

/*
 * One factorized linear layer (Section 3.1, first paragraph):
 *     y[M, d_out] = (x[M, d_in] * U[d_in, r]) * V[r, d_out]  (+ bias[d_out] if bias != NULL)
 */
int lowrank_linear(const void *x, const void *U, const void *V, const void *bias /* nullable */,
                   void *y, int64_t M, int64_t d_in, int64_t r, int64_t d_out,
                   int dtype /* lr_dtype */, int phase /* lr_phase */,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * lowrank_linear for callers that cannot provide or allocate a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same operation and same results to rounding; the rank-space rows
 * live in a 512 KiB scratch area built into the library image (one copy per GPU, held until the process ends), so
 * M * r may be at most 131072 (e.g. 32 rows at rank 4096); larger calls return LR_ERR_WORKSPACE and launch nothing.
 * Nothing is allocated or freed, here or in any routine it calls.  Up to 32 rows of bf16 with aligned operands run the
 * decode kernels as one launch per stage (no cross-workgroup waits, so no residency requirement); every other call
 * runs the generic kernels.  All calls on one GPU share that GPU's scratch area: calls that overlap in time on one
 * GPU race, even on different streams; order them.  The area is cleared on the stream at the start of each call.
 */
int lowrank_linear_noalloc(const void *x, const void *U, const void *V, const void *bias /* nullable */,
                           void *y, int64_t M, int64_t d_in, int64_t r, int64_t d_out,
                           int dtype /* lr_dtype */, void *stream);

/*
 * Where the K and V projections of lowrank_qkv are written besides `out` (Section 3.1,
 * second paragraph: a standard dense KV cache; layout [batch, position, head, head_dim]).
 * The M rows of x are B sequences of tokens_per_seq consecutive tokens (M = B * tokens_per_seq).
 * Row b*tokens_per_seq + s of projection k_index goes to
 *     k_cache[b, pos[b] + s, h, e]   for column c = h * head_dim + e,
 * likewise v_index -> v_cache.  d_out of both projections must equal n_heads * head_dim.
 * pos is a DEVICE array of B int32; the caller guarantees 0 <= pos[b] and
 * pos[b] + tokens_per_seq <= S_max (rows that would fall outside are skipped, never written
 * out of bounds).  B * S_max must be below 2^31 (LR_ERR_SHAPE otherwise).  This struct itself
 * lives in HOST memory.
 */
typedef struct {
    void *k_cache;             /* device, [B, S_max, n_heads, head_dim], element type = dtype */
    void *v_cache;             /* device, same shape */
    const int32_t *pos;        /* device, int32[B] */
    int64_t B, S_max, n_heads, head_dim, tokens_per_seq;
    int32_t k_index, v_index;  /* which projection is K, which is V (0-based) */
} lr_kv_target;

/*
 * n_proj (1..8) factorized projections of the same x (Q, K, V of one attention block; or the
 * layers that share one basis):
 *     out[i][M, d_out[i]] = (x * U[i]) * V[i] (+ bias[i])
 * U, V, bias, out, r, d_out are HOST arrays of n_proj entries; U[i], V[i], out[i] are device
 * pointers.  bias may be NULL (no projection has a bias) or hold NULL entries.  out[i] may be
 * NULL when projection i is wanted only in the cache.  If U[i] == U[j] (same pointer, hence
 * r[i] == r[j]) the product x * U[i] is formed once and reused: the shared-basis form.
 * kv may be NULL.
 */
int lowrank_qkv(const void *x, const void *const *U, const void *const *V,
                const void *const *bias /* nullable */, void *const *out,
                const int64_t *r, const int64_t *d_out, int n_proj,
                int64_t M, int64_t d_in, const lr_kv_target *kv /* nullable */,
                int dtype, int phase, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Packed MLP (Section 3.1, third paragraph).  U_gu[d, r_g + r_u] is the offline-packed
 * operand [U_gate | U_up], gate columns first:
 *     t    = x[M, d] * U_gu
 *     g    = t[:, :r_g] * V_g[r_g, ffn] + b_g         u = t[:, r_g:] * V_u[r_u, ffn] + b_u
 *     h    = SiLU(g) .* u,   SiLU(z) = z / (1 + exp(-z))
 *     out[M, d] = (h * U_d[ffn, r_d]) * V_d[r_d, d] + b_d
 * b_g, b_u (ffn entries) and b_d (d entries) are nullable.  g, u and h never reach `out`'s
 * caller; h may be staged in the workspace.
 */
int lowrank_packed_mlp(const void *x, const void *U_gu, const void *V_g, const void *V_u,
                       const void *U_d, const void *V_d,
                       const void *b_g, const void *b_u, const void *b_d,
                       void *out, int64_t M, int64_t d, int64_t ffn,
                       int64_t r_g, int64_t r_u, int64_t r_d,
                       int dtype, int phase, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decode attention over the dense KV cache that lowrank_qkv writes (Section 3.1, second paragraph:
 * the present token's q/k/v are reconstructed once and the history is read from a standard dense
 * cache; Section 4: rotary position embedding on q and k).  kv describes the caches as for
 * lowrank_qkv (k_index / v_index are ignored): M = B * tokens_per_seq token rows, row
 * b*tokens_per_seq + s stands at position p = pos[b] + s, and rows pos[b] .. pos[b]+tokens_per_seq-1
 * of both caches already hold the new tokens' k and v (every head: multi-head attention, one K/V
 * head per query head).
 *   1. If rope_base > 0: the new k rows are rotated IN PLACE in k_cache (so that the cache holds
 *      rotated keys at every position, as after earlier calls) and the queries are rotated (q itself
 *      is not written).  Pairing "rotate-half": for i < head_dim/2 and a = p * rope_base^(-2i/head_dim),
 *      (x[i], x[i + head_dim/2]) -> (x[i] cos a - x[i + head_dim/2] sin a, x[i + head_dim/2] cos a + x[i] sin a).
 *      Call this exactly once per new token after lowrank_qkv has written its raw k.
 *   2. For every row and head h, over the n = p + 1 visible positions j (causal):
 *      out[row, h*head_dim + e] = sum_j softmax_j(scale * <q_h, K[b, j, h, :]>) * V[b, j, h, e].
 * q and out are [M, n_heads * head_dim], element type = dtype; out must not alias q.  head_dim must be
 * even and at most 1024.  The caller guarantees 0 <= pos[b] and pos[b] + tokens_per_seq <= S_max
 * (positions outside are clamped for memory safety, results for such rows are meaningless).
 * Workspace: lowrank_workspace_bytes(LR_OP_DECODE_ATTENTION, ...); pure scratch, no preparation needed.
 * Bound by streaming the visible K and V rows once; meant for the 1..32 rows of a decode step.
 */
int lowrank_decode_attention(const void *q, const lr_kv_target *kv, void *out, float scale, float rope_base,
                             int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Prefill attention over the dense KV cache: the same operation as lowrank_decode_attention, steps 1 and 2
 * word for word (causal attention of the new tokens' queries over cache positions [0, pos[b] + s], new key rows
 * rotated in place when rope_base > 0), organised for the hundreds to thousands of new tokens per sequence of
 * a prefill pass (Section 3.1, second paragraph; Section 4): tiles of 128 query rows x 64 keys on the bf16
 * matrix cores with an online softmax, so that the work is bound by arithmetic, not by re-reading the cache per
 * row.  Arguments as for lowrank_decode_attention; no workspace.  Supported: dtype LR_BF16, head_dim 128,
 * 16-byte aligned q / out / caches; anything else returns LR_ERR_UNSUPPORTED (lowrank_decode_attention accepts
 * every shape).  out must not alias q.
 */
int lowrank_prefill_attention(const void *q, const lr_kv_target *kv, void *out, float scale, float rope_base,
                              int dtype, void *stream);

/*
 * Prefill attention with FACTORIZED queries (Section 3.1, second paragraph: the prefill path consumes the low-rank factors
 * directly and avoids materialising dense Q/K/V in memory; K and V still go to the dense cache through lowrank_qkv, which
 * is what decode reads later).  Same operation as lowrank_prefill_attention with
 *     q[M, n_heads * head_dim] = t_q[M, r_q] * V_q[r_q, n_heads * head_dim] (+ b_q),
 * where every workgroup rebuilds its own 128 x 128 tile of q on the matrix cores, rounds it to the element type (as a
 * stored q would be) and rotates / scales it in registers: the dense q never exists in memory.  t_q are the rank-space rows
 * x * U_q of the new tokens (lowrank_rank_project), row-major; b_q (n_heads * head_dim entries) may be NULL.
 * Supported: dtype LR_BF16, head_dim 128, r_q a multiple of 64, 16-byte aligned operands; otherwise LR_ERR_UNSUPPORTED.
 * No workspace.  out must not alias t_q.
 */
int lowrank_prefill_factorized_attention(const void *t_q, const void *V_q, const void *b_q /* nullable */, int64_t r_q,
                                         const lr_kv_target *kv, void *out, float scale, float rope_base,
                                         int dtype, void *stream);

/*
 * First half of a factorized linear layer on its own (Section 3.1, first paragraph: the layer is a factor pair):
 *     t[M, r] = x[M, d_in] * U[d_in, r], rounded once to the element type.
 * These are the rank-space rows that lowrank_prefill_factorized_attention consumes.  Workspace as for
 * lowrank_workspace_bytes(LR_OP_LINEAR, M, d_in, r, 0, ...).
 */
int lowrank_rank_project(const void *x, const void *U, void *t, int64_t M, int64_t d_in, int64_t r,
                         int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Offline prepack (Section 3.1, third paragraph; Figure 3): concatenate n (1..8) factors
 * U_list[i][d_in, r_list[i]] along the rank axis into U_packed[d_in, sum r_list].  U_list and
 * r_list are HOST arrays; the matrices are device memory.  Pure data movement: bit-exact.
 */
int lowrank_pack_concat(const void *const *U_list, const int64_t *r_list, int n, int64_t d_in,
                        int dtype, void *U_packed, void *stream);

/*
 * Offline prepack for decode (Section 3.1, first paragraph: factors are "loaded into a common native factorized
 * representation"; the layout is the library's choice): re-lay a row-major bf16 factor W[K, N], N a multiple of 64, as
 * N / 64 panels of 64 columns,
 *     W_panels[((n / 64) * K + k) * 64 + n % 64] = W[k * N + n],
 * so that the 64-column tile a decode workgroup streams is one contiguous run instead of K row segments of 128 bytes
 * N * 2 bytes apart.  Panels of a concatenation are the concatenation of the panels (ranks that are multiples of 64).
 * dtype must be LR_BF16; W and W_panels are distinct 16-byte aligned device buffers of K * N elements.  Pure data
 * movement: bit-exact.  A server keeps this copy for decode beside the row-major one that prefill reads.
 */
int lowrank_pack_panels(const void *W, int64_t K, int64_t N, void *W_panels, int dtype, void *stream);

/*
 * Workspace size in bytes (pure host function, no GPU needed).  Meaning of the size arguments:
 *   LR_OP_LINEAR      d_in, r_total = r,                 d_out
 *   LR_OP_QKV         d_in, r_total = sum of r[i],       d_out = sum of d_out[i]
 *   LR_OP_PACKED_MLP  d_in = d, r_total = r_g + r_u + r_d, d_out = ffn
 *   LR_OP_DECODE_ATTENTION  d_in = n_heads * head_dim, r_total = n_heads, d_out unused
 * Returns 0 for invalid arguments.  The value covers both phases whatever `phase` says and grows with M: a
 * workspace sized for M rows serves every call of the same kind with fewer rows.  Every workspace of the three
 * linear entry points starts with a fixed part of 16 MiB + 20 KiB (control block, flags, partial-tile area, two
 * accumulator areas) followed by scratch for the rank-space and hidden rows; for more than 32 rows another 64 MiB
 * hold the partial sums that workgroups of a prefill product sharing one tile's K range hand to each other.
 */
size_t lowrank_workspace_bytes(int op, int64_t M, int64_t d_in, int64_t r_total, int64_t d_out,
                               int dtype, int phase);

/*
 * Optional: prepare a workspace ahead of its first use, or again after lowrank_workspace_status reported a
 * failure (enqueues two small launches on `stream`; no synchronisation).  The decode-attention workspace keeps
 * no state between calls and needs no preparation.
 */
int lowrank_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, the only function here that SYNCHRONISES `stream`: reads the workspace's control
 * block back and returns LR_OK, or LR_ERR_LAUNCH if a bounded device-side wait gave up (see "Residency"
 * above; that call's results are NaN where they could not be completed).
 */
int lowrank_workspace_status(const void *workspace, void *stream);

/*
 * Process-wide settings (host only; not thread-safe against concurrent calls of the entry points).
 *   LR_CFG_DEVICE_SHARED  value != 0: other work may occupy compute units while calls run, so no launch may
 *                         depend on all of its workgroups being resident (see "Residency").  Default 0.
 *   LR_CFG_WAIT_LIMIT     number of polls after which a device-side wait gives up (default 2^20, about half a
 *                         second).  A robustness knob for callers that prefer an early NaN to a long stall.
 */
typedef enum { LR_CFG_DEVICE_SHARED = 0, LR_CFG_WAIT_LIMIT = 1 } lr_config;
int lowrank_configure(int option, int64_t value);

/*
 * Name of the kernel family the dispatcher picks for a call of this shape, e.g.
 * "decode_mfma", "prefill_mfma", "generic" (pure host function; static storage); with LR_BF16_PANELS
 * "decode_mfma" or "unsupported".
 * `aligned` is nonzero when every pointer of the call is 16-byte aligned.
 */
const char *lowrank_plan_name(int op, int64_t M, int64_t d_in, int64_t r_total, int64_t d_out,
                              int dtype, int phase, int aligned);

/*
 * Tile selection of the prefill phase (Section 3: phase-specific kernels; heterogeneous ranks multiply the GEMM
 * shapes a layer runs): for n_products (1..8) dense products C[M, N] = A[M, K] * B[K, N] of one launch -- the
 * rank-space products x U_i of one call, or its reconstruction products t_i V_i -- the workgroup tile
 * tile_m x tile_n (256x256, 256x192 or 128x128) and how the K range is divided: *share_k = 0 (every tile runs its whole K),
 * 1 (long K, few tiles, thousands of rows -- the h U_d product of the MLP: workgroups share a tile's K range and hand
 * partial tiles to the one that holds its first k-step) or n >= 2 (few rows and a long K -- the rank-space products of a
 * prompt of some hundred tokens: K is cut into n chunks that run as products of one launch, a second small launch adds
 * their fp32 partial sums).  gate_up != 0 asks for the fused gate/up kernel (always 128x128, two accumulator sets).  Pure host function, deterministic, no GPU needed.  LR_ERR_UNSUPPORTED when
 * the shape is outside the matrix-core rule (K % 64 == 0, N % 128 == 0).
 */
int lowrank_prefill_tile(int64_t M, int64_t K, int64_t N, int n_products, int gate_up,
                         int *tile_m, int *tile_n, int *share_k);

const char *lowrank_last_error(void);   /* thread-local, static storage, never NULL */
const char *lowrank_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOWRANK_H */
