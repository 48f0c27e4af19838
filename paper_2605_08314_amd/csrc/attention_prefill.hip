// Prefill attention over the dense KV cache (paper Section 3.1, attention paragraph: the present tokens' K/V go
// to a standard dense cache [batch, position, head, head_dim]; Section 4: RoPE on q and k): causal softmax
// attention of thousands of new tokens per sequence on the matrix cores, bf16, head_dim 128.
// Same operation as the decode-attention kernels (token s of sequence b sees cache positions [0, pos[b] + s]),
// organised for compute instead of for streaming:
//
//   k_rope_new_keys   rotates the new key rows in place in the cache (the projection call stores them raw).
//   k_attn_prefill    one workgroup (4 waves) per (128 query rows, head, sequence); a wave owns 32 query rows and
//                     walks the visible keys 64 at a time.  Everything is computed transposed, so that a lane owns
//                     ONE query row throughout and every softmax statistic is a per-lane scalar:
//                       S^T[key, row] = K Q^T      A = K rows from LDS (16-byte reads), B = the wave's rotated queries
//                                                  (registers, loaded once), v_mfma_f32_32x32x16_bf16
//                       online softmax             lane (row l % 32, half l / 32) holds 32 of the 64 scores of its row
//                       O^T[e, row] += V^T P^T     A = V^T through the transposing LDS read ds_read_b64_tr_b16,
//                                                  B = the probabilities straight from the score registers: the
//                                                  accumulator layout hands a lane keys {8a + 4h .. +3}, so one
//                                                  16-key MFMA step takes keys {16a' + 4h ..+3, 16a' + 8 + 4h ..+3}
//                                                  and the V^T operand is read in the same order.
//                     K and V tiles (64 x 128) are double-buffered in LDS (direct-to-LDS loads, swizzled 16-byte pieces).
#include "attention.hpp"

namespace lr {

typedef __bf16 pbf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 pbf16x2_t __attribute__((ext_vector_type(2)));
typedef float pf32x2_t __attribute__((ext_vector_type(2)));
typedef float pf32x16_t __attribute__((ext_vector_type(16)));
typedef short ps16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) ps16x4_t lds_ps16x4_t;

struct PAttnArgs {
    const bf16_t* q; bf16_t* k_cache; const bf16_t* v_cache; const int32_t* pos; bf16_t* out;
    int B, T, H, S_max;
    int ldq;                 // elements between query rows (H * 128)
    float scale_log2e;       // softmax scale * log2(e)
    double rope_base;        // <= 0: no rotation
    // factorized queries (k_attn_prefill<true>): q = t_q V_q (+ b_q), rebuilt tile by tile inside the kernel; q above is unused
    const bf16_t* tq; const bf16_t* vq; const bf16_t* bq; int r_q;     // t_q [B * T, r_q], V_q [r_q, H * 128], b_q [H * 128] or NULL
};

constexpr float kLazyExp = 8.f;      // a row's reference maximum is moved when a score exceeds it by more than this (log2 units)
constexpr int PA_E = 128, PA_BQ = 128, PA_BK = 64;
// K and V tiles in LDS: 64 rows of 256 bytes each, unpadded (they arrive by direct-to-LDS loads, 1 KB = 4 rows per
// request), with the sixteen 16-byte pieces of row r stored at position piece ^ f(r), f(r) = ((r & 3) << 2) | ((r >> 2) & 3):
//   K is read 16 bytes per lane by 16 lanes of 16 consecutive rows, the same piece of each: f is a bijection on the 4
//     row bits, so the 16 reads fall into 16 different bank groups;
//   V is read by the transposing read, whose 32 lanes of a pass touch 4 consecutive rows x 64 bytes (4 pieces): the
//     high two bits of f are r & 3, so the four rows use four different 64-byte quarters of the bank space.
// The permutation costs nothing: a lane of the load writes LDS position (request base + lane) and simply fetches the
// global piece that belongs there.
constexpr int PA_TROW = 256;
constexpr int PA_KTILE = PA_BK * PA_TROW;                // 16384
constexpr int PA_TILE = 2 * PA_KTILE;                    // one buffer: K tile | V tile
constexpr int PA_ROW = 272;                              // bytes per row of the output staging at the end (256 + 16)
__host__ __device__ constexpr int pa_f(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// 64 lanes x 16 bytes: global (sbase + voff[lane]) -> LDS (lds_byte + 16 * lane); counted by vmcnt.  (Inline assembly, so
// that the compiler does not put a full vmcnt(0) in front of every LDS read that might alias the destination; the waits
// are written out below.  voff registers are never rewritten while requests are in flight.)
__device__ __forceinline__ void pa_dma16(uint32_t lds_byte, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_byte), "v"(voff), "s"(sbase) : "memory");
}
__device__ __forceinline__ const char* pa_uniform_ptr(const char* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>((uintptr_t)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ uint32_t pa_pack2(float lo, float hi) {
    union { pbf16x2_t v; uint32_t u; } x;
    x.v = __builtin_convertvector(pf32x2_t{lo, hi}, pbf16x2_t);
    return x.u;
}
// acc + lo + hi of a packed bf16 pair (v_dot2_f32_bf16 with a pair of ones)
__device__ __forceinline__ float pa_sum2(uint32_t pair, float acc) {
    union { uint32_t u; pbf16x2_t v; } x, one;
    x.u = pair; one.u = 0x3f803f80u;
    return __builtin_amdgcn_fdot2_f32_bf16(x.v, one.v, acc, false);
}
__device__ __forceinline__ pbf16x8_t pa_frag(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    union { uint32_t u[4]; pbf16x8_t v; } x;
    x.u[0] = a; x.u[1] = b; x.u[2] = c; x.u[3] = d;
    return x.v;
}

// cos / sin of position * base^(-2i/128): angle and range reduction in fp64, the functions in fp32 (the same
// arithmetic as the decode path, so a key rotated here equals a key rotated there bit for bit)
__device__ __forceinline__ void pa_cos_sin(long long p, double theta, float& c, float& sn) {
    const double ang = (double)p * theta;
    const double k = rint(ang * 0.15915494309189535);
    const double red = fma(-k, 1.2246467991473532e-16 * 2.0, fma(-k, 6.283185307179586, ang));
    sincosf((float)red, &sn, &c);
}

// One thread rotates 8 pairs (i .. i + 7, i + 64 .. i + 71) of one (token, head): two 16-byte loads and stores.
__global__ void __launch_bounds__(256) k_rope_new_keys(PAttnArgs a) {
    __shared__ double s_theta[64];
    if (threadIdx.x < 64) s_theta[threadIdx.x] = exp2(-2.0 * (double)threadIdx.x / 128.0 * log2(a.rope_base));
    __syncthreads();
    const long long total = (long long)a.B * a.T * a.H * 8;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
        const int i0 = (int)(idx & 7) * 8;
        const int h = (int)((idx >> 3) % a.H);
        const long long r = (idx >> 3) / a.H;
        const int b = (int)(r / a.T), s = (int)(r - (long long)b * a.T);
        const long long p = (long long)a.pos[b] + s;
        if (p < 0 || p >= a.S_max) continue;
        bf16_t* k = a.k_cache + (((size_t)b * a.S_max + (size_t)p) * a.H + h) * PA_E + i0;
        const uint4 lo4 = *reinterpret_cast<const uint4*>(k), hi4 = *reinterpret_cast<const uint4*>(k + 64);
        const uint32_t lo[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
        uint32_t olo[4], ohi[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            bf16_t rl[2], rh[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float c, sn;
                pa_cos_sin(p, s_theta[i0 + 2 * w + t], c, sn);
                const double klo = (double)__uint_as_float(t ? (lo[w] & 0xffff0000u) : (lo[w] << 16));
                const double khi = (double)__uint_as_float(t ? (hi[w] & 0xffff0000u) : (hi[w] << 16));
                rl[t] = f32_to_bf16((float)(klo * (double)c - khi * (double)sn));
                rh[t] = f32_to_bf16((float)(khi * (double)c + klo * (double)sn));
            }
            olo[w] = (uint32_t)rl[0] | ((uint32_t)rl[1] << 16);
            ohi[w] = (uint32_t)rh[0] | ((uint32_t)rh[1] << 16);
        }
        *reinterpret_cast<uint4*>(k) = make_uint4(olo[0], olo[1], olo[2], olo[3]);
        *reinterpret_cast<uint4*>(k + 64) = make_uint4(ohi[0], ohi[1], ohi[2], ohi[3]);
    }
}

// FACT: the queries arrive in rank space (Section 3.1, attention paragraph: prefill consumes the low-rank factors without
// materialising dense Q in memory).  The workgroup first forms its 128 x 128 tile of Q = t_q V_q (+ b_q) on the matrix cores
// -- transposed, Q^T = V_q^T t_q^T, with the very machinery of O^T += V^T P^T: 64-row tiles of V_q (row-major, [k][e], the
// geometry of a V cache tile) arrive by direct-to-LDS loads and are read through the transposing LDS read, the rank-space
// row of a lane is the other operand straight from memory -- rounds it to bf16 as a stored q would be, and hands it to the
// rotation below through LDS.
template <bool FACT>
__global__ void __launch_bounds__(256, 2) k_attn_prefill(PAttnArgs a) {
    __shared__ __attribute__((aligned(1024))) char lds[2 * PA_TILE];     // K0 | V0 | K1 | V1
    __shared__ double s_theta[64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, hh = lane >> 5;
    const int nqb = (a.T + PA_BQ - 1) / PA_BQ;
    // Workgroups go to the 8 XCDs (each with its own L2) round-robin by index.  All query blocks of one (sequence, head)
    // walk the same keys from position 0 upwards, so they are given to ONE XCD, next to each other in its sequence of
    // workgroups: they then run at the same time and share each K / V tile in that L2 (with query blocks of a head spread
    // over all XCDs the kernel fetched 1.8 GB from memory for 0.19 GB of operands).  Long blocks first.
    const int xcd = (int)(blockIdx.x & 7), j = (int)(blockIdx.x >> 3);
    const int group = xcd + 8 * (j / nqb);                    // (sequence, head) pair
    if (group >= a.H * a.B) return;                           // padding of the last round of groups
    const int qb = nqb - 1 - j % nqb;
    const int head = group % a.H;
    const int b = group / a.H;
    const int s0 = qb * PA_BQ;
    const long long pos_b = a.pos[b];
    // visible keys of the block: [0, n_keys)
    long long nk = pos_b + (s0 + PA_BQ < a.T ? s0 + PA_BQ : a.T);
    if (nk > a.S_max) nk = a.S_max;
    if (nk < 0) nk = 0;
    const int n_keys = (int)nk;
    const int nkb = (n_keys + PA_BK - 1) / PA_BK;

    // ---- this lane's query row, rotated, as the B operand of S^T = K Q^T: step ks holds e = 16 ks + 8 hh .. + 7 ----
    const int s_row = s0 + wave * 32 + li;                     // token index inside the sequence
    const bool row_ok = s_row < a.T;
    const int s_clamped = row_ok ? s_row : a.T - 1;            // rows past T repeat the last one; never stored
    const int p_row = (int)(pos_b + s_clamped);                // position of the row
    pbf16x8_t qf[8];
    {
        uint4 raw[8];
        if constexpr (FACT) {
            const uint32_t lds0q = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)lds);
            const size_t vrow_bytes = (size_t)a.H * PA_E * 2;                  // bytes between rows of V_q
            const char* vqbase = reinterpret_cast<const char*>(a.vq + (size_t)head * PA_E);
            const bf16_t* tqrow = a.tq + ((size_t)b * a.T + (size_t)s_clamped) * a.r_q + 4 * hh;
            const int nkt = a.r_q / PA_BK;
            uint32_t voffq[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = 16 * wave + 4 * q + (lane >> 4);
                voffq[q] = (uint32_t)r * (uint32_t)vrow_bytes + (uint32_t)(((lane & 15) ^ pa_f(r & 15)) * 16);
            }
            const int wave_q = __builtin_amdgcn_readfirstlane(wave);
            // transposing-read offsets (as for the V operand of the main loop, see below)
            uint32_t q_lo[4], q_hi[4];
            {
                const int sl = lane & 15, g1 = (lane >> 4) & 1;
                const int rlo = 4 * hh + (sl >> 2), rhi = rlo + 8;
                const int lowp = 2 * g1 + ((sl & 3) >> 1);
#pragma unroll
                for (int eb = 0; eb < 4; ++eb) {
                    q_lo[eb] = (uint32_t)rlo * PA_TROW + (uint32_t)((((4 * eb + lowp) ^ pa_f(rlo & 15)) * 16) + (sl & 1) * 8);
                    q_hi[eb] = (uint32_t)rhi * PA_TROW + (uint32_t)((((4 * eb + lowp) ^ pa_f(rhi & 15)) * 16) + (sl & 1) * 8);
                }
            }
            pf32x16_t acc_q[4];
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_q[eb][i] = 0.f;
#define PA_REQUEST_VQ(KT, BUF)                                                                                 \
            do {                                                                                               \
                const char* vs_ = pa_uniform_ptr(vqbase + (size_t)(KT) * PA_BK * vrow_bytes);                  \
                const uint32_t d_ = lds0q + (uint32_t)(BUF) * PA_TILE + PA_KTILE + (uint32_t)wave_q * 4096u;   \
                _Pragma("unroll") for (int q = 0; q < 4; ++q) pa_dma16(d_ + 1024u * q, voffq[q], vs_);         \
            } while (0)
            if (nkt > 0) PA_REQUEST_VQ(0, 0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            for (int kt = 0; kt < nkt; ++kt) {
                const int buf = kt & 1;
                if (kt + 1 < nkt) PA_REQUEST_VQ(kt + 1, buf ^ 1);
                const char* vt = lds + buf * PA_TILE + PA_KTILE;
                // this lane's rank-space values of the tile, in the k order of the transposed operand: step a2 takes
                // k = 64 kt + 16 a2 + {4 hh .. + 3} and {8 + 4 hh .. + 3}
                uint2 tlo[4], thi[4];
#pragma unroll
                for (int a2 = 0; a2 < 4; ++a2) {
                    const bf16_t* tp = tqrow + PA_BK * kt + 16 * a2;
                    tlo[a2] = *reinterpret_cast<const uint2*>(tp);
                    thi[a2] = *reinterpret_cast<const uint2*>(tp + 8);
                }
#pragma unroll
                for (int a2 = 0; a2 < 4; ++a2) {
                    const pbf16x8_t tf = pa_frag(tlo[a2].x, tlo[a2].y, thi[a2].x, thi[a2].y);
#pragma unroll
                    for (int eb = 0; eb < 4; ++eb) {
                        union { struct { ps16x4_t lo, hi; } h; pbf16x8_t v; } x;
                        const char* vp = vt + (uint32_t)(16 * a2) * PA_TROW;
                        x.h.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ps16x4_t*)(vp + q_lo[eb]));
                        x.h.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ps16x4_t*)(vp + q_hi[eb]));
                        acc_q[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, tf, acc_q[eb], 0, 0, 0);
                    }
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next tile has landed
                __syncthreads();
            }
#undef PA_REQUEST_VQ
            // Q^T of this lane: e = 32 eb + 8 g4 + 4 hh .. + 3 of query row li; + bias, rounded to bf16 (as a stored q is),
            // through the wave's own rows of the staging area, and back as whole 16-byte pieces of the row
            char* stage = lds + wave * (32 * PA_ROW);
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int e = eb * 32 + 8 * g4 + 4 * hh;
                    float bq4[4] = {0.f, 0.f, 0.f, 0.f};
                    if (a.bq) {
                        const uint2 braw = *reinterpret_cast<const uint2*>(a.bq + (size_t)head * PA_E + e);
                        bq4[0] = __uint_as_float(braw.x << 16); bq4[1] = __uint_as_float(braw.x & 0xffff0000u);
                        bq4[2] = __uint_as_float(braw.y << 16); bq4[3] = __uint_as_float(braw.y & 0xffff0000u);
                    }
                    const uint2 o = make_uint2(pa_pack2(acc_q[eb][4 * g4 + 0] + bq4[0], acc_q[eb][4 * g4 + 1] + bq4[1]),
                                               pa_pack2(acc_q[eb][4 * g4 + 2] + bq4[2], acc_q[eb][4 * g4 + 3] + bq4[3]));
                    *reinterpret_cast<uint2*>(stage + li * PA_ROW + e * 2) = o;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // LDS traffic of a wave completes in order; these rows are this wave's
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) raw[ks] = *reinterpret_cast<const uint4*>(stage + li * PA_ROW + (16 * ks + 8 * hh) * 2);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __syncthreads();                                            // everyone holds its row: the area may be overwritten
        } else {
            const bf16_t* qrow = a.q + ((size_t)b * a.T + (size_t)s_clamped) * a.ldq + (size_t)head * PA_E + 8 * hh;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) raw[ks] = *reinterpret_cast<const uint4*>(qrow + 16 * ks);
        }
        if (a.rope_base > 0.0) {
            // cos / sin of the block's 128 positions x 64 frequencies, computed once by all threads into LDS (the tiles
            // are not loaded yet): [row][i] as float2
            if (tid < 64) s_theta[tid] = exp2(-2.0 * (double)tid / 128.0 * log2(a.rope_base));
            __syncthreads();
            float2* cs = reinterpret_cast<float2*>(lds);
            for (int t = tid; t < PA_BQ * 64; t += 256) {
                const int r = t >> 6, i = t & 63;
                const int sr = s0 + r < a.T ? s0 + r : a.T - 1;
                float c, sn;
                pa_cos_sin(pos_b + sr, s_theta[i], c, sn);
                cs[t] = make_float2(c, sn);
            }
            __syncthreads();
            const float2* my = cs + (wave * 32 + li) * 64 + 8 * hh;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const uint32_t lo[4] = {raw[ks].x, raw[ks].y, raw[ks].z, raw[ks].w};
                const uint32_t hi[4] = {raw[ks + 4].x, raw[ks + 4].y, raw[ks + 4].z, raw[ks + 4].w};
                uint32_t olo[4], ohi[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    float rl[2], rh[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float2 c_s = my[16 * ks + 2 * w + t];           // pair (i, i + 64), i = 16 ks + 8 hh + 2 w + t
                        const float ql = __uint_as_float(t ? (lo[w] & 0xffff0000u) : (lo[w] << 16));
                        const float qh = __uint_as_float(t ? (hi[w] & 0xffff0000u) : (hi[w] << 16));
                        rl[t] = (float)((double)ql * (double)c_s.x - (double)qh * (double)c_s.y) * a.scale_log2e;
                        rh[t] = (float)((double)qh * (double)c_s.x + (double)ql * (double)c_s.y) * a.scale_log2e;
                    }
                    olo[w] = pa_pack2(rl[0], rl[1]);
                    ohi[w] = pa_pack2(rh[0], rh[1]);
                }
                qf[ks] = pa_frag(olo[0], olo[1], olo[2], olo[3]);
                qf[ks + 4] = pa_frag(ohi[0], ohi[1], ohi[2], ohi[3]);
            }
            __syncthreads();                                    // the table has been read: the tiles may overwrite it
        } else {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint32_t rw[4] = {raw[ks].x, raw[ks].y, raw[ks].z, raw[ks].w};
                uint32_t o[4];
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    o[w] = pa_pack2(__uint_as_float(rw[w] << 16) * a.scale_log2e, __uint_as_float(rw[w] & 0xffff0000u) * a.scale_log2e);
                qf[ks] = pa_frag(o[0], o[1], o[2], o[3]);
            }
        }
    }

    // ---- K / V tile requests: wave w, request q covers rows 16 w + 4 q + lane / 16 of the tile, LDS piece lane % 16 ----
    const size_t row_bytes = (size_t)a.H * PA_E * 2;                       // bytes between cache positions
    const char* kbase = reinterpret_cast<const char*>(a.k_cache + ((size_t)b * a.S_max * a.H + head) * PA_E);
    const char* vbase = reinterpret_cast<const char*>(a.v_cache + ((size_t)b * a.S_max * a.H + head) * PA_E);
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)lds);
    const int last_rows = n_keys - (nkb - 1) * PA_BK;                       // rows of the last tile that exist (1..64)
    uint32_t voff[4], voff_last[4];                                         // loop-invariant: see pa_dma16
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = 16 * wave + 4 * q + (lane >> 4);
        const int piece = (lane & 15) ^ pa_f(r & 15);
        const int rl = r < last_rows ? r : last_rows - 1;                   // rows past the end repeat the last one (masked below)
        voff[q] = (uint32_t)r * (uint32_t)row_bytes + (uint32_t)piece * 16u;
        voff_last[q] = (uint32_t)rl * (uint32_t)row_bytes + (uint32_t)piece * 16u;
    }
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#define PA_REQUEST_TILE(KB, BUF)                                                                               \
    do {                                                                                                       \
        const char* ks_ = pa_uniform_ptr(kbase + (size_t)(KB) * PA_BK * row_bytes);                            \
        const char* vs_ = pa_uniform_ptr(vbase + (size_t)(KB) * PA_BK * row_bytes);                            \
        const uint32_t d_ = lds0 + (uint32_t)(BUF) * PA_TILE + (uint32_t)wave_u * 4096u;                       \
        if ((KB) == nkb - 1) {                                                                                 \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                    \
                pa_dma16(d_ + 1024u * q, voff_last[q], ks_);                                                   \
                pa_dma16(d_ + PA_KTILE + 1024u * q, voff_last[q], vs_);                                        \
            }                                                                                                  \
        } else {                                                                                               \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                    \
                pa_dma16(d_ + 1024u * q, voff[q], ks_);                                                        \
                pa_dma16(d_ + PA_KTILE + 1024u * q, voff[q], vs_);                                             \
            }                                                                                                  \
        }                                                                                                      \
    } while (0)

    pf32x16_t acc_o[4];
#pragma unroll
    for (int eb = 0; eb < 4; ++eb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_o[eb][i] = 0.f;
    float l_run = 0.f;
    pf32x16_t negm;                       // minus the reference maximum of this lane's query row, in every element
#pragma unroll
    for (int i = 0; i < 16; ++i) negm[i] = 0.f;

    if (nkb > 0) PA_REQUEST_TILE(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // this lane's fixed LDS offsets
    // K operand: row 32 kbk + li, logical piece 2 ks + hh
    uint32_t k_off[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_off[ks] = (uint32_t)li * PA_TROW + (uint32_t)(((2 * ks + hh) ^ pa_f(li & 15)) * 16);
    // V operand through the transposing read: inside a group of 16 lanes, source lane s hands in key row s / 4 and columns
    // 4 (s % 4)..; the group (lane / 16) & 1 covers columns 16 .. 31 of the 32-column block eb, the half hh selects the
    // keys: rows 16 a2 + 4 hh + s / 4 (first four keys of the step) and + 8 (last four).  Logical piece of the 8 bytes:
    // 4 eb + 2 g1 + (s % 4) / 2; its position: high bits eb ^ (row & 3), low bits ^ ((row >> 2) & 3).
    uint32_t v_lo[4], v_hi[4];
    {
        const int sl = lane & 15, g1 = (lane >> 4) & 1;
        const int rlo = 4 * hh + (sl >> 2), rhi = rlo + 8;
        const int lowp = 2 * g1 + ((sl & 3) >> 1);
#pragma unroll
        for (int eb = 0; eb < 4; ++eb) {
            v_lo[eb] = (uint32_t)rlo * PA_TROW + (uint32_t)((((4 * eb + lowp) ^ pa_f(rlo & 15)) * 16) + (sl & 1) * 8);
            v_hi[eb] = (uint32_t)rhi * PA_TROW + (uint32_t)((((4 * eb + lowp) ^ pa_f(rhi & 15)) * 16) + (sl & 1) * 8);
        }
    }

    for (int kb = 0; kb < nkb; ++kb) {
        const int buf = kb & 1;
        if (kb + 1 < nkb) PA_REQUEST_TILE(kb + 1, buf ^ 1);      // that buffer was last read before the previous barrier
        const char* kt = lds + buf * PA_TILE;
        const char* vt = kt + PA_KTILE;

        // S^T = K Q^T for the 64 keys of the tile: two 32-key blocks
        // (the two blocks' accumulation chains alternate, so that consecutive MFMAs do not depend on each other)
        // The accumulation starts from -m_ref of the lane's query row (negm, sixteen copies: the C operand of the first
        // MFMA), so the scores come out relative to the row's reference maximum and need no subtraction before exp2.
        pf32x16_t acc_s[2];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk) {
                const uint4 kv4 = *reinterpret_cast<const uint4*>(kt + k_off[ks] + kbk * 32 * PA_TROW);
                if (ks == 0) acc_s[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa_frag(kv4.x, kv4.y, kv4.z, kv4.w), qf[ks], negm, 0, 0, 0);
                else         acc_s[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa_frag(kv4.x, kv4.y, kv4.z, kv4.w), qf[ks], acc_s[kbk], 0, 0, 0);
            }
        }

        // scores of this lane: key = 64 kb + 32 kbk + 8 (i / 4) + 4 hh + i % 4
        const int key0 = kb * PA_BK + 4 * hh;
        // (the queries carry the softmax scale and log2 e, so the scores are exponents of 2 as they are)
        // tiles entirely below the diagonal of this wave's rows need no mask
        const bool need_mask = (long long)(kb * PA_BK + PA_BK - 1) > pos_b + s0 + wave * 32 || kb * PA_BK + PA_BK > n_keys;
        float m_blk = -INFINITY;
        if (need_mask) {
            const int limit = p_row < n_keys - 1 ? p_row : n_keys - 1;        // last visible key of this row
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int key = key0 + 32 * kbk + 8 * (i >> 2) + (i & 3);
                    const float sv = key <= limit ? acc_s[kbk][i] : -INFINITY;
                    acc_s[kbk][i] = sv;
                    m_blk = fmaxf(m_blk, sv);
                }
        } else {
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
                for (int i = 0; i < 16; ++i) m_blk = fmaxf(m_blk, acc_s[kbk][i]);
        }
        m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32));
        // The reference maximum of a row moves only when the tile's relative maximum exceeds 2^kLazyExp (the weights stay
        // below that bound in the meantime; numerator and denominator carry the same reference, so the result does not
        // depend on it) and on the first tile, where every row sees key 0 and takes that tile's maximum.  A wave in which
        // no row moves -- nearly all tiles -- skips the subtraction, the rescaling of O and the update of negm.
        const bool move = kb == 0 || m_blk > kLazyExp;
        if (__builtin_amdgcn_ballot_w64(move) != 0ull) {
            const float delta = (move && m_blk != -INFINITY) ? m_blk : 0.f;
            const float alpha = __builtin_amdgcn_exp2f(-delta);
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_s[kbk][i] -= delta;
            const float nm = negm[0] - delta;
#pragma unroll
            for (int i = 0; i < 16; ++i) negm[i] = nm;
            l_run *= alpha;
#pragma unroll
            for (int eb = 0; eb < 4; ++eb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc_o[eb][i] *= alpha;
        }
        // weights, rounded to bf16 pairs as the MFMA will see them; their sum by v_dot2_f32_bf16 against (1, 1): one
        // instruction per pair, and the denominator adds up exactly the values that enter the numerator
        uint32_t pp[2][8];
        float l_a = 0.f, l_b = 0.f;
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
            for (int g2 = 0; g2 < 8; ++g2) {
                const uint32_t w = pa_pack2(__builtin_amdgcn_exp2f(acc_s[kbk][2 * g2]), __builtin_amdgcn_exp2f(acc_s[kbk][2 * g2 + 1]));
                pp[kbk][g2] = w;
                if (g2 & 1) l_b = pa_sum2(w, l_b); else l_a = pa_sum2(w, l_a);
            }
        l_run += l_a + l_b;

        // O^T += V^T P^T, 16 keys per step: step a2 = 2 kbk + j takes score groups i / 4 = 2 j and 2 j + 1 of block kbk
#pragma unroll
        for (int a2 = 0; a2 < 4; ++a2) {
            const int kbk = a2 >> 1, j = a2 & 1;
            const pbf16x8_t pf = pa_frag(pp[kbk][4 * j + 0], pp[kbk][4 * j + 1], pp[kbk][4 * j + 2], pp[kbk][4 * j + 3]);
#pragma unroll
            for (int eb = 0; eb < 4; ++eb) {
                union { struct { ps16x4_t lo, hi; } h; pbf16x8_t v; } x;
                const char* vp = vt + (uint32_t)(16 * a2) * PA_TROW;
                x.h.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ps16x4_t*)(vp + v_lo[eb]));
                x.h.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ps16x4_t*)(vp + v_hi[eb]));
                acc_o[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, pf, acc_o[eb], 0, 0, 0);
            }
        }

        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next tile has landed
        __syncthreads();
    }

    // ---- normalise, transpose through LDS (the tiles are no longer needed), store whole rows ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    char* stage = lds + wave * (32 * PA_ROW);                               // 32 rows x 272 bytes per wave
#pragma unroll
    for (int eb = 0; eb < 4; ++eb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int e = eb * 32 + 8 * g4 + 4 * hh;
            const uint2 o = make_uint2(pa_pack2(acc_o[eb][4 * g4 + 0] * inv, acc_o[eb][4 * g4 + 1] * inv),
                                       pa_pack2(acc_o[eb][4 * g4 + 2] * inv, acc_o[eb][4 * g4 + 3] * inv));
            *reinterpret_cast<uint2*>(stage + li * PA_ROW + e * 2) = o;
        }
    // LDS traffic of a wave completes in order; the rows below belong to this wave only
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int ps = 0; ps < 8; ++ps) {
        const int r = 4 * ps + (lane >> 4), c16 = lane & 15;
        const int s_out = s0 + wave * 32 + r;
        const uint4 o = *reinterpret_cast<const uint4*>(stage + r * PA_ROW + c16 * 16);
        if (s_out < a.T)
            *reinterpret_cast<uint4*>(a.out + ((size_t)b * a.T + (size_t)s_out) * a.ldq + (size_t)head * PA_E + c16 * 8) = o;
    }
}

bool attn_prefill_ok(int dtype, int64_t E, bool aligned) { return dtype == LR_BF16 && aligned && E == 128; }

// q == NULL: factorized queries (tq, vq, bq, r_q)
int attn_prefill(const void* q, const lr_kv_target* kv, void* out, float scale, float rope_base, hipStream_t s,
                 const void* tq, const void* vq, const void* bq, int64_t r_q) {
    PAttnArgs a;
    a.tq = (const bf16_t*)tq; a.vq = (const bf16_t*)vq; a.bq = (const bf16_t*)bq; a.r_q = (int)r_q;
    a.q = (const bf16_t*)q; a.k_cache = (bf16_t*)kv->k_cache; a.v_cache = (const bf16_t*)kv->v_cache; a.pos = kv->pos;
    a.out = (bf16_t*)out;
    a.B = (int)kv->B; a.T = (int)kv->tokens_per_seq; a.H = (int)kv->n_heads; a.S_max = (int)kv->S_max;
    a.ldq = a.H * PA_E;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.rope_base = (double)rope_base;
    if (a.rope_base > 0.0) {
        const long long pairs = (long long)a.B * a.T * a.H * 8;
        const unsigned pg = (unsigned)((pairs + 255) / 256 < 8192 ? (pairs + 255) / 256 : 8192);
        hipLaunchKernelGGL(k_rope_new_keys, dim3(pg), dim3(256), 0, s, a);
    }
    const long long nqb = (a.T + PA_BQ - 1) / PA_BQ;
    const long long groups = (long long)a.H * a.B;
    const long long grid = 8 * nqb * ((groups + 7) / 8);       // see the index mapping in the kernel
    if (grid >= (1ll << 31)) { set_error("prefill attention: too many blocks"); return LR_ERR_SHAPE; }
    if (q) hipLaunchKernelGGL(k_attn_prefill<false>, dim3((unsigned)grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(k_attn_prefill<true>, dim3((unsigned)grid), dim3(256), 0, s, a);
    return launch_status("prefill attention");
}

}  // namespace lr
