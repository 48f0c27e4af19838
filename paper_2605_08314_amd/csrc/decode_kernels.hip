// Decode-phase kernels (1..32 token rows, bf16): each stage of the factorized layer is a skinny
// product C[M, N] (+)= A[M, K] * W[K, N] whose cost is streaming W from HBM exactly once.
//
// Work decomposition.  A workgroup (4 wavefronts of 64 lanes) owns one tile of W:
// KS rows x NC columns (NC = 16 * CPL, CPL = bf16 columns per lane: 4 -> 8-byte loads,
// 8 -> 16-byte loads).  Its waves take the tile's 32-row blocks round-robin.  For one block a lane
// (j = lane % 16, g = lane / 16) loads rows 8g..8g+7, columns CPL*j..CPL*j+CPL-1: every load
// instruction of the wave covers four full row segments of NC*2 bytes, i.e. coalesced and
// contiguous, straight from the row-major factor -- no repacking of U or V is needed.
//
// The token rows ride on the matrix cores: v_mfma_f32_16x16x32_bf16 with the activations as the
// 16-row operand (rows >= M are zero) and the weights as the 16-column operand.  That operand
// wants, per lane, 8 consecutive k for ONE column; the lane holds 8 k-rows x CPL columns, so a
// 16-bit transpose inside the lane (v_perm_b32) yields CPL operands, one per column offset b,
// and MFMA number b produces output columns {CPL*j + b}.  Lane (j, g) of result b holds rows
// 4g..4g+3 of column CPL*j + b, so a lane ends up with CPL contiguous output columns per row.
//
// The four waves' partial sums are combined through LDS in a fixed order; then either
//   EPI_ATOMIC : added into an fp32 accumulator in global memory (split-K stages: t = x U, t_d = h U_d),
//   EPI_STORE  : + bias, rounded to bf16, stored to y and/or scattered into the dense KV cache,
//   EPI_GATEUP : two products (gate, up) of the same columns -> SiLU(g + b_g) * (u + b_u) -> bf16 h.
#include "decode.hpp"

namespace lr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x8_t __attribute__((ext_vector_type(8)));

template <int CPL> struct WFrag { uint32_t w[8][CPL / 2]; };   // 8 k-rows x CPL bf16 columns
struct AFrag { uint32_t a[4]; };                               // 8 consecutive k of one token row

template <int CPL>
__device__ __forceinline__ void load_w(WFrag<CPL>& f, const bf16_t* __restrict__ W, int N, int row0, int col) {
    const bf16_t* p = W + (size_t)row0 * (size_t)N + col;
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        if constexpr (CPL == 8) {
            const uint4 v = *reinterpret_cast<const uint4*>(p + (size_t)a * N);
            f.w[a][0] = v.x; f.w[a][1] = v.y; f.w[a][2] = v.z; f.w[a][3] = v.w;
        } else {
            const uint2 v = *reinterpret_cast<const uint2*>(p + (size_t)a * N);
            f.w[a][0] = v.x; f.w[a][1] = v.y;
        }
    }
}

template <bool AF32>
__device__ __forceinline__ void load_a(AFrag& f, const void* __restrict__ A, int lda, int m, int M, int k) {
    if (m < M) {
        if constexpr (AF32) {
            const float* p = reinterpret_cast<const float*>(A) + (size_t)m * lda + k;
            const float4 lo = *reinterpret_cast<const float4*>(p);
            const float4 hi = *reinterpret_cast<const float4*>(p + 4);
            f.a[0] = (uint32_t)f32_to_bf16(lo.x) | ((uint32_t)f32_to_bf16(lo.y) << 16);
            f.a[1] = (uint32_t)f32_to_bf16(lo.z) | ((uint32_t)f32_to_bf16(lo.w) << 16);
            f.a[2] = (uint32_t)f32_to_bf16(hi.x) | ((uint32_t)f32_to_bf16(hi.y) << 16);
            f.a[3] = (uint32_t)f32_to_bf16(hi.z) | ((uint32_t)f32_to_bf16(hi.w) << 16);
        } else {
            const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(A) + (size_t)m * lda + k);
            f.a[0] = v.x; f.a[1] = v.y; f.a[2] = v.z; f.a[3] = v.w;
        }
    } else {
        f.a[0] = f.a[1] = f.a[2] = f.a[3] = 0u;
    }
}

__device__ __forceinline__ bf16x8_t as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    union { uint32_t u[4]; bf16x8_t v; } x;
    x.u[0] = a; x.u[1] = b; x.u[2] = c; x.u[3] = d;
    return x.v;
}

// acc[mb][b] += A_mb (16 x 32) * W(:, column offset b) (32 x 16 lanes)
template <int MB, int CPL>
__device__ __forceinline__ void mma_block(f32x4_t (&acc)[MB][CPL], const WFrag<CPL>& wf, const AFrag (&af)[MB]) {
    bf16x8_t av[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) av[mb] = as_bf16x8(af[mb].a[0], af[mb].a[1], af[mb].a[2], af[mb].a[3]);
#pragma unroll
    for (int b = 0; b < CPL; ++b) {
        const int q = b >> 1;
        const uint32_t sel = (b & 1) ? 0x07060302u : 0x05040100u;   // pick the high / low bf16 of each dword
        // dword s of the operand = { row 2s (low half), row 2s+1 (high half) } of column b
        const bf16x8_t bv = as_bf16x8(__builtin_amdgcn_perm(wf.w[1][q], wf.w[0][q], sel),
                                      __builtin_amdgcn_perm(wf.w[3][q], wf.w[2][q], sel),
                                      __builtin_amdgcn_perm(wf.w[5][q], wf.w[4][q], sel),
                                      __builtin_amdgcn_perm(wf.w[7][q], wf.w[6][q], sel));
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            acc[mb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mb], bv, acc[mb][b], 0, 0, 0);
    }
}

// This wave's share of rows [32*kb0, 32*kb1) of W: blocks kb0 + wave, kb0 + wave + 4, ...
template <int MB, int CPL, bool AF32, int PF>
__device__ __forceinline__ void mma_range(f32x4_t (&acc)[MB][CPL], const bf16_t* __restrict__ W, int N,
                                          const void* __restrict__ A, int lda, int M, int col, int kb0, int kb1,
                                          int wave, int j, int g) {
    WFrag<CPL> wf[PF];
    AFrag af[PF][MB];
    int blk = kb0 + wave;
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int bb = blk + 4 * p;
        if (bb < kb1) {
            load_w<CPL>(wf[p], W, N, 32 * bb + 8 * g, col);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) load_a<AF32>(af[p][mb], A, lda, 16 * mb + j, M, 32 * bb + 8 * g);
        }
    }
    for (; blk < kb1; blk += 4 * PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int bb = blk + 4 * p;
            if (bb < kb1) {
                mma_block<MB, CPL>(acc, wf[p], af[p]);
                const int nb = bb + 4 * PF;
                if (nb < kb1) {
                    load_w<CPL>(wf[p], W, N, 32 * nb + 8 * g, col);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) load_a<AF32>(af[p][mb], A, lda, 16 * mb + j, M, 32 * nb + 8 * g);
                }
            }
        }
    }
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

template <int CPL>
__device__ __forceinline__ void store_bf16_row(bf16_t* dst, const float (&v)[CPL]) {
    if constexpr (CPL == 8) {
        uint4 o; o.x = pack2(v[0], v[1]); o.y = pack2(v[2], v[3]); o.z = pack2(v[4], v[5]); o.w = pack2(v[6], v[7]);
        *reinterpret_cast<uint4*>(dst) = o;
    } else {
        uint2 o; o.x = pack2(v[0], v[1]); o.y = pack2(v[2], v[3]);
        *reinterpret_cast<uint2*>(dst) = o;
    }
}

template <int CPL>
__device__ __forceinline__ void load_bf16_row(float (&v)[CPL], const bf16_t* src) {
#pragma unroll
    for (int b = 0; b < CPL; ++b) v[b] = bf16_to_f32(src[b]);
}

// One workgroup tile, from loads to epilogue.  `red` is LDS scratch of red_floats<...>() floats.
template <int MB, int CPL, bool AF32, int EPI, int PF>
__device__ __forceinline__ void decode_tile(const DProb& P, int M, int lt, float4* __restrict__ red) {
    constexpr int NMAT = (EPI == EPI_GATEUP) ? 2 : 1;
    constexpr int NC = 16 * CPL;
    constexpr int Q = CPL / 4;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 15, g = lane >> 4;
    const int tn = lt % P.tiles_n, tk = lt / P.tiles_n;
    const int n0 = tn * NC;
    const int col = n0 + CPL * j;

    f32x4_t acc[NMAT][MB][CPL];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int b = 0; b < CPL; ++b) acc[mt][mb][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    {
        const int kb0 = tk * (P.KS >> 5);
        int kb1 = kb0 + (P.KS >> 5);
        if (kb1 > (P.K >> 5)) kb1 = P.K >> 5;
        mma_range<MB, CPL, AF32, PF>(acc[0], P.W, P.N, P.A, P.lda, M, col, kb0, kb1, wave, j, g);
    }
    if constexpr (NMAT == 2)
        mma_range<MB, CPL, AF32, PF>(acc[1], P.W2, P.N, P.A2, P.lda2, M, col, 0, P.K2 >> 5, wave, j, g);

    // cross-wave reduction through LDS: red[wave][slot = (mat*MB + mb)*4 + v][q][lane]
    constexpr int NSL = NMAT * MB * 4;
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    red[((wave * NSL + (mt * MB + mb) * 4 + v) * Q + q) * 64 + lane] =
                        make_float4(acc[mt][mb][4 * q + 0][v], acc[mt][mb][4 * q + 1][v],
                                    acc[mt][mb][4 * q + 2][v], acc[mt][mb][4 * q + 3][v]);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < MB; ++it) {
        const int pidx = tid + 256 * it;          // (mb, v, lane') triple
        const int sl = pidx >> 6, ln = pidx & 63;
        const int mb = sl >> 2, v = sl & 3;
        const int m = 16 * mb + 4 * (ln >> 4) + v;
        const int n = n0 + CPL * (ln & 15);
        float val[NMAT][CPL];
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                float4 s = red[((0 * NSL + mt * MB * 4 + sl) * Q + q) * 64 + ln];
#pragma unroll
                for (int w = 1; w < 4; ++w) {
                    const float4 o = red[((w * NSL + mt * MB * 4 + sl) * Q + q) * 64 + ln];
                    s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
                }
                val[mt][4 * q + 0] = s.x; val[mt][4 * q + 1] = s.y; val[mt][4 * q + 2] = s.z; val[mt][4 * q + 3] = s.w;
            }
        if (m < M) {
            if constexpr (EPI == EPI_ATOMIC) {
                float* c = P.C + (size_t)m * P.ldc + n;
#pragma unroll
                for (int b = 0; b < CPL; ++b) unsafeAtomicAdd(c + b, val[0][b]);
            } else if constexpr (EPI == EPI_STORE) {
                if (P.bias) {
                    float bv[CPL];
                    load_bf16_row<CPL>(bv, P.bias + n);
#pragma unroll
                    for (int b = 0; b < CPL; ++b) val[0][b] += bv[b];
                }
                if (P.Y) store_bf16_row<CPL>(P.Y + (size_t)m * P.N + n, val[0]);
                if (P.cache) {
                    const int bi = m / P.T, s = m - bi * P.T;
                    const int64_t pp = (int64_t)P.pos[bi] + s;
                    if (pp >= 0 && pp < P.S_max)
                        store_bf16_row<CPL>(reinterpret_cast<bf16_t*>(P.cache) + ((size_t)bi * P.S_max + (size_t)pp) * P.N + n, val[0]);
                }
            } else {
                float hv[CPL];
                float bg[CPL], bu[CPL];
#pragma unroll
                for (int b = 0; b < CPL; ++b) { bg[b] = 0.f; bu[b] = 0.f; }
                if (P.bias) load_bf16_row<CPL>(bg, P.bias + n);
                if (P.bias2) load_bf16_row<CPL>(bu, P.bias2 + n);
#pragma unroll
                for (int b = 0; b < CPL; ++b) hv[b] = silu_f32(val[0][b] + bg[b]) * (val[NMAT - 1][b] + bu[b]);
                store_bf16_row<CPL>(P.Y + (size_t)m * P.N + n, hv);
            }
        }
    }
}

template <int MB, int CPL, int EPI>
constexpr int red_float4s() { return 4 * ((EPI == EPI_GATEUP) ? 2 : 1) * MB * 4 * (CPL / 4) * 64; }

template <int MB, int CPL, bool AF32, int EPI, int PF>
__global__ void __launch_bounds__(256) k_decode_stage(DStage st) {
    __shared__ float4 red[red_float4s<MB, CPL, EPI>()];
    const int tile = blockIdx.x;
    int pi = 0;
#pragma unroll
    for (int i = 1; i < kMaxProb; ++i)
        if (i < st.nprob && tile >= st.p[i].tile_begin) pi = i;
    const DProb& P = st.p[pi];
    decode_tile<MB, CPL, AF32, EPI, PF>(P, st.M, tile - P.tile_begin, red);
}

template <int MB, int CPL>
static int launch_stage_cfg(const DStage& st, bool a_f32, int epi, hipStream_t s) {
    const dim3 grid((unsigned)st.total_tiles), block(256);
    constexpr int PF = 3;
    if (epi == EPI_ATOMIC) {
        if (a_f32) hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_ATOMIC, PF>), grid, block, 0, s, st);
        else       hipLaunchKernelGGL((k_decode_stage<MB, CPL, false, EPI_ATOMIC, PF>), grid, block, 0, s, st);
    } else if (epi == EPI_STORE) {
        if (a_f32) hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_STORE, PF>), grid, block, 0, s, st);
        else       hipLaunchKernelGGL((k_decode_stage<MB, CPL, false, EPI_STORE, PF>), grid, block, 0, s, st);
    } else {
        if (!a_f32) { set_error("gate/up stage expects the fp32 rank-space input"); return LR_ERR_UNSUPPORTED; }
        hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_GATEUP, PF>), grid, block, 0, s, st);
    }
    return launch_status("decode stage");
}

int decode_launch_stage(const DStage& st, int cpl, bool a_f32, int epi, hipStream_t s) {
    if (st.total_tiles <= 0 || st.M <= 0) return LR_OK;
    const int mb = st.M <= 16 ? 1 : 2;
    if (mb == 1 && cpl == 4) return launch_stage_cfg<1, 4>(st, a_f32, epi, s);
    if (mb == 1 && cpl == 8) return launch_stage_cfg<1, 8>(st, a_f32, epi, s);
    if (mb == 2 && cpl == 4) return launch_stage_cfg<2, 4>(st, a_f32, epi, s);
    if (mb == 2 && cpl == 8) return launch_stage_cfg<2, 8>(st, a_f32, epi, s);
    set_error("bad decode tile configuration");
    return LR_ERR_UNSUPPORTED;
}

}  // namespace lr
