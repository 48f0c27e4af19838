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
#pragma once
#include "decode.hpp"

namespace lr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x8_t __attribute__((ext_vector_type(8)));

template <int CPL> struct WFrag { uint32_t w[8][CPL / 2]; };   // 8 k-rows x CPL bf16 columns
// 8 consecutive k of one token row, as loaded: packed bf16 (4 dwords) or raw fp32 (8 dwords, converted
// only when the MFMA consumes it, so that issuing the load never waits on earlier loads).
template <bool AF32> struct AFrag { uint32_t a[AF32 ? 8 : 4]; };

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    union { bf16x2_t v; uint32_t u; } x;
    x.v = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return x.u;
}

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

// 8-byte load that is coherent across the whole device (agent scope): used for data that other
// workgroups of the SAME launch produced (rank-space accumulators, hidden rows).
__device__ __forceinline__ uint2 ld_coherent_b64(const void* p) {
    const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void st_coherent_b64(void* p, uint2 v) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), (uint64_t)v.x | ((uint64_t)v.y << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte device-coherent load, issued without a wait (the 64-bit atomic load above is the widest the compiler offers); the
// caller passes all destinations of a batch to wait_loads_b128 before it reads any of them.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t ld_coherent_b128_issue(const void* p) {
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
template <int N>
__device__ __forceinline__ void wait_loads_b128(u32x4_t (&v)[N]) {
    static_assert(N == 8 || N == 12, "batch size");
    if constexpr (N == 8)
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) :: "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                                            "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]) :: "memory");
}

// COH: the rows were written earlier in this launch by other workgroups -> coherent loads.
template <bool AF32, bool COH>
__device__ __forceinline__ void load_a(AFrag<AF32>& f, const void* A, int lda, int m, int M, int k) {
    constexpr int ND = AF32 ? 8 : 4;
    if (m < M) {
        const uint32_t* p = AF32 ? reinterpret_cast<const uint32_t*>(reinterpret_cast<const float*>(A) + (size_t)m * lda + k)
                                 : reinterpret_cast<const uint32_t*>(reinterpret_cast<const bf16_t*>(A) + (size_t)m * lda + k);
        if constexpr (COH) {
#pragma unroll
            for (int i = 0; i < ND; i += 2) { const uint2 v = ld_coherent_b64(p + i); f.a[i] = v.x; f.a[i + 1] = v.y; }
        } else {
#pragma unroll
            for (int i = 0; i < ND; i += 4) {
                const uint4 v = *reinterpret_cast<const uint4*>(p + i);
                f.a[i] = v.x; f.a[i + 1] = v.y; f.a[i + 2] = v.z; f.a[i + 3] = v.w;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < ND; ++i) f.a[i] = 0u;
    }
}

__device__ __forceinline__ bf16x8_t as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    union { uint32_t u[4]; bf16x8_t v; } x;
    x.u[0] = a; x.u[1] = b; x.u[2] = c; x.u[3] = d;
    return x.v;
}

// acc[mb][b] += A_mb (16 x 32) * W(:, column offset b) (32 x 16 lanes)
template <int MB, int CPL, bool AF32>
__device__ __forceinline__ void mma_block(f32x4_t (&acc)[MB][CPL], const WFrag<CPL>& wf, const AFrag<AF32> (&af)[MB]) {
    bf16x8_t av[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        if constexpr (AF32) {
            const uint32_t* a = af[mb].a;
            av[mb] = as_bf16x8(pack2(__uint_as_float(a[0]), __uint_as_float(a[1])), pack2(__uint_as_float(a[2]), __uint_as_float(a[3])),
                               pack2(__uint_as_float(a[4]), __uint_as_float(a[5])), pack2(__uint_as_float(a[6]), __uint_as_float(a[7])));
        } else {
            av[mb] = as_bf16x8(af[mb].a[0], af[mb].a[1], af[mb].a[2], af[mb].a[3]);
        }
    }
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

// Hook run between the first weight loads of a tile and its first activation loads.  Its argument receives the
// workspace's error word when the hook is the wait in front of a call's last stage (read right after the wait, used in
// the epilogue: any workgroup that gave up anywhere in the launch raised that word before it arrived at the barrier
// just passed, so the whole result turns NaN, not only the failing workgroup's part).
// kCoherent: the activation rows were produced earlier in this launch by other workgroups and are read with
// agent-coherent loads; kFused: hidden rows written by this tile are read by other workgroups of this launch.
#ifdef LR_DECODE_COHERENT_ACTS
constexpr bool kPlainActsFwd = false;      // see GridWaitPlain
#else
constexpr bool kPlainActsFwd = true;
#endif
struct NoSync { static constexpr bool kCoherent = false, kFused = false; __device__ __forceinline__ void operator()(uint32_t&) const {}
                __device__ __forceinline__ void before_epilogue() const {} };
// Same, for later tiles of a stage whose input other workgroups of this launch produced.
struct NoSyncCoherent { static constexpr bool kCoherent = true, kFused = true; __device__ __forceinline__ void operator()(uint32_t&) const {}
                        __device__ __forceinline__ void before_epilogue() const {} };
// Later tiles of a stage whose input (accumulators added with device-scope atomics, hidden rows or a finalised bf16
// copy written with device-coherent stores) no workgroup on this XCD has read before the stage's barrier in this
// launch: plain cached loads are safe (first touch misses L2) and let the other workgroups hit in L2.
struct NoSyncPlain { static constexpr bool kCoherent = !kPlainActsFwd, kFused = true; __device__ __forceinline__ void operator()() const {}
                     __device__ __forceinline__ void operator()(uint32_t&) const {}
                     __device__ __forceinline__ void before_epilogue() const {} };

// This wave's share of rows [32*kb0, 32*kb1) of W: blocks kb0 + wave, kb0 + wave + NW, ...
// The first PF weight blocks are requested before `sync()` runs and the activations after it, so
// that a wait for the producer of A overlaps with weight traffic already in flight.
template <int MB, int CPL, bool AF32, int PF, int NW, class Sync>
__device__ __forceinline__ void mma_range(f32x4_t (&acc)[MB][CPL], const bf16_t* __restrict__ W, int N,
                                          const void* A, int lda, int M, int col, int kb0, int kb1,
                                          int wave, int j, int g, const Sync& sync, uint32_t& late_err) {
    WFrag<CPL> wf[PF];
    AFrag<AF32> af[PF][MB];
    int blk = kb0 + wave;
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int bb = blk + NW * p;
        if (bb < kb1) load_w<CPL>(wf[p], W, N, 32 * bb + 8 * g, col);
    }
    sync(late_err);
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int bb = blk + NW * p;
        if (bb < kb1) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) load_a<AF32, Sync::kCoherent>(af[p][mb], A, lda, 16 * mb + j, M, 32 * bb + 8 * g);
        }
    }
    for (; blk < kb1; blk += NW * PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int bb = blk + NW * p;
            if (bb < kb1) {
                mma_block<MB, CPL, AF32>(acc, wf[p], af[p]);
                const int nb = bb + NW * PF;
                if (nb < kb1) {
                    load_w<CPL>(wf[p], W, N, 32 * nb + 8 * g, col);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) load_a<AF32, Sync::kCoherent>(af[p][mb], A, lda, 16 * mb + j, M, 32 * nb + 8 * g);
                }
            }
        }
    }
}

// Gate/up tiles: the blocks of both products as ONE sequence (nb1 blocks of W, then nb2 blocks of W2; this wave takes
// entries wave, wave + NW, ...), so that the prefetch runs across the border between the two products.  Two ranges one
// after the other let the requests drain at the end of the first: a memory latency per tile with nothing in flight.
template <int MB, int CPL, bool AF32, int PF, int NW, class Sync>
__device__ __forceinline__ void mma_range2(f32x4_t (&acc1)[MB][CPL], f32x4_t (&acc2)[MB][CPL],
                                           const bf16_t* __restrict__ W, const bf16_t* __restrict__ W2, int N,
                                           const void* A, const void* A2, int lda, int lda2, int M, int col, int nb1, int nb2,
                                           int wave, int j, int g, const Sync& sync, uint32_t& late_err) {
    WFrag<CPL> wf[PF];
    AFrag<AF32> af[PF][MB];
    const int nv = nb1 + nb2;
    int blk = wave;
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int v = blk + NW * p;
        if (v < nv) {
            if (v < nb1) load_w<CPL>(wf[p], W, N, 32 * v + 8 * g, col);
            else         load_w<CPL>(wf[p], W2, N, 32 * (v - nb1) + 8 * g, col);
        }
    }
    sync(late_err);
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        const int v = blk + NW * p;
        if (v < nv) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (v < nb1) load_a<AF32, Sync::kCoherent>(af[p][mb], A, lda, 16 * mb + j, M, 32 * v + 8 * g);
                else         load_a<AF32, Sync::kCoherent>(af[p][mb], A2, lda2, 16 * mb + j, M, 32 * (v - nb1) + 8 * g);
            }
        }
    }
    for (; blk < nv; blk += NW * PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int v = blk + NW * p;
            if (v < nv) {
                if (v < nb1) mma_block<MB, CPL, AF32>(acc1, wf[p], af[p]);
                else         mma_block<MB, CPL, AF32>(acc2, wf[p], af[p]);
                const int nx = v + NW * PF;
                if (nx < nv) {
                    if (nx < nb1) load_w<CPL>(wf[p], W, N, 32 * nx + 8 * g, col);
                    else          load_w<CPL>(wf[p], W2, N, 32 * (nx - nb1) + 8 * g, col);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        if (nx < nb1) load_a<AF32, Sync::kCoherent>(af[p][mb], A, lda, 16 * mb + j, M, 32 * nx + 8 * g);
                        else          load_a<AF32, Sync::kCoherent>(af[p][mb], A2, lda2, 16 * mb + j, M, 32 * (nx - nb1) + 8 * g);
                    }
                }
            }
        }
    }
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
template <int MB, int CPL, bool AF32, int EPI, int PF, int NW, class Sync>
__device__ __forceinline__ void decode_tile(const DProb& P, int M, int lt, float4* __restrict__ red,
                                            const Sync& sync, const size_t& acc_shift, uint32_t* const& tcnt = nullptr,
                                            const uint32_t* poison = nullptr) {
    constexpr int NMAT = (EPI == EPI_GATEUP) ? 2 : 1;
    constexpr int NC = 16 * CPL;
    constexpr int Q = CPL / 4;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 15, g = lane >> 4;
    const int tn = lt % P.tiles_n, tk = lt / P.tiles_n;
    const int n0 = tn * NC;
    const int col = n0 + CPL * j;

    uint32_t late_err = 0u;
    f32x4_t acc[NMAT][MB][CPL];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int b = 0; b < CPL; ++b) acc[mt][mb][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    if constexpr (NMAT == 1) {
        const int kb0 = tk * (P.KS >> 5);
        int kb1 = kb0 + (P.KS >> 5);
        if (kb1 > (P.K >> 5)) kb1 = P.K >> 5;
        const void* A = AF32 ? (const void*)((const char*)P.A + acc_shift) : P.A;
        mma_range<MB, CPL, AF32, PF, NW>(acc[0], P.W + (size_t)tn * P.wtile, P.wstride, A, P.lda, M, CPL * j, kb0, kb1, wave, j, g, sync, late_err);
    } else {
        // gate/up: the blocks of both products as one request sequence, one set of weight and activation registers for both (two
        // ranges one after the other, each with its own registers, leave the compiler twice the prefetch registers live at the
        // border between the products: at two 16-row blocks per wave that spills from two blocks ahead on)
        const void* A = AF32 ? (const void*)((const char*)P.A + acc_shift) : P.A;
        const void* A2 = AF32 ? (const void*)((const char*)P.A2 + acc_shift) : P.A2;
        mma_range2<MB, CPL, AF32, PF, NW>(acc[0], acc[NMAT - 1], P.W + (size_t)tn * P.wtile, P.W2 + (size_t)tn * P.wtile2, P.wstride, A, A2, P.lda, P.lda2, M, CPL * j, P.K >> 5, P.K2 >> 5,
                                          wave, j, g, sync, late_err);
    }

    sync.before_epilogue();       // (the first tile of a call resolves the workspace's control block here: after its loads, before its first use)
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
    // a call whose device-wide wait gave up (or whose workspace carries an earlier failure) delivers NaN, never plausible numbers
    const bool nan_out = (EPI == EPI_STORE) && poison != nullptr && (*poison != 0u || late_err != 0u);
    float atomic_returns = 0.f;
    // Split-K stage that accumulates with atomics: one atomic per thread on CONSECUTIVE floats of a row (a wave-level atomic then
    // covers two whole 128-byte lines; in the operand layout a lane owns 4 columns of 4 rows, 16 bytes apart from its neighbours'),
    // over the M valid rows only, by all waves.
    const bool contiguous_atomics = EPI == EPI_ATOMIC && tcnt == nullptr;
    if constexpr (EPI == EPI_ATOMIC) {
        if (contiguous_atomics) {
            float* const cbase = (float*)((char*)P.C + acc_shift) + n0;
            for (int e = tid; e < M * NC; e += 64 * NW) {
                const int m = e / NC, c = e - m * NC;
                const int sl = (m >> 4) * 4 + (m & 3), ln = ((m & 15) >> 2) * 16 + c / CPL, b = c % CPL;
                const float* r0 = reinterpret_cast<const float*>(&red[(sl * Q + (b >> 2)) * 64 + ln]) + (b & 3);
                float sum = r0[0];
#pragma unroll
                for (int w = 1; w < NW; ++w) sum += r0[(size_t)w * NSL * Q * 64 * 4];
                // RETURNING atomics: a non-returning one is acknowledged as soon as the L2 has accepted it,
                // before it is performed where other XCDs can see it; its return value only exists once it
                // has been performed, and consuming the values below orders them before the arrival signal.
                atomic_returns += unsafeAtomicAdd(cbase + (size_t)m * P.ldc + c, sum);
            }
        }
    }
#pragma unroll
    for (int pidx = tid; pidx < (contiguous_atomics ? 0 : 256 * MB); pidx += 64 * NW) {   // (mb, v, lane') triples
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
                for (int w = 1; w < NW; ++w) {
                    const float4 o = red[((w * NSL + mt * MB * 4 + sl) * Q + q) * 64 + ln];
                    s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
                }
                val[mt][4 * q + 0] = s.x; val[mt][4 * q + 1] = s.y; val[mt][4 * q + 2] = s.z; val[mt][4 * q + 3] = s.w;
            }
        if (m < M) {
            if constexpr (EPI == EPI_ATOMIC) {
                if (tcnt) {
                    // larger row counts: the partial tile goes to its own slot (plain device-coherent stores, no
                    // atomics: 2048 of them per workgroup were what bound these stages); see the finalisation below
                    float* ps = P.part + (size_t)(P.tile_begin + lt) * (16 * MB * NC) + (size_t)m * NC + (n - n0);
#pragma unroll
                    for (int b = 0; b < CPL; b += 2) st_coherent_b64(ps + b, make_uint2(__float_as_uint(val[0][b]), __float_as_uint(val[0][b + 1])));
                }
            } else if constexpr (EPI == EPI_STORE) {
                if (nan_out) {
#pragma unroll
                    for (int b = 0; b < CPL; ++b) val[0][b] = __uint_as_float(0x7fc00000u);
                }
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
                if constexpr (CPL == 4 && Sync::kFused) {   // fused launch: another workgroup reads h next
                    st_coherent_b64(P.Y + (size_t)m * P.N + n, make_uint2(pack2(hv[0], hv[1]), pack2(hv[2], hv[3])));
                } else {
                    store_bf16_row<CPL>(P.Y + (size_t)m * P.N + n, hv);
                }
            }
        }
    }
    if constexpr (EPI == EPI_ATOMIC) asm volatile("" ::"v"(atomic_returns));   // every atomic above has returned
    if constexpr (EPI == EPI_STORE) {
        if (poison != nullptr && late_err != 0u && tid == 0) *const_cast<uint32_t*>(poison) = 1u;   // later tiles of this workgroup see it too
    }

    // bf16 finalisation of a split-K stage (larger row counts, chosen by the host planner): the workgroup whose K-slice of this column
    // tile arrives last adds up all slices' partial tiles and writes the tile as bf16 once, so that the next
    // stage's workgroups read half the bytes with plain cached loads instead of each converting the whole of t.
    if constexpr (EPI == EPI_ATOMIC) {
        if (tcnt) {
            __shared__ uint32_t s_last;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // this wave's atomics have been performed
            __syncthreads();
            if (tid == 0) {
                const uint32_t slices = (uint32_t)((P.K + P.KS - 1) / P.KS);
                const uint32_t old = __hip_atomic_fetch_add(tcnt + P.ctile_begin + tn, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last = (old == slices - 1u) ? 1u : 0u;
            }
            __syncthreads();
            if (s_last) {
                // add the K-slices of this column tile in slice order (deterministic), 8 or 12 slots in flight per lane
                const int slices = (P.K + P.KS - 1) / P.KS;
                const size_t slot = (size_t)16 * MB * NC, step = (size_t)P.tiles_n * slot;
                // A thread takes IT outputs (4 columns of one row each) at a time and has the slices of all of them in
                // flight together, SB slices per round trip: the sum is bound by those round trips, not by bytes.
                // (Eight waves, measured in one run: 12 instead of 8 slices per round trip gains 0.6-1.1 us per call from
                // 17 rows on, where a stage has 10-21 slices of 8 KB, and loses 0.2 us at 9-16 rows; 22 lose everywhere.)
                constexpr int IT = NW == 4 ? 2 : 1, SB = (NW == 4 || MB == 2) ? 12 : 8;
                const int items = M * (NC / 4);
                for (int it0 = tid; it0 < items; it0 += 64 * NW * IT) {
                    const float* src[IT];
                    float acc4[IT][4];
#pragma unroll
                    for (int q = 0; q < IT; ++q) {
                        int it = it0 + 64 * NW * q;
                        it = it < items ? it : items - 1;
                        const int m = it / (NC / 4), c4 = 4 * (it % (NC / 4));
                        src[q] = P.part + (size_t)(P.tile_begin + tn) * slot + (size_t)m * NC + c4;
                        acc4[q][0] = acc4[q][1] = acc4[q][2] = acc4[q][3] = 0.f;
                    }
                    for (int sl0 = 0; sl0 < slices; sl0 += SB) {
                        u32x4_t a[IT][SB];
#pragma unroll
                        for (int q = 0; q < IT; ++q)
#pragma unroll
                            for (int u = 0; u < SB; ++u) {
                                const int sl = sl0 + u < slices ? sl0 + u : slices - 1;
                                a[q][u] = ld_coherent_b128_issue(src[q] + (size_t)sl * step);
                            }
                        // (the loads above are issued by hand: the compiler does not count them, so the wait is written out and
                        // takes every destination as an operand, which keeps their uses behind it)
#pragma unroll
                        for (int q = 0; q < IT; ++q) wait_loads_b128<SB>(a[q]);
#pragma unroll
                        for (int q = 0; q < IT; ++q)
#pragma unroll
                            for (int u = 0; u < SB; ++u)
                                if (sl0 + u < slices) {
                                    acc4[q][0] += __uint_as_float(a[q][u].x); acc4[q][1] += __uint_as_float(a[q][u].y);
                                    acc4[q][2] += __uint_as_float(a[q][u].z); acc4[q][3] += __uint_as_float(a[q][u].w);
                                }
                    }
#pragma unroll
                    for (int q = 0; q < IT; ++q) {
                        const int it = it0 + 64 * NW * q;
                        if (it < items) {
                            const int m = it / (NC / 4), c4 = 4 * (it % (NC / 4));
                            st_coherent_b64(P.Y + (size_t)m * P.ldy + n0 + c4, make_uint2(pack2(acc4[q][0], acc4[q][1]), pack2(acc4[q][2], acc4[q][3])));
                        }
                    }
                }
            }
        }
    }
}

template <int MB, int CPL, int EPI, int NW>
constexpr int red_float4s() { return NW * ((EPI == EPI_GATEUP) ? 2 : 1) * MB * 4 * (CPL / 4) * 64; }

template <int MB, int CPL, bool AF32, int EPI, int PF>
__global__ void __launch_bounds__(256) k_decode_stage(DStage st) {
    __shared__ float4 red[red_float4s<MB, CPL, EPI, 4>()];
    const int tile = blockIdx.x;
    int pi = 0;
#pragma unroll
    for (int i = 1; i < kMaxProb; ++i)
        if (i < st.nprob && tile >= st.p[i].tile_begin) pi = i;
    const DProb& P = st.p[pi];
    const size_t no_shift = 0;
    decode_tile<MB, CPL, AF32, EPI, PF, 4>(P, st.M, tile - P.tile_begin, red, NoSync(), no_shift);
}

// ---------------------------------------------------------------------------------------------
// Fused decode calls: all stages of one entry point in ONE launch.  The grid is small enough for
// every workgroup to be resident at once when the device runs nothing else, stages are separated by a
// device-wide arrive/wait counter in the workspace control block, and a workgroup asks for the first
// weight blocks of its next tile BEFORE it waits, so HBM keeps streaming across the dependency.
// Waiting is bounded: after `spin_limit` polls the workgroup sets the control block's error word, marks
// itself poisoned and carries on without further waits; a poisoned workgroup writes NaN as its results,
// and the error word (watched by every waiting wave, checked at the start of every later call) poisons
// all other workgroups and all later calls on that workspace, so that a failure cannot pass for a
// result.  Every wave always reaches the end of the kernel.
//
// Split-K accumulators live in one of two areas picked by the parity of the control block's epoch;
// while a call accumulates into area p it clears what the previous call dirtied in area 1-p, and
// workgroup 0, once it has seen the first barrier complete, publishes epoch+1 and the new dirty extents.

// Optional timeline of the fused kernels (builds with -DLR_TRACE only; never in the shipped library):
// thread 0 of every workgroup stores the 100 MHz wall clock at numbered points.
#ifdef LR_TRACE
#define LR_STAMP_TO(tr, i) do { if (threadIdx.x == 0 && (tr)) (tr)[blockIdx.x * 16 + (i)] = wall_clock64(); } while (0)
#else
#define LR_STAMP_TO(tr, i) do { } while (0)
#endif
#define LR_STAMP(i) LR_STAMP_TO(fa.fc.trace, i)

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_agent64(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- control block: start of a call -------------------------------------------------------------------
// Three 8-byte device-coherent reads {magic} {epoch, error} {dirty[0], dirty[1]}, issued at the top of the
// kernel; nothing waits on them until ctrl_resolve, which a wave calls once its first weight blocks are on
// their way.
struct CtrlLoads { uint2 m, e, d; };
struct CtrlSnap { uint32_t epoch, p, dirty_other, error; };

__device__ __forceinline__ CtrlLoads ctrl_issue(const Ctrl* c) {
    CtrlLoads L;
    L.m = ld_coherent_b64(&c->magic);
    L.e = ld_coherent_b64(&c->epoch);
    L.d = ld_coherent_b64(&c->dirty[0]);
    return L;
}

constexpr uint32_t kPrepareSpinLimit = 1u << 24;

// Rare path (first call on a workspace that nobody prepared): one wave of the whole launch wins the right to
// prepare, everyone else waits for kCtrlReady.  Wave-uniform; returns false if the wait gave up.
__device__ __noinline__ bool ctrl_prepare(Ctrl* c, char* acc0, size_t acc_bytes, uint64_t observed) {
    const int lane = threadIdx.x & 63;
    uint32_t won = 0;
    if (lane == 0 && observed != kCtrlBusy) {
        uint64_t expect = observed;
        won = __hip_atomic_compare_exchange_strong(&c->magic, &expect, kCtrlBusy, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT) ? 1u : 0u;
    }
    won = __builtin_amdgcn_readfirstlane(won);
    if (won) {
        // header behind the magic word + shared-K flags (contiguous), then both accumulator areas
        uint2* h = reinterpret_cast<uint2*>(c) + 1;
        const uint32_t n8 = (uint32_t)((kHeaderBytes + kSkFlagBytes) / 8 - 1);
        for (uint32_t i = lane; i < n8; i += 64) h[i] = make_uint2(0u, 0u);
        uint4* a = reinterpret_cast<uint4*>(acc0);
        const uint32_t n16 = (uint32_t)(2 * acc_bytes / 16);
        for (uint32_t i = lane; i < n16; i += 64) a[i] = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");             // the zeroes are in memory before the word says so
        if (lane == 0) __hip_atomic_store(&c->magic, kCtrlReady, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return true;
    }
    uint32_t spins = 0;
    bool ok = true;
    while (__builtin_amdgcn_readfirstlane((uint32_t)(ld_agent64(&c->magic) == kCtrlReady)) == 0u) {
        if (++spins > kPrepareSpinLimit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(8);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return ok;
}

// Wave-uniform.  `bad` (LDS word of the workgroup) is raised when the workspace carries an earlier failure.
__device__ __forceinline__ CtrlSnap ctrl_resolve(Ctrl* ctrl, char* acc0, size_t acc_bytes, CtrlLoads L, uint32_t* bad) {
    const uint64_t magic = (uint64_t)L.m.x | ((uint64_t)L.m.y << 32);
    if (__builtin_amdgcn_readfirstlane((uint32_t)(magic != kCtrlReady)) != 0u) {
        const bool ok = ctrl_prepare(ctrl, acc0, acc_bytes, magic);
        L = ctrl_issue(ctrl);
        if (!ok) {
            if ((threadIdx.x & 63) == 0) { __hip_atomic_store(&ctrl->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); *bad = 1u; }
        }
    }
    CtrlSnap c;
    c.epoch = L.e.x; c.error = L.e.y; c.p = L.e.x & 1u;
    c.dirty_other = c.p ? L.d.x : L.d.y;
    if (c.error != 0u && (threadIdx.x & 63) == 0) *bad = 1u;
    return c;
}

// Hook of the first tile of a call's first stage: resolves the control block (and with it the parity of the
// accumulator areas) after the tile's blocks have been multiplied, right before its epilogue needs the parity.
struct CtrlGate {
    static constexpr bool kCoherent = false, kFused = false;
    Ctrl* ctrl; char* acc0; size_t acc_bytes;       // by value: taking the address of a kernel argument would force a private copy of all of them
    const CtrlLoads* loads; CtrlSnap* snap; size_t* shift;
    uint32_t** tcnt; bool t16;      // tile counters of the call's parity (bf16 finalisation), else NULL
    uint32_t* bad;
    __device__ __forceinline__ void operator()(uint32_t&) const {}
    __device__ __forceinline__ void before_epilogue() const { (*this)(); }
    __device__ __forceinline__ void operator()() const {
        *snap = ctrl_resolve(ctrl, acc0, acc_bytes, *loads, bad);
        *shift = (size_t)snap->p * acc_bytes;
        *tcnt = t16 ? ctrl->tcnt[snap->p] : nullptr;
    }
};

// Stage barrier.  Data shared inside a launch is only touched by atomics and by agent-coherent
// loads / stores, so no cache maintenance is needed: it is enough that every wave has drained its
// memory operations (workgroup-scope release = s_waitcnt) before the workgroup's arrival is counted.
// (Agent-scope release / acquire fences here cost tens of microseconds per barrier: they write back
// and invalidate the L2.)
// All threads of the workgroup call this after their last store / atomic of the stage.
__device__ __forceinline__ void grid_arrive(uint32_t* slots) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0)
        __hip_atomic_fetch_add(slots + (blockIdx.x % kSlots) * kSlotStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct GridWait {
    static constexpr bool kCoherent = true, kFused = true;
    const uint32_t* slots;
    uint32_t grid;
    uint32_t* err;
    uint32_t spin_limit;
    uint32_t* bad;          // LDS word of the workgroup: a wait gave up, or the error word was seen set
    int stamp;
    unsigned long long* trace;
    bool last;              // the wait in front of the call's last stage: hand the error word to the epilogue
    __device__ __forceinline__ void before_epilogue() const {}
    __device__ __forceinline__ void operator()(uint32_t& late_err) const {
        (*this)();
        if (last) late_err = ld_agent(err);
    }
    __device__ __forceinline__ void operator()() const {
        if (threadIdx.x < 64) {     // wave 0: lane s < kSlots watches slot s, lane kSlots watches the error word
            const uint32_t lane = threadIdx.x;
            const uint32_t want = lane < kSlots ? (grid + kSlots - 1 - lane) / kSlots : 0u;   // workgroups with w % kSlots == lane
            const uint32_t* p = lane < kSlots ? slots + lane * kSlotStride : (lane == kSlots ? err : slots);
            uint32_t spins = 0;
            bool poisoned = __builtin_amdgcn_readfirstlane(*bad) != 0u;
            while (!poisoned) {
                const uint32_t v = ld_agent(p);
                if (__builtin_amdgcn_ballot_w64(lane == kSlots && v != 0u) != 0ull) { poisoned = true; break; }
                if (__builtin_amdgcn_ballot_w64(lane < kSlots && v < want) == 0ull) break;
                if (++spins > spin_limit) {
                    // returning atomic, consumed: the word is set where every workgroup sees it before this one moves on
                    uint32_t old = 0u;
                    if (lane == 0) old = __hip_atomic_exchange(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    asm volatile("" ::"v"(old));
                    poisoned = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (poisoned && lane == 0) *bad = 1u;
        }
        __syncthreads();
        LR_STAMP_TO(trace, stamp);
    }
};

// The same wait in front of a stage that reads its input with plain cached loads (see NoSyncPlain).
// Building with -DLR_DECODE_COHERENT_ACTS makes every such stage read its input with device-coherent loads instead
// (the fallback should the first-touch argument ever stop holding: about 1 us slower per packed-MLP call).
#ifdef LR_DECODE_COHERENT_ACTS
constexpr bool kPlainActs = false;
#else
constexpr bool kPlainActs = true;
#endif
struct GridWaitPlain : GridWait {
    static constexpr bool kCoherent = !kPlainActs, kFused = true;
    __device__ __forceinline__ GridWaitPlain(const GridWait& g) : GridWait(g) {}
};

// Clear what the previous call left in the other accumulator area and the other parity's barrier
// counters (nobody uses them during this call).  Called by every workgroup before its first arrive.
__device__ __forceinline__ void fused_clear_other(const FusedCommon& fc, const CtrlSnap& c) {
    const uint32_t n4 = (c.dirty_other + 3u) >> 2;
    float4* other = reinterpret_cast<float4*>(fc.acc0 + (size_t)(1u - c.p) * fc.acc_bytes);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += gridDim.x * blockDim.x)
        other[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0) {
        for (uint32_t i = threadIdx.x; i < (uint32_t)(kBarriers * kSlots); i += blockDim.x)
            fc.ctrl->cnt[1u - c.p][i / kSlots][(i % kSlots) * kSlotStride] = 0u;
        for (uint32_t i = threadIdx.x; i < (uint32_t)kTileCounters; i += blockDim.x) fc.ctrl->tcnt[1u - c.p][i] = 0u;
    }
}

// First barrier of a fused kernel: every workgroup clears its share of the other accumulator area,
// then arrives.
__device__ __forceinline__ void fused_first_arrive(const FusedCommon& fc, const CtrlSnap& c) {
    fused_clear_other(fc, c);
    grid_arrive(fc.ctrl->cnt[c.p][0]);
}

// Workgroup 0, once it has seen the first barrier complete (every workgroup has read the control
// block by then), publishes the next epoch and the new dirty extents.
__device__ __forceinline__ void fused_publish(const FusedCommon& fc, const CtrlSnap& c) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        fc.ctrl->dirty[c.p] = fc.dirty_floats;
        fc.ctrl->dirty[1u - c.p] = 0u;
        __hip_atomic_store(&fc.ctrl->epoch, c.epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int NP>
__device__ __forceinline__ const DProb& find_prob(const DStageT<NP>& st, int tile) {
    int pi = 0;
#pragma unroll
    for (int i = 1; i < NP; ++i)
        if (i < st.nprob && tile >= st.p[i].tile_begin) pi = i;
    return st.p[pi];
}

// lowrank_linear / lowrank_qkv: t += x U (split-K, atomics)  ->  barrier  ->  y = t V (+bias, cache).
// PF1, PF2: weight blocks a wave requests ahead in either stage.
template <int MB, int CPL1, int CPL2, int PF1, int PF2, int NP, int NW>
__global__ void __launch_bounds__(64 * NW) k_decode_fused2(Fused2Args<NP> fa) {
    constexpr int R1 = red_float4s<MB, CPL1, EPI_ATOMIC, NW>(), R2 = red_float4s<MB, CPL2, EPI_STORE, NW>();
    __shared__ float4 red[R1 > R2 ? R1 : R2];
    __shared__ uint32_t s_bad;
    const CtrlLoads cl = ctrl_issue(fa.fc.ctrl);
    if (threadIdx.x == 0) s_bad = 0u;
    __syncthreads();
    CtrlSnap cs;
    size_t shift = 0;
    uint32_t* tcp = nullptr;
    const CtrlGate gate = {fa.fc.ctrl, fa.fc.acc0, fa.fc.acc_bytes, &cl, &cs, &shift, &tcp, false, &s_bad};
    bool resolved = false;
    LR_STAMP(0);
    for (int tile = blockIdx.x; tile < fa.s1.total_tiles; tile += gridDim.x) {
        const DProb& P = find_prob<NP>(fa.s1, tile);
        if (!resolved) decode_tile<MB, CPL1, false, EPI_ATOMIC, PF1, NW>(P, fa.s1.M, tile - P.tile_begin, red, gate, shift);
        else           decode_tile<MB, CPL1, false, EPI_ATOMIC, PF1, NW>(P, fa.s1.M, tile - P.tile_begin, red, NoSync(), shift);
        resolved = true;
        __syncthreads();
    }
    if (!resolved) gate();
    const uint32_t p = cs.p;
    LR_STAMP(1);
    fused_first_arrive(fa.fc, cs);
    LR_STAMP(2);
    const GridWait gw = {fa.fc.ctrl->cnt[p][0], gridDim.x, &fa.fc.ctrl->error, fa.fc.spin_limit, &s_bad, 3, fa.fc.trace, true};
    bool waited = false;
    for (int tile = blockIdx.x; tile < fa.s2.total_tiles; tile += gridDim.x) {
        const DProb& P = find_prob<NP>(fa.s2, tile);
        if (!waited) decode_tile<MB, CPL2, true, EPI_STORE, PF2, NW>(P, fa.s2.M, tile - P.tile_begin, red, GridWaitPlain(gw), shift, nullptr, &s_bad);
        else         decode_tile<MB, CPL2, true, EPI_STORE, PF2, NW>(P, fa.s2.M, tile - P.tile_begin, red, NoSyncPlain(), shift, nullptr, &s_bad);
        if (!waited) fused_publish(fa.fc, cs);
        waited = true;
        __syncthreads();
    }
    if (blockIdx.x == 0 && !waited) { gw(); fused_publish(fa.fc, cs); }
    LR_STAMP(10);
}

// lowrank_packed_mlp: four stages, three barriers.  PFA..PFD: weight blocks a wave requests ahead in each stage (the blocks
// requested before a stage's barrier are what streams while the barrier is pending; the gate/up stage, with two accumulator
// sets, has the fewest registers to spare).
template <int MB, int CPLA, int CPLC, int CPLD, int PFA, int PFB, int PFC, int PFD, int NW, bool T16>
__global__ void __launch_bounds__(64 * NW) k_decode_fused_mlp(FusedMlpArgs fa) {
    constexpr int RA = red_float4s<MB, CPLA, EPI_ATOMIC, NW>(), RB = red_float4s<MB, 4, EPI_GATEUP, NW>();
    constexpr int RC = red_float4s<MB, CPLC, EPI_ATOMIC, NW>(), RD = red_float4s<MB, CPLD, EPI_STORE, NW>();
    constexpr int R01 = RA > RB ? RA : RB, R23 = RC > RD ? RC : RD;
    __shared__ float4 red[R01 > R23 ? R01 : R23];
    __shared__ uint32_t s_bad;
    const CtrlLoads cl = ctrl_issue(fa.fc.ctrl);
    if (threadIdx.x == 0) s_bad = 0u;
    __syncthreads();
    CtrlSnap cs;
    size_t shift = 0;
    uint32_t* tcp = nullptr;
    const CtrlGate gate = {fa.fc.ctrl, fa.fc.acc0, fa.fc.acc_bytes, &cl, &cs, &shift, &tcp, T16, &s_bad};
    const uint32_t G = gridDim.x;
    LR_STAMP(0);
    // A: t_gu += x U_gu
    bool resolved = false;
    for (int tile = blockIdx.x; tile < fa.a.total_tiles; tile += G) {
        if (!resolved) decode_tile<MB, CPLA, false, EPI_ATOMIC, PFA, NW>(fa.a.p[0], fa.a.M, tile, red, gate, shift, tcp);
        else           decode_tile<MB, CPLA, false, EPI_ATOMIC, PFA, NW>(fa.a.p[0], fa.a.M, tile, red, NoSync(), shift, tcp);
        resolved = true;
        __syncthreads();
    }
    if (!resolved) gate();
    const uint32_t p = cs.p;
    uint32_t (*cnt)[kSlots * kSlotStride] = fa.fc.ctrl->cnt[p];
    LR_STAMP(1);
    fused_first_arrive(fa.fc, cs);
    LR_STAMP(2);
    // B: h = SiLU(t_g V_g + b_g) * (t_u V_u + b_u)
    {
        const GridWait gw = {cnt[0], G, &fa.fc.ctrl->error, fa.fc.spin_limit, &s_bad, 3, fa.fc.trace, false};
        bool waited = false;
        for (int tile = blockIdx.x; tile < fa.b.total_tiles; tile += G) {
            if constexpr (T16) {
                if (!waited) decode_tile<MB, 4, false, EPI_GATEUP, PFB, NW>(fa.b.p[0], fa.b.M, tile, red, GridWaitPlain(gw), shift);
                else         decode_tile<MB, 4, false, EPI_GATEUP, PFB, NW>(fa.b.p[0], fa.b.M, tile, red, NoSyncPlain(), shift);
            } else {
                if (!waited) decode_tile<MB, 4, true, EPI_GATEUP, PFB, NW>(fa.b.p[0], fa.b.M, tile, red, GridWaitPlain(gw), shift);
                else         decode_tile<MB, 4, true, EPI_GATEUP, PFB, NW>(fa.b.p[0], fa.b.M, tile, red, NoSyncPlain(), shift);
            }
            if (!waited) fused_publish(fa.fc, cs);
            waited = true;
            __syncthreads();
        }
        if (blockIdx.x == 0 && !waited) { gw(); fused_publish(fa.fc, cs); }
    }
    LR_STAMP(4);
    grid_arrive(cnt[1]);
    LR_STAMP(5);
    // C: t_d += h U_d
    {
        const GridWait gw = {cnt[1], G, &fa.fc.ctrl->error, fa.fc.spin_limit, &s_bad, 6, fa.fc.trace, false};
        bool waited = false;
        for (int tile = blockIdx.x; tile < fa.c.total_tiles; tile += G) {
            if (!waited) decode_tile<MB, CPLC, false, EPI_ATOMIC, PFC, NW>(fa.c.p[0], fa.c.M, tile, red, GridWaitPlain(gw), shift, tcp);
            else         decode_tile<MB, CPLC, false, EPI_ATOMIC, PFC, NW>(fa.c.p[0], fa.c.M, tile, red, NoSyncPlain(), shift, tcp);
            waited = true;
            __syncthreads();
        }
    }
    LR_STAMP(7);
    grid_arrive(cnt[2]);
    LR_STAMP(8);
    // D: out = t_d V_d + b_d
    {
        const GridWait gw = {cnt[2], G, &fa.fc.ctrl->error, fa.fc.spin_limit, &s_bad, 9, fa.fc.trace, true};
        bool waited = false;
        for (int tile = blockIdx.x; tile < fa.d.total_tiles; tile += G) {
            if constexpr (T16) {
                if (!waited) decode_tile<MB, CPLD, false, EPI_STORE, PFD, NW>(fa.d.p[0], fa.d.M, tile, red, GridWaitPlain(gw), shift, nullptr, &s_bad);
                else         decode_tile<MB, CPLD, false, EPI_STORE, PFD, NW>(fa.d.p[0], fa.d.M, tile, red, NoSyncPlain(), shift, nullptr, &s_bad);
            } else {
                if (!waited) decode_tile<MB, CPLD, true, EPI_STORE, PFD, NW>(fa.d.p[0], fa.d.M, tile, red, GridWaitPlain(gw), shift, nullptr, &s_bad);
                else         decode_tile<MB, CPLD, true, EPI_STORE, PFD, NW>(fa.d.p[0], fa.d.M, tile, red, NoSyncPlain(), shift, nullptr, &s_bad);
            }
            waited = true;
            __syncthreads();
        }
    }
    LR_STAMP(10);
}

}  // namespace lr
