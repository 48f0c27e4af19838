// Prefill-phase GEMM (bf16 MFMA, LDS-staged): C[M, N] = A[M, K] * B[K, N] with A, B, C row-major.
//
// Tile: BM x BN x 64 per workgroup of 4 waves (2 x 2), each wave (BM/2) x (BN/2) built from
// v_mfma_f32_32x32x16_bf16.  Both operands sit in LDS "chunk-major": the 8 consecutive k of one
// row are one 16-byte unit, units of one k-chunk are contiguous over rows (one pad unit every
// 8 rows), so a fragment read (lane = row, 16 bytes) is linear and conflict-free.  A comes from
// global memory in that shape already (k contiguous); B is row-major [K, N] (n contiguous), so each
// thread loads 4 k-rows x 8 columns and transposes them inside the lane with v_perm_b32 before the
// LDS write -- the factors are used as stored, no repacked copy of U or V exists.
//
// The MFMA is issued with the B fragment as the row operand: a lane then holds, for one token row,
// 4 consecutive output columns per accumulator group, which packs to 8-byte bf16 stores into an LDS
// staging tile; from there rows leave as 16-byte fully coalesced stores (to C and/or scattered to
// the dense KV cache).  Epilogues: + bias, or the gate/up pair -> SiLU(g + b_g) * (u + b_u).
#include "prefill.hpp"
#include "decode.hpp"

namespace lr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int PBK = 64;

__host__ __device__ constexpr int plane_units(int rows) { return rows + rows / 8 + 1; }
__device__ __forceinline__ int unit_of(int plane, int chunk, int row) { return chunk * plane + row + (row >> 3); }

template <int BM, int BN> constexpr int stage_units() { return 8 * plane_units(BM) + 8 * plane_units(BN); }
template <int BM, int BN> constexpr int epi_bytes() { return BM * (BN + 4) * 2; }
template <int BM, int BN> constexpr int lds_bytes() {
    return stage_units<BM, BN>() * 16 > epi_bytes<BM, BN>() ? stage_units<BM, BN>() * 16 : epi_bytes<BM, BN>();
}

__device__ __forceinline__ uint32_t ppack2(float lo, float hi) {
    union { bf16x2_t v; uint32_t u; } x;
    x.v = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return x.u;
}

__device__ __forceinline__ bf16x8_t frag_of(const uint4& v) {
    union { uint4 u; bf16x8_t b; } x;
    x.u = v;
    return x.b;
}

__device__ __forceinline__ uint32_t dword_of(const uint4& v, int q) { return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w; }

// Global -> register loads of one k-step (64 k): NA 16-byte chunks of A per thread; of B, NR k-rows x 8
// columns per thread (NR = BN / 32: the 256 threads cover 64 k-rows x BN columns).
template <int NA, int NR, int BN>
__device__ __forceinline__ void load_tiles(uint4 (&ra)[NA], uint4 (&rb)[NR], const bf16_t* __restrict__ A, int lda,
                                           const bf16_t* __restrict__ B, int N, int M, int m0, int n0, int k0, int tid) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        const int m = m0 + row;
        if (m < M) ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)m * lda + k0 + kc * 8);
        else ra[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    constexpr int CGS = BN / 8;                          // column groups of 8
    const int cg = tid % CGS, rg = tid / CGS;            // rg: group of NR consecutive k-rows
    const bf16_t* bp = B + (size_t)(k0 + rg * NR) * N + n0 + cg * 8;
#pragma unroll
    for (int a = 0; a < NR; ++a) rb[a] = *reinterpret_cast<const uint4*>(bp + (size_t)a * N);
}

// Registers -> LDS: A chunks as they are; B transposed inside the lane: the NR k-values of one column
// become NR*2 contiguous bytes of that column's 16-byte unit.
template <int NA, int NR, int BM, int BN>
__device__ __forceinline__ void store_tiles(const uint4 (&ra)[NA], const uint4 (&rb)[NR], uint4* As, uint4* Bs, int tid) {
    constexpr int PA = plane_units(BM), PB = plane_units(BN);
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
        As[unit_of(PA, kc, row)] = ra[i];
    }
    constexpr int CGS = BN / 8;
    const int cg = tid % CGS, rg = tid / CGS;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint32_t sel = (b & 1) ? 0x07060302u : 0x05040100u;
        if constexpr (NR == 8) {
            uint4 v;
            v.x = __builtin_amdgcn_perm(dword_of(rb[1], b >> 1), dword_of(rb[0], b >> 1), sel);
            v.y = __builtin_amdgcn_perm(dword_of(rb[3], b >> 1), dword_of(rb[2], b >> 1), sel);
            v.z = __builtin_amdgcn_perm(dword_of(rb[5], b >> 1), dword_of(rb[4], b >> 1), sel);
            v.w = __builtin_amdgcn_perm(dword_of(rb[7], b >> 1), dword_of(rb[6], b >> 1), sel);
            Bs[unit_of(PB, rg, cg * 8 + b)] = v;
        } else {
            uint2 v;
            v.x = __builtin_amdgcn_perm(dword_of(rb[1], b >> 1), dword_of(rb[0], b >> 1), sel);   // k rows 4rg+0, 4rg+1 of column b
            v.y = __builtin_amdgcn_perm(dword_of(rb[3], b >> 1), dword_of(rb[2], b >> 1), sel);   // k rows 4rg+2, 4rg+3
            reinterpret_cast<uint2*>(Bs)[unit_of(PB, rg >> 1, cg * 8 + b) * 2 + (rg & 1)] = v;
        }
    }
}

template <int MI, int NI>
__device__ __forceinline__ void load_frags(bf16x8_t (&af)[MI], bf16x8_t (&bf)[NI], const uint4* a_base, const uint4* b_base,
                                           int a_step, int b_step) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) af[mi] = frag_of(a_base[a_step + mi * 36]);   // 32 rows = 36 units (pad every 8)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bf[ni] = frag_of(b_base[b_step + ni * 36]);
}

template <int MI, int NI>
__device__ __forceinline__ void mma_step(f32x16_t (&acc)[MI][NI], const bf16x8_t (&af)[MI], const bf16x8_t (&bf)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ni], af[mi], acc[mi][ni], 0, 0, 0);
}

// The matrix work of one k-step from the LDS stage at `st`.  Each sched_barrier pins the order
// "reads of substep kk+1, then MFMAs of substep kk", so the fragments of the next substep are in
// flight for a whole substep of matrix work.
template <int BM, int BN>
__device__ __forceinline__ void compute_stage(f32x16_t (&acc)[BM / 64][BN / 64], const uint4* st, int a_off, int b_off) {
    constexpr int MI = BM / 64, NI = BN / 64;
    constexpr int PA = plane_units(BM), PB = plane_units(BN);
    const uint4* a_base = st + a_off;
    const uint4* b_base = st + b_off;
    bf16x8_t af0[MI], bf0[NI], af1[MI], bf1[NI];
    load_frags<MI, NI>(af0, bf0, a_base, b_base, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    load_frags<MI, NI>(af1, bf1, a_base, b_base, 2 * PA, 2 * PB);
    __builtin_amdgcn_sched_barrier(0);
    mma_step<MI, NI>(acc, af0, bf0);
    __builtin_amdgcn_sched_barrier(0);
    load_frags<MI, NI>(af0, bf0, a_base, b_base, 4 * PA, 4 * PB);
    __builtin_amdgcn_sched_barrier(0);
    mma_step<MI, NI>(acc, af1, bf1);
    __builtin_amdgcn_sched_barrier(0);
    load_frags<MI, NI>(af1, bf1, a_base, b_base, 6 * PA, 6 * PB);
    __builtin_amdgcn_sched_barrier(0);
    mma_step<MI, NI>(acc, af0, bf0);
    __builtin_amdgcn_sched_barrier(0);
    mma_step<MI, NI>(acc, af1, bf1);
    __builtin_amdgcn_sched_barrier(0);
}

// One K loop: acc[mi][ni] += (B tile)^T x (A tile)^T over k in [0, K).  One LDS buffer, two barriers
// per k-step, global data of the next step prefetched into registers; two or three workgroups per
// CU overlap each other's store phases.  (A two-buffer variant with one barrier per step and a
// 256 x 256 tile were measured slower on this chip: 786 / 909 vs 941 TFLOP/s on an 8192^3 product.)
template <int BM, int BN>
__device__ __forceinline__ void gemm_loop(f32x16_t (&acc)[BM / 64][BN / 64], const bf16_t* __restrict__ A, int lda,
                                          const bf16_t* __restrict__ B, int N, int K, int M, int m0, int n0, uint4* lds) {
    constexpr int NA = BM / 32, NR = BN / 32;
    constexpr int PA = plane_units(BM), PB = plane_units(BN);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lg = lane >> 5;
    // fragment offsets of this lane for k-substep 0 (chunk lg); substep kk adds 2*kk planes
    const int a_off = unit_of(PA, lg, wm * (BM / 2) + li);
    const int b_off = 8 * PA + unit_of(PB, lg, wn * (BN / 2) + li);

    uint4 ra[NA], rb[NR];
    const int nk = K / PBK;
    load_tiles<NA, NR, BN>(ra, rb, A, lda, B, N, M, m0, n0, 0, tid);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();                 // everyone finished reading the previous tile
        store_tiles<NA, NR, BM, BN>(ra, rb, lds, lds + 8 * PA, tid);
        __syncthreads();
        if (kt + 1 < nk) load_tiles<NA, NR, BN>(ra, rb, A, lda, B, N, M, m0, n0, (kt + 1) * PBK, tid);
        compute_stage<BM, BN>(acc, lds, a_off, b_off);
    }
}

// ---- direct-to-LDS pipeline ---------------------------------------------------------------------
// Measured on this chip: loads that return through the vector registers deliver at most ~76 B/ns per
// CU (a 256 x 256 x 64 tile step then needs as long for its 64 KB as for its 2048 MFMA cycles, and
// with one wave per SIMD the two do not overlap), while global_load_lds_dwordx4 streams 126-144 B/ns
// per CU into LDS with no register, no ds_write and no issue slot beyond the instruction itself.
// So both operands travel global -> LDS directly, as they are in memory:
//   A tile [BM rows][32 k]: row = 4 units of 16 bytes; unit c of row m sits at m*4 + (c ^ ((m >> 2) & 3)),
//     which makes the 16-byte fragment reads of 16 consecutive rows sweep all 64 banks;
//   B tile [32 k][BN columns], n contiguous as in memory: unit u of row k sits at k*(BN/8) + (u ^ ((k & 3) << 2));
//     ds_read_b64_tr_b16 turns 4 k-rows x 16 columns into "4 consecutive k of one column per lane",
//     two of them make the 8-k MFMA fragment; the XOR spreads the 4 rows of one read over the banks.
// The permutation costs nothing: a lane of the load writes LDS unit (block base + lane) and simply
// fetches the global unit that belongs there.
// Ring of 4 stages of 32 k; per step one barrier, placed between the two 16-k substeps so the
// fragments of the next stage are read under the second substep's MFMAs.  The tile of step kt+4 is
// requested right after the barrier of step kt (which frees its stage) and is first needed after
// the barrier of step kt+3.
constexpr int DBK = 32;                 // k per stage
constexpr int DSTAGES = 4;
template <int BM, int BN> constexpr int dma_stage_bytes() { return BM * 64 + 32 * BN * 2; }
template <int BM, int BN> constexpr int dma_lds_bytes() {
    return DSTAGES * dma_stage_bytes<BM, BN>() > epi_bytes<BM, BN>() ? DSTAGES * dma_stage_bytes<BM, BN>() : epi_bytes<BM, BN>();
}

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

// 64 lanes x 16 bytes: global (sbase + voff[lane]) -> LDS (lds_byte + 16 * lane); counted by vmcnt.
__device__ __forceinline__ void dma16(uint32_t lds_byte, uint32_t voff, const void* sbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_byte), "v"(voff), "s"(sbase) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vm_lgkm0() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(N) : "memory");
}

template <int BM, int BN>
struct DmaCtx {
    static constexpr int NA = BM / 64, NR = BN / 64;      // load instructions per wave and step
    static constexpr int UR = BN / 8;                     // 16-byte units per B row
    const char* sa; const char* sb;                       // uniform: tile origin of A (row m0, k 0) and B (k 0, column n0)
    uint32_t voa[NA], vob[NR];                            // per-lane byte offsets inside the step's tile
    uint32_t step_a, step_b;                              // bytes per k-step
    uint32_t lds0;                                        // LDS byte address of stage 0
    int wave;
};

template <int BM, int BN>
__device__ __forceinline__ void dma_setup(DmaCtx<BM, BN>& c, const bf16_t* A, int lda, const bf16_t* B, int N, int M, int m0, int n0, uint4* lds) {
    constexpr int NA = DmaCtx<BM, BN>::NA, NR = DmaCtx<BM, BN>::NR, UR = DmaCtx<BM, BN>::UR;
    const int tid = threadIdx.x, lane = tid & 63;
    c.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    c.sa = reinterpret_cast<const char*>(A + (size_t)m0 * lda);
    c.sb = reinterpret_cast<const char*>(B + n0);
    c.step_a = DBK * 2; c.step_b = (uint32_t)DBK * (uint32_t)N * 2u;
    c.lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)lds);
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int row = (c.wave * NA + j) * 16 + (lane >> 2), pos = lane & 3;
        int m = m0 + row; m = m < M ? m : M - 1;          // rows past the end repeat the last row; never stored
        c.voa[j] = (uint32_t)(m - m0) * (uint32_t)lda * 2u + (uint32_t)((pos ^ ((row >> 2) & 3)) * 16);
    }
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int k = (c.wave * NR + j) * (64 / UR) + lane / UR, pos = lane % UR;
        c.vob[j] = (uint32_t)k * (uint32_t)N * 2u + (uint32_t)((pos ^ ((k & 3) << 2)) * 16);
    }
}

// request tile t (k range [32 t, 32 t + 32)) into its ring stage
template <int BM, int BN>
__device__ __forceinline__ void dma_issue(const DmaCtx<BM, BN>& c, int t) {
    constexpr int NA = DmaCtx<BM, BN>::NA, NR = DmaCtx<BM, BN>::NR;
    const uint32_t st = c.lds0 + (uint32_t)(t & (DSTAGES - 1)) * dma_stage_bytes<BM, BN>();
    const char* ga = c.sa + (size_t)t * c.step_a;
    const char* gb = c.sb + (size_t)t * c.step_b;
#pragma unroll
    for (int j = 0; j < NA; ++j) dma16(st + (uint32_t)(c.wave * NA + j) * 1024u, c.voa[j], ga);
#pragma unroll
    for (int j = 0; j < NR; ++j) dma16(st + (uint32_t)(BM * 64) + (uint32_t)(c.wave * NR + j) * 1024u, c.vob[j], gb);
}

template <int BM, int BN>
struct FragAddr {
    uint32_t a[2];              // byte offset in a stage of this lane's A unit for substep kk (row block 0)
    uint32_t b[BN / 64];        // byte offset in a stage of this lane's B word for column block ni (substep 0, first half)
};

template <int BM, int BN>
__device__ __forceinline__ void frag_setup(FragAddr<BM, BN>& f) {
    constexpr int NI = BN / 64;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lg = lane >> 5;
    const int row = wm * (BM / 2) + li;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) f.a[kk] = (uint32_t)(row * 64 + (((2 * kk + lg) ^ ((row >> 2) & 3)) * 16));
    // transposing read: inside each block of 16 lanes, source lane s hands in row (s >> 2) and the
    // 4 columns 4 * (s & 3)...; result lane i then holds column i of the block, 4 consecutive rows
    const int s = lane & 15, blk = (lane >> 4) & 1, q = s >> 2;
    const int k = lg * 8 + q;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int col = wn * (BN / 2) + ni * 32 + blk * 16 + 4 * (s & 3);
        const int u = col >> 3, half = (col >> 2) & 1;
        f.b[ni] = (uint32_t)(BM * 64 + k * (BN * 2) + ((u ^ (q << 2)) * 16) + half * 8);
    }
}

template <int BM, int BN, int MI_ONE>
__device__ __forceinline__ bf16x8_t dma_read_a(const char* stage, const FragAddr<BM, BN>& f, int kk) {
    return frag_of(*reinterpret_cast<const uint4*>(stage + f.a[kk] + MI_ONE * 32 * 64));
}
template <int BM, int BN, int NI_ONE>
__device__ __forceinline__ bf16x8_t dma_read_b(const char* stage, const FragAddr<BM, BN>& f, int kk) {
    union { struct { s16x4_t lo, hi; } h; bf16x8_t b; } x;
    const char* p = stage + f.b[NI_ONE] + kk * 16 * (BN * 2);
    x.h.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p));
    x.h.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * (BN * 2)));
    return x.b;
}

// Fragment reads of one "chunk" C (one of the MI row blocks of the wave tile): A fragment C and the
// B fragments dealt evenly over the chunks.
template <int BM, int BN, int C, int NIi>
__device__ __forceinline__ void dma_maybe_read_b(bf16x8_t (&bfn)[BN / 64], const char* stage, const FragAddr<BM, BN>& f, int kk) {
    constexpr int MI = BM / 64, NI = BN / 64;
    if constexpr (NIi < NI) {
        if constexpr ((NIi * MI) / NI == C) {
#ifndef LR_ABLATE_READS_B
            bfn[NIi] = dma_read_b<BM, BN, NIi>(stage, f, kk);
#endif
        }
    }
}
template <int BM, int BN, int C>
__device__ __forceinline__ void dma_read_chunk(bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* stage, const FragAddr<BM, BN>& f, int kk) {
#ifndef LR_ABLATE_READS
#ifndef LR_ABLATE_READS_A
    afn[C] = dma_read_a<BM, BN, C>(stage, f, kk);
#endif
    dma_maybe_read_b<BM, BN, C, 0>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 1>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 2>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 3>(bfn, stage, f, kk);
#endif
}

// chunk C of a substep: its share of the next substep's fragment reads, then the MFMAs of row block C
template <int BM, int BN, int C>
__device__ __forceinline__ void dma_chunk(f32x16_t (&acc)[BM / 64][BN / 64], const bf16x8_t (&afc)[BM / 64], const bf16x8_t (&bfc)[BN / 64],
                                          bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* nstage,
                                          const FragAddr<BM, BN>& f, int nkk) {
    constexpr int MI = BM / 64, NI = BN / 64;
    if constexpr (C < MI) {
        dma_read_chunk<BM, BN, C>(afn, bfn, nstage, f, nkk);
#ifndef LR_ABLATE_MFMA
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc[C][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfc[ni], afc[C], acc[C][ni], 0, 0, 0);
#endif
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int BM, int BN>
__device__ __forceinline__ void dma_substep(f32x16_t (&acc)[BM / 64][BN / 64], const bf16x8_t (&afc)[BM / 64], const bf16x8_t (&bfc)[BN / 64],
                                            bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* nstage,
                                            const FragAddr<BM, BN>& f, int nkk) {
    dma_chunk<BM, BN, 0>(acc, afc, bfc, afn, bfn, nstage, f, nkk);
    dma_chunk<BM, BN, 1>(acc, afc, bfc, afn, bfn, nstage, f, nkk);
    dma_chunk<BM, BN, 2>(acc, afc, bfc, afn, bfn, nstage, f, nkk);
    dma_chunk<BM, BN, 3>(acc, afc, bfc, afn, bfn, nstage, f, nkk);
}

template <int BM, int BN>
__device__ __forceinline__ void gemm_loop_dma(f32x16_t (&acc)[BM / 64][BN / 64], const bf16_t* __restrict__ A, int lda,
                                              const bf16_t* __restrict__ B, int N, int K, int M, int m0, int n0, uint4* lds) {
    constexpr int MI = BM / 64, NI = BN / 64;
    constexpr int L = DmaCtx<BM, BN>::NA + DmaCtx<BM, BN>::NR;     // loads per wave and tile
    constexpr int SB = dma_stage_bytes<BM, BN>();
    DmaCtx<BM, BN> c;
    FragAddr<BM, BN> f;
    dma_setup<BM, BN>(c, A, lda, B, N, M, m0, n0, lds);
    frag_setup<BM, BN>(f);
    const char* ring = reinterpret_cast<const char*>(lds);
    const int nk = K / DBK;

    // all waves are past their last use of this LDS (a previous K loop or nothing)
    __builtin_amdgcn_s_barrier();
    for (int t = 0; t < DSTAGES; ++t) if (t < nk) dma_issue<BM, BN>(c, t);
    if (nk >= DSTAGES) wait_vm_lgkm0<3 * L>(); else wait_vm_lgkm0<0>();
    __builtin_amdgcn_s_barrier();
    bf16x8_t af0[MI], bf0[NI], af1[MI], bf1[NI];
    dma_read_chunk<BM, BN, 0>(af0, bf0, ring, f, 0);
    if constexpr (MI > 1) dma_read_chunk<BM, BN, 1>(af0, bf0, ring, f, 0);
    if constexpr (MI > 2) dma_read_chunk<BM, BN, 2>(af0, bf0, ring, f, 0);
    if constexpr (MI > 3) dma_read_chunk<BM, BN, 3>(af0, bf0, ring, f, 0);
    __builtin_amdgcn_sched_barrier(0);

    for (int kt = 0; kt < nk; ++kt) {
        const char* cur = ring + (kt & (DSTAGES - 1)) * SB;
        const char* nxt = ring + ((kt + 1) & (DSTAGES - 1)) * SB;
        const bool more = kt + DSTAGES < nk;          // uniform
        dma_substep<BM, BN>(acc, af0, bf0, af1, bf1, cur, f, 1);
        // own part of tile kt+1 has landed (tiles kt+2, kt+3 may still fly; near the end simply wait for
        // everything) and own reads of stage kt are done
        if (more) wait_vm_lgkm0<2 * L>(); else wait_vm_lgkm0<0>();
        __builtin_amdgcn_s_barrier();
#ifndef LR_ABLATE_DMA
        if (more) dma_issue<BM, BN>(c, kt + DSTAGES); // the stage of tile kt is free now
#endif
        __builtin_amdgcn_sched_barrier(0);
        // after the last step this reads a stale stage: in bounds, never used
        dma_substep<BM, BN>(acc, af1, bf1, af0, bf0, nxt, f, 0);
    }
}

template <int BM, int BN, int EPI, int MINB, bool DMA>
__global__ void __launch_bounds__(256, MINB) k_prefill_gemm(PArgs pa) {
    constexpr int MI = BM / 64, NI = BN / 64;
    __shared__ uint4 lds[(DMA ? dma_lds_bytes<BM, BN>() : lds_bytes<BM, BN>()) / 16];
    // Tile order.  Workgroups are dealt round-robin to the 8 XCDs, each with its own 4 MB L2: workgroup
    // id -> (id % 8) * total/8 + id / 8 gives every XCD a contiguous range of the logical order, and the
    // logical order walks groups of pa.group_m tile rows column by column, so the workgroups that run
    // together on one XCD share both a few A row-tiles and a few B column-tiles.
    const int per_prob = pa.tiles_m * pa.tiles_n_max;
    const int total = per_prob * pa.nprob;
    int id = blockIdx.x;
    if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int prob = id / per_prob;
    const int rem = id - prob * per_prob;
    const int gsz = pa.group_m * pa.tiles_n_max;
    const int mg = rem / gsz, r = rem - mg * gsz;
    const int rows_here = (pa.tiles_m - mg * pa.group_m) < pa.group_m ? (pa.tiles_m - mg * pa.group_m) : pa.group_m;
    const int tn = r / rows_here, tm = mg * pa.group_m + (r - tn * rows_here);
    const PProb& P = pa.p[prob];
    if (tn * BN >= P.N) return;
    const int m0 = tm * BM, n0 = tn * BN, M = pa.M;

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    if constexpr (DMA) gemm_loop_dma<BM, BN>(acc, P.A, P.lda, P.B, P.N, P.K, M, m0, n0, lds);
    else gemm_loop<BM, BN>(acc, P.A, P.lda, P.B, P.N, P.K, M, m0, n0, lds);

    f32x16_t acc2[(EPI == PEPI_GATEUP) ? MI : 1][(EPI == PEPI_GATEUP) ? NI : 1];
    if constexpr (EPI == PEPI_GATEUP) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[mi][ni][v] = 0.f;
        if constexpr (DMA) gemm_loop_dma<BM, BN>(acc2, P.A2, P.lda2, P.B2, P.N, P.K2, M, m0, n0, lds);
        else gemm_loop<BM, BN>(acc2, P.A2, P.lda2, P.B2, P.N, P.K2, M, m0, n0, lds);
    }

    // ---- epilogue: registers -> bf16 staging tile in LDS -> coalesced 16-byte row stores
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lg = lane >> 5;
    constexpr int CS = BN + 4;                        // staging row stride in bf16: 8-byte lanes of a wave sweep the banks
    __syncthreads();                                  // main-loop LDS no longer needed
    bf16_t* Cs = reinterpret_cast<bf16_t*>(lds);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const int col = wn * (BN / 2) + ni * 32 + 8 * vg + 4 * lg;    // first of this lane's 4 consecutive columns
            float bg[4] = {0.f, 0.f, 0.f, 0.f}, bu[4] = {0.f, 0.f, 0.f, 0.f};
            if (P.bias) {
                const uint2 raw = *reinterpret_cast<const uint2*>(P.bias + n0 + col);
                bg[0] = __uint_as_float(raw.x << 16); bg[1] = __uint_as_float(raw.x & 0xffff0000u);
                bg[2] = __uint_as_float(raw.y << 16); bg[3] = __uint_as_float(raw.y & 0xffff0000u);
            }
            if constexpr (EPI == PEPI_GATEUP) {
                if (P.bias2) {
                    const uint2 raw = *reinterpret_cast<const uint2*>(P.bias2 + n0 + col);
                    bu[0] = __uint_as_float(raw.x << 16); bu[1] = __uint_as_float(raw.x & 0xffff0000u);
                    bu[2] = __uint_as_float(raw.y << 16); bu[3] = __uint_as_float(raw.y & 0xffff0000u);
                }
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row = wm * (BM / 2) + mi * 32 + li;             // token row inside the tile
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (EPI == PEPI_GATEUP)
                        v[e] = silu_f32(acc[mi][ni][4 * vg + e] + bg[e]) * (acc2[mi][ni][4 * vg + e] + bu[e]);
                    else
                        v[e] = acc[mi][ni][4 * vg + e] + bg[e];
                }
                uint2 o; o.x = ppack2(v[0], v[1]); o.y = ppack2(v[2], v[3]);
                *reinterpret_cast<uint2*>(Cs + row * CS + col) = o;
            }
        }
    __syncthreads();
    constexpr int CPR = BN / 8;                       // 16-byte chunks per tile row
    constexpr int CHUNKS = BM * CPR;
#pragma unroll 4
    for (int c = tid; c < CHUNKS; c += 256) {
        const int row = c / CPR, ch = c % CPR;
        const int m = m0 + row;
        if (m >= M) continue;
        const uint2 lo = *reinterpret_cast<const uint2*>(Cs + row * CS + ch * 8);
        const uint2 hi = *reinterpret_cast<const uint2*>(Cs + row * CS + ch * 8 + 4);
        const uint4 val = make_uint4(lo.x, lo.y, hi.x, hi.y);
        if (P.C) *reinterpret_cast<uint4*>(P.C + (size_t)m * P.ldc + n0 + ch * 8) = val;
        if constexpr (EPI == PEPI_STORE) {
            if (P.cache) {
                const int bi = m / P.T, s = m - bi * P.T;
                const int64_t pp = (int64_t)P.pos[bi] + s;
                if (pp >= 0 && pp < P.S_max)
                    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(P.cache) + ((size_t)bi * P.S_max + (size_t)pp) * P.N + n0 + ch * 8) = val;
            }
        }
    }
}

// Fast-path rule: K in 64-row steps, N in 128-column tiles, any M >= 1.
bool prefill_shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && M < (1 << 30) && K >= 64 && (K % 64) == 0 && N >= 128 && (N % 128) == 0 &&
           K < (1 << 24) && N < (1 << 24);
}

template <int BM, int BN, int EPI, int MINB, bool DMA>
static int launch_cfg(PArgs a, hipStream_t s) {
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n_max = 0;
    for (int i = 0; i < a.nprob; ++i) { const int t = (a.p[i].N + BN - 1) / BN; if (t > a.tiles_n_max) a.tiles_n_max = t; }
    const int total = a.tiles_m * a.tiles_n_max * a.nprob;
    a.group_m = 8;
    a.trace = g_trace_buffer;
    hipLaunchKernelGGL((k_prefill_gemm<BM, BN, EPI, MINB, DMA>), dim3((unsigned)total), dim3(256), 0, s, a);
    return launch_status("prefill gemm");
}

static int env_int(const char* name) { const char* v = getenv(name); return v ? atoi(v) : -1; }
static int env_shape() { static int v = env_int("LOWRANK_PREFILL_SHAPE"); return v; }
static int env_gu() { static int v = env_int("LOWRANK_PREFILL_GU"); return v; }

static bool want_bm256(const PArgs& a) {
    long tiles = 0;
    for (int i = 0; i < a.nprob; ++i) tiles += (long)((a.M + 255) / 256) * (a.p[i].N / 128);
    return tiles >= 4 * 512;
}

int prefill_launch(const PArgs& a, int epi, hipStream_t s) {
    if (a.M <= 0 || a.nprob <= 0) return LR_OK;
    bool n256 = true;
    for (int i = 0; i < a.nprob; ++i) n256 = n256 && (a.p[i].N % 256 == 0);
    if (epi == PEPI_GATEUP) {
        switch (env_gu()) {
            case 0: return launch_cfg<128, 128, PEPI_GATEUP, 2, false>(a, s);
            case 2: return launch_cfg<256, 128, PEPI_GATEUP, 1, true>(a, s);
            default: return launch_cfg<128, 128, PEPI_GATEUP, 2, true>(a, s);
        }
    }
    switch (env_shape()) {
        case 0: if (n256) return launch_cfg<256, 256, PEPI_STORE, 1, true>(a, s); break;
        case 1: return launch_cfg<256, 128, PEPI_STORE, 2, false>(a, s);
        case 2: return launch_cfg<128, 128, PEPI_STORE, 2, false>(a, s);
        case 3: return launch_cfg<256, 128, PEPI_STORE, 1, true>(a, s);
        case 4: if (n256) return launch_cfg<128, 256, PEPI_STORE, 1, true>(a, s); break;
        case 5: return launch_cfg<128, 128, PEPI_STORE, 2, true>(a, s);
        default: break;
    }
    return launch_cfg<128, 128, PEPI_STORE, 2, true>(a, s);
}

}  // namespace lr
