// Prefill-phase GEMM (bf16 MFMA): C[M, N] = A[M, K] * B[K, N] with A, B, C row-major, as a persistent
// kernel whose operands travel global memory -> LDS directly (global_load_lds_dwordx4).
//
// Tile BM x BN per workgroup of 4 waves (2 x 2), each wave (BM/2) x (BN/2) built from
// v_mfma_f32_32x32x16_bf16.  The factors are used as stored -- no repacked copy of U or V exists:
// A is k-contiguous in memory and its 16-byte units are read back as MFMA fragments as they are;
// B is [K, N] with n contiguous and its fragments ("8 consecutive k of one column per lane") are
// produced by the transposing LDS read ds_read_b64_tr_b16.
//
// The MFMA is issued with the B fragment as the row operand: a lane then holds, for one token row,
// 4 consecutive output columns per accumulator group, which packs to 8-byte bf16 writes into a small
// per-wave LDS patch; from there rows leave as 16-byte stores covering whole 128-byte lines (to C
// and/or scattered to the dense KV cache).  Epilogues: + bias, or the gate/up pair ->
// SiLU(g + b_g) * (u + b_u).
#include <string.h>
#include <stdlib.h>
#include "prefill.hpp"
#include "decode.hpp"

namespace lr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

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

// Where unit u (16 bytes = 8 columns) of row k of a B tile sits inside its LDS row of UR = BN/8 units, and the
// inverse.  Power-of-two rows: XOR with 4 * (k & 3).  192-column tiles (24 units, 384 bytes = 1.5 times the
// bank space, so rows k and k+2 would meet): rows with bit 1 of k set are rotated by 4 units.  Either way the
// 4 rows x 2 column blocks that one half-wave of a transposing read touches fall into 8 different 32-byte bank groups.
template <int BN> __device__ __forceinline__ int b_lds_pos(int k, int u) {
    constexpr int UR = BN / 8;
    if constexpr ((UR & (UR - 1)) == 0) return u ^ ((k & 3) << 2);
    else { const int p = u + 4 * ((k >> 1) & 1); return p >= UR ? p - UR : p; }
}
template <int BN> __device__ __forceinline__ int b_unit_at(int k, int pos) {
    constexpr int UR = BN / 8;
    if constexpr ((UR & (UR - 1)) == 0) return pos ^ ((k & 3) << 2);
    else { const int u = pos - 4 * ((k >> 1) & 1); return u < 0 ? u + UR : u; }
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
        f.b[ni] = (uint32_t)(BM * 64 + k * (BN * 2) + b_lds_pos<BN>(k, u) * 16 + half * 8);   // k & 3 and bit 1 of k do not change with substep or half
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
            bfn[NIi] = dma_read_b<BM, BN, NIi>(stage, f, kk);
        }
    }
}
template <int BM, int BN, int C>
__device__ __forceinline__ void dma_read_chunk(bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* stage, const FragAddr<BM, BN>& f, int kk) {
    afn[C] = dma_read_a<BM, BN, C>(stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 0>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 1>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 2>(bfn, stage, f, kk);
    dma_maybe_read_b<BM, BN, C, 3>(bfn, stage, f, kk);
}

// chunk C of a substep: its share of the next substep's fragment reads, then the MFMAs of row block C
// No requests between the MFMAs of a substep.
struct NoIssue { template <int J> __device__ __forceinline__ void issue() const {} };

// MFMA number NIi of chunk C, followed by the request instruction (if any) that belongs behind it: the
// L request instructions of a step are spread evenly over the MI * NI MFMAs of a substep.  A request
// occupies the issue port for tens of cycles while the memory pipeline takes it in; right behind an
// MFMA it hides under that MFMA's 32 cycles, whereas a burst of 8 stalls the matrix pipeline.
template <int BM, int BN, int C, int NIi, bool ZERO, class IS>
__device__ __forceinline__ void dma_mfma_one(f32x16_t (&acc)[BM / 64][BN / 64], const bf16x8_t (&afc)[BM / 64], const bf16x8_t (&bfc)[BN / 64], const IS& is) {
    constexpr int MI = BM / 64, NI = BN / 64, S = MI * NI, L = MI + NI;
    if constexpr (NIi < NI) {
        if constexpr (ZERO) {       // first product of a tile: the accumulator starts from the constant 0
            const f32x16_t z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[C][NIi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfc[NIi], afc[C], z, 0, 0, 0);
        } else {
            acc[C][NIi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfc[NIi], afc[C], acc[C][NIi], 0, 0, 0);
        }
        constexpr int slot = C * NI + NIi;
        constexpr int j = (slot * L + S - 1) / S;           // the request whose place floor(j * S / L) could be this slot
        if constexpr (j < L && (j * S) / L == slot) {
            __builtin_amdgcn_sched_barrier(0);
            is.template issue<j>();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// chunk C of a substep: its share of the next substep's fragment reads, then the MFMAs of row block C
template <int BM, int BN, int C, bool ZERO, bool READ, class IS>
__device__ __forceinline__ void dma_chunk(f32x16_t (&acc)[BM / 64][BN / 64], const bf16x8_t (&afc)[BM / 64], const bf16x8_t (&bfc)[BN / 64],
                                          bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* nstage,
                                          const FragAddr<BM, BN>& f, int nkk, const IS& is) {
    constexpr int MI = BM / 64;
    if constexpr (C < MI) {
        // the reads are packed into the first chunks so that the last ones are a chunk of MFMAs old when
        // the wave waits for them in front of the barrier
        if constexpr (READ) {
            if constexpr (C == 0) {
                dma_read_chunk<BM, BN, 0>(afn, bfn, nstage, f, nkk);
                if constexpr (MI > 1) dma_read_chunk<BM, BN, 1>(afn, bfn, nstage, f, nkk);
            } else if constexpr (C + 1 < MI) {
                dma_read_chunk<BM, BN, C + 1>(afn, bfn, nstage, f, nkk);
            }
        }
        dma_mfma_one<BM, BN, C, 0, ZERO, IS>(acc, afc, bfc, is);
        dma_mfma_one<BM, BN, C, 1, ZERO, IS>(acc, afc, bfc, is);
        dma_mfma_one<BM, BN, C, 2, ZERO, IS>(acc, afc, bfc, is);
        dma_mfma_one<BM, BN, C, 3, ZERO, IS>(acc, afc, bfc, is);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int BM, int BN, bool ZERO, bool READ, class IS>
__device__ __forceinline__ void dma_substep(f32x16_t (&acc)[BM / 64][BN / 64], const bf16x8_t (&afc)[BM / 64], const bf16x8_t (&bfc)[BN / 64],
                                            bf16x8_t (&afn)[BM / 64], bf16x8_t (&bfn)[BN / 64], const char* nstage,
                                            const FragAddr<BM, BN>& f, int nkk, const IS& is) {
    dma_chunk<BM, BN, 0, ZERO, READ, IS>(acc, afc, bfc, afn, bfn, nstage, f, nkk, is);
    dma_chunk<BM, BN, 1, ZERO, READ, IS>(acc, afc, bfc, afn, bfn, nstage, f, nkk, is);
    dma_chunk<BM, BN, 2, ZERO, READ, IS>(acc, afc, bfc, afn, bfn, nstage, f, nkk, is);
    dma_chunk<BM, BN, 3, ZERO, READ, IS>(acc, afc, bfc, afn, bfn, nstage, f, nkk, is);
}

// ---- persistent form ----------------------------------------------------------------------------
// One workgroup per CU slot walks a list of tiles; the request ring never drains between tiles: while
// a tile's last steps are multiplied and its result leaves, the first stages of the next tile are
// already on their way.  Each wave stores its own part of the result through a private 4 KB LDS patch
// (32 rows x 64 columns, 16-byte units XOR-swizzled by row), so the epilogue needs no workgroup
// barrier and the rows leave as full 128-byte lines.
template <int BM, int BN> constexpr int persist_lds_bytes() { return DSTAGES * dma_stage_bytes<BM, BN>() + 4 * 4096; }

// what the requester needs to know about one operand pair (A, B over K) of one tile
template <int BM, int BN>
struct Stream {
    const char* sa; const char* sb;
    uint32_t voa[BM / 64], vob[BN / 64];
    uint32_t step_b;
};

template <int BM, int BN>
__device__ __forceinline__ void stream_setup(Stream<BM, BN>& c, const bf16_t* A, int lda, const bf16_t* B, int N, int K,
                                             int M, int m0, int n0, int wave, int lane) {
    constexpr int NA = BM / 64, NR = BN / 64, UR = BN / 8;
    c.sa = reinterpret_cast<const char*>(A + (size_t)m0 * lda);
    c.sb = reinterpret_cast<const char*>(B + n0);
    c.step_b = (uint32_t)DBK * (uint32_t)N * 2u;
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        const int row = (wave * NA + j) * 16 + (lane >> 2), pos = lane & 3;
        int m = m0 + row; m = m < M ? m : M - 1;          // rows past the end repeat the last row; never stored
        c.voa[j] = (uint32_t)(m - m0) * (uint32_t)lda * 2u + (uint32_t)((pos ^ ((row >> 2) & 3)) * 16);
    }
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int lin = (wave * NR + j) * 64 + lane;          // LDS unit of the tile this lane fills
        const int k = lin / UR, pos = lin % UR;
        int col = b_unit_at<BN>(k, pos) * 8;
        col = (n0 + col + 8 <= N) ? col : N - 8 - n0;     // columns past the end repeat the last unit; never stored
        c.vob[j] = (uint32_t)k * (uint32_t)N * 2u + (uint32_t)(col * 2);
    }
}

// a wave-uniform pointer, said so to the compiler (it then sits in scalar registers)
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>((uintptr_t)(((uint64_t)hi << 32) | lo));
}

// The request instructions of one k-step, to be issued one by one (issue<J>, J < NA + NR).
template <int BM, int BN>
struct StepIssue {
    static constexpr int NA = BM / 64, NR = BN / 64;
    const Stream<BM, BN>* st;
    const char* ga; const char* gb;         // uniform: this step's origin in A and B
    uint32_t stage_lds;                     // uniform: LDS byte address of the ring stage
    int wave;
    bool on;                                // uniform: false when nothing is left to request
    template <int J> __device__ __forceinline__ void issue() const {
        if (on) {
            if constexpr (J < NA) dma16(stage_lds + (uint32_t)(wave * NA + J) * 1024u, st->voa[J], ga);
            else dma16(stage_lds + (uint32_t)(BM * 64) + (uint32_t)(wave * NR + (J - NA)) * 1024u, st->vob[J - NA], gb);
        }
    }
};

template <int BM, int BN>
__device__ __forceinline__ StepIssue<BM, BN> stream_step(const Stream<BM, BN>& c, int kt, uint32_t stage_lds, int wave, bool on) {
    StepIssue<BM, BN> is;
    is.st = &c;
    is.ga = uniform_ptr(c.sa + (size_t)kt * (DBK * 2));
    is.gb = uniform_ptr(c.sb + (size_t)kt * c.step_b);
    is.stage_lds = __builtin_amdgcn_readfirstlane(stage_lds);
    is.wave = wave; is.on = on;
    return is;
}

template <int BM, int BN, int J>
__device__ __forceinline__ void issue_all(const StepIssue<BM, BN>& is) {
    if constexpr (J < BM / 64 + BN / 64) { is.template issue<J>(); issue_all<BM, BN, J + 1>(is); }
}

// The work of one workgroup, as a sequence of segments: a tile and a range of its k-steps.
// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so "logical" workgroup
// (id % 8) * (grid / 8) + id / 8 makes the workgroups of one XCD neighbours in the logical order.
// The logical tile order walks groups of group_m tile rows column by column, so tiles in flight on
// one XCD share A row-panels and B column-panels.
//   tile walk (pa.sk == 0): XCD x owns a contiguous eighth of the tiles and its workgroups take
//     consecutive tiles together, round after round; every segment is a whole tile.
//   shared-K walk (pa.sk == 1, all problems of one shape): the launch is one long sequence of k-steps
//     (tile after tile), cut into equal ranges, one per logical workgroup.  A workgroup whose range
//     starts inside a tile hands its partial sums (fp32) to the workgroup holding the tile's k = 0 step.
struct Seg { int prob, m0, n0, kb, ke; };
struct Walk { int next, end, stride; };      // tile walk: tile ids; shared-K walk: k-step units [next, end)

__device__ __forceinline__ int logical_wg() { return (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3); }
__device__ __forceinline__ int sk_unit_begin(const PArgs& pa, int wl) {   // first k-step unit of logical workgroup wl
    const long long units = (long long)pa.tiles_m * pa.tiles_n_max * pa.nprob * pa.sk_nk;
    return (int)(units * wl / (int)gridDim.x);
}

__device__ __forceinline__ Walk walk_begin(const PArgs& pa) {
    Walk w;
    if (pa.sk) {
        const int wl = logical_wg();
        w.next = sk_unit_begin(pa, wl); w.end = sk_unit_begin(pa, wl + 1); w.stride = 0;
    } else {
        const int total = pa.tiles_m * pa.tiles_n_max * pa.nprob;
        const int per_xcd = (total + 7) >> 3;
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3, slots = gridDim.x >> 3;
        w.next = x * per_xcd + j;
        w.end = (x + 1) * per_xcd < total ? (x + 1) * per_xcd : total;
        w.stride = slots;
    }
    return w;
}

template <int BM, int BN>
__device__ __forceinline__ bool tile_of(const PArgs& pa, int id, Seg& sg) {
    const int per_prob = pa.tiles_m * pa.tiles_n_max;
    const int gsz = pa.group_m * pa.tiles_n_max;
    const int pr = id / per_prob, rem = id - pr * per_prob;
    const int mg = rem / gsz, r = rem - mg * gsz;
    const int rows_here = (pa.tiles_m - mg * pa.group_m) < pa.group_m ? (pa.tiles_m - mg * pa.group_m) : pa.group_m;
    const int tn = r / rows_here, tm = mg * pa.group_m + (r - tn * rows_here);
    sg.prob = pr; sg.m0 = tm * BM; sg.n0 = tn * BN;
    return tn * BN < pa.p[pr].N;
}

template <int BM, int BN>
__device__ __forceinline__ bool walk_next(Walk& w, const PArgs& pa, Seg& sg) {
    if (pa.sk) {
        if (w.next >= w.end) return false;
        const int tile = w.next / pa.sk_nk;
        sg.kb = w.next - tile * pa.sk_nk;
        const int left = w.end - w.next;
        sg.ke = sg.kb + left < pa.sk_nk ? sg.kb + left : pa.sk_nk;
        w.next += sg.ke - sg.kb;
        tile_of<BM, BN>(pa, tile, sg);           // every tile of a shared-K launch is a real one
        return true;
    }
    while (w.next < w.end) {
        const int id = w.next;
        w.next += w.stride;
        if (tile_of<BM, BN>(pa, id, sg)) { sg.kb = 0; sg.ke = pa.p[sg.prob].K / DBK; return true; }
    }
    return false;
}

template <int BM, int BN, int EPI>
struct Requester {
    Walk w;
    Seg sg;
    Stream<BM, BN> st;
    int kt, kend, phase;
    bool live;
    uint32_t issued;
};

template <int BM, int BN, int EPI>
__device__ __forceinline__ void requester_open(Requester<BM, BN, EPI>& q, const PArgs& pa, int wave, int lane) {
    const PProb& P = pa.p[q.sg.prob];
    if (q.phase == 0) {
        stream_setup<BM, BN>(q.st, P.A, P.lda, P.B, P.N, P.K, pa.M, q.sg.m0, q.sg.n0, wave, lane);
        q.kt = q.sg.kb; q.kend = q.sg.ke;
    } else {
        stream_setup<BM, BN>(q.st, P.A2, P.lda2, P.B2, P.N, P.K2, pa.M, q.sg.m0, q.sg.n0, wave, lane);
        q.kt = 0; q.kend = P.K2 / DBK;
    }
}

// the requests of the next step, not yet issued
template <int BM, int BN, int EPI>
__device__ __forceinline__ StepIssue<BM, BN> requester_next(const Requester<BM, BN, EPI>& q, uint32_t lds0, int wave) {
    return stream_step<BM, BN>(q.st, q.kt, lds0 + (q.issued & (DSTAGES - 1)) * dma_stage_bytes<BM, BN>(), wave, q.live);
}
// ... and the bookkeeping once they have been issued
template <int BM, int BN, int EPI>
__device__ __forceinline__ void requester_advance(Requester<BM, BN, EPI>& q, const PArgs& pa, int wave, int lane) {
    if (!q.live) return;
    ++q.issued;
    if (++q.kt == q.kend) {
        if (EPI == PEPI_GATEUP && q.phase == 0) { q.phase = 1; }
        else { q.phase = 0; q.live = walk_next<BM, BN>(q.w, pa, q.sg); }
        if (q.live) requester_open<BM, BN, EPI>(q, pa, wave, lane);
    }
}

// wait until at most `groups` request groups of this wave (L instructions each) are still in flight;
// requests complete in order, so the older groups have landed then -- whatever stores are also pending
template <int L>
__device__ __forceinline__ void wait_groups(int groups) {
    if (groups >= 2) wait_vm_lgkm0<2 * L>();
    else if (groups == 1) wait_vm_lgkm0<L>();
    else wait_vm_lgkm0<0>();
}

// one k-step of the persistent loop on accumulator set `acc`.  ZERO: first step of a tile.  LAST: last
// step of a tile -- the fragments of the following step are not read ahead, so that nothing but the
// accumulators has to survive the epilogue.
template <int BM, int BN, int EPI, bool ZERO, bool LAST>
__device__ __forceinline__ void persist_step(f32x16_t (&acc)[BM / 64][BN / 64], bf16x8_t (&af0)[BM / 64], bf16x8_t (&bf0)[BN / 64],
                                             bf16x8_t (&af1)[BM / 64], bf16x8_t (&bf1)[BN / 64], const char* ring, const FragAddr<BM, BN>& f,
                                             Requester<BM, BN, EPI>& q, const PArgs& pa, uint32_t lds0, uint32_t& done, int wave, int lane) {
    constexpr int L = BM / 64 + BN / 64;
    constexpr int SB = dma_stage_bytes<BM, BN>();
    const char* cur = ring + (done & (DSTAGES - 1)) * SB;
    const char* nxt = ring + ((done + 1) & (DSTAGES - 1)) * SB;
    dma_substep<BM, BN, ZERO, true, NoIssue>(acc, af0, bf0, af1, bf1, cur, f, 1, NoIssue());
    wait_groups<L>((int)(q.issued - done) - 2);       // group done+1 has landed (own part), own reads of this stage are done
    __builtin_amdgcn_s_barrier();
    // the next requests go into the stage just read by everyone.  (Spreading them between the MFMAs of
    // the second substep instead of issuing them together was measured: no gain for 256 x 256 tiles,
    // a loss for 128 x 128.)
    issue_all<BM, BN, 0>(requester_next<BM, BN, EPI>(q, lds0, wave));
    requester_advance<BM, BN, EPI>(q, pa, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    dma_substep<BM, BN, false, !LAST, NoIssue>(acc, af1, bf1, af0, bf0, nxt, f, 0, NoIssue());
    ++done;
}

// fragments of substep 0 of the stage at `stage` (which has landed and is barrier-visible)
template <int BM, int BN>
__device__ __forceinline__ void read_first_frags(bf16x8_t (&af)[BM / 64], bf16x8_t (&bf)[BN / 64], const char* stage, const FragAddr<BM, BN>& f) {
    constexpr int MI = BM / 64;
    dma_read_chunk<BM, BN, 0>(af, bf, stage, f, 0);
    if constexpr (MI > 1) dma_read_chunk<BM, BN, 1>(af, bf, stage, f, 0);
    if constexpr (MI > 2) dma_read_chunk<BM, BN, 2>(af, bf, stage, f, 0);
    if constexpr (MI > 3) dma_read_chunk<BM, BN, 3>(af, bf, stage, f, 0);
    __builtin_amdgcn_sched_barrier(0);
}

// One accumulator element, read from where the MFMA left it.  Written as an explicit accvgpr read so
// that the register allocator keeps the whole tile in the accumulator file until the moment of use
// (left alone it moves every remaining element into vector registers at once and spills the rest).
// The caller guarantees the MFMA -> read distance (s_nop after the last MFMA).
__device__ __forceinline__ float acc_elem(float a) {
    float r;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(a));
    return r;
}

// 8-byte accesses that are coherent across the whole device (they go past this XCD's L2): for the
// partial sums and flags that workgroups of one launch hand to each other.
__device__ __forceinline__ uint2 ld_dev_b64(const void* p) {
    const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void st_dev_b64(void* p, float lo, float hi) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), (uint64_t)__float_as_uint(lo) | ((uint64_t)__float_as_uint(hi) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Slot layout of a partial tile: float4 index ((wave * MI * NI + mi * NI + ni) * 4 + vg) * 64 + lane holds
// accumulator elements 4 vg .. 4 vg + 3 of block (mi, ni) -- every store instruction of a wave covers
// 1 KB of consecutive memory, and the reader is the same lane of the same wave of another workgroup.
template <int BM, int BN>
__device__ __forceinline__ size_t part_index(int wave, int mi, int ni, int vg, int lane) {
    constexpr int MI = BM / 64, NI = BN / 64;
    return ((size_t)((wave * MI * NI + mi * NI + ni) * 4 + vg) * 64 + lane) * 4;
}

template <int BM, int BN>
__device__ __forceinline__ void store_partial(const f32x16_t (&acc)[BM / 64][BN / 64], float* slot, int wave, int lane) {
    constexpr int MI = BM / 64, NI = BN / 64;
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(lane));    // MFMA -> accumulator read distance
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                float* d = slot + part_index<BM, BN>(wave, mi, ni, vg, lane);
                st_dev_b64(d, acc_elem(acc[mi][ni][4 * vg + 0]), acc_elem(acc[mi][ni][4 * vg + 1]));
                st_dev_b64(d + 2, acc_elem(acc[mi][ni][4 * vg + 2]), acc_elem(acc[mi][ni][4 * vg + 3]));
            }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Bounded wait for a flag another workgroup of this launch sets; on giving up the error word of the
// workspace is set (lowrank_workspace_status reports it) and the caller writes NaN into the tile it could not finish.
__device__ __forceinline__ bool sk_wait_flag(const uint32_t* flag, uint32_t* err, uint32_t limit) {
    uint32_t spins = 0;
    while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        if (++spins > limit) { __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); return false; }
        __builtin_amdgcn_s_sleep(2);
    }
    return true;
}

// Dense-cache rows.  A span of consecutive token rows that touches at most two sequences is described by
// four wave-uniform numbers, found once (one division, two position loads through the scalar path); the
// cache row of any token row m of the span then costs a compare and an add.
struct CacheSpan {
    int edge;          // first token row of the second sequence
    int bi0;           // batch index of the first sequence
    int p0, p1;        // position of the first new token of either sequence
};
__device__ __forceinline__ CacheSpan cache_span(const int32_t* pos, int T, int M, int r0) {
    CacheSpan cs;
    const int rc = r0 < M ? r0 : M - 1;
    cs.bi0 = __builtin_amdgcn_readfirstlane(rc / T);
    const int bl = (M - 1) / T;
    const int bi1 = cs.bi0 + 1 < bl ? cs.bi0 + 1 : bl;
    cs.p0 = pos[cs.bi0]; cs.p1 = pos[bi1];
    cs.edge = (cs.bi0 + 1) * T;
    return cs;
}
// batch * S_max + position of token row m (inside the span), or -1 when the row does not exist or falls outside the cache
__device__ __forceinline__ int cache_row(const CacheSpan& cs, int T, int S_max, int M, int m) {
    const bool second = m >= cs.edge;
    const int bi = second ? cs.bi0 + 1 : cs.bi0;
    const int64_t pp = (int64_t)(second ? cs.p1 : cs.p0) + (m - bi * T);
    return (m < M && pp >= 0 && pp < S_max) ? bi * S_max + (int)pp : -1;
}
// The 4 rows this lane stores for one block of 32 tile rows starting at row r0 (uniform) when sequences are
// shorter than a wave's strip of rows: a block of 32 rows still touches at most two sequences from 32 tokens
// per sequence on; below that every lane looks its rows up by itself.
__device__ __forceinline__ void cache_rows(int (&crow)[4], const int32_t* pos, int T, int S_max, int M, int r0, int rrow) {
    if (T >= 32) {
        const CacheSpan cs = cache_span(pos, T, M, r0);
#pragma unroll
        for (int it = 0; it < 4; ++it) crow[it] = cache_row(cs, T, S_max, M, r0 + it * 8 + rrow);
    } else {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int m = r0 + it * 8 + rrow;
            const int mc = m < M ? m : M - 1;
            const int bi = mc / T;
            const int64_t pp = (int64_t)pos[bi] + (mc - bi * T);
            crow[it] = (m < M && pp >= 0 && pp < S_max) ? bi * S_max + (int)pp : -1;
        }
    }
}

template <int BM, int BN, int EPI, bool SK = false>
__device__ __forceinline__ void wave_epilogue(const f32x16_t (&acc)[BM / 64][BN / 64],
                                              const f32x16_t (&acc2)[(EPI == PEPI_GATEUP) ? BM / 64 : 1][(EPI == PEPI_GATEUP) ? BN / 64 : 1],
                                              const PProb& P, int M, int m0, int n0, char* patch, int wave, int lane,
                                              const float* parts = nullptr, int part0 = 0, int part1 = 0, float poison = 0.f) {
    // parts: partial tiles of slots [part0, part1) are added (shared-K owner), skipping empty ones
    constexpr int MI = BM / 64, NI = BN / 64;
    if constexpr (EPI == PEPI_PARTIAL) {
        // fp32 partial sums of one K chunk, straight from the accumulators: lane (li, lg) holds, for tile row 32 mi + li of
        // its wave's quarter, columns 32 ni + 8 vg + 4 lg .. + 3
        asm volatile("s_nop 15\n\ts_nop 15" : "+v"(lane));
        const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lg = lane >> 5;
        float* const Cf = P.Cf;
        const int ldc = P.ldc, N = P.N;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = m0 + wm * (BM / 2) + mi * 32 + li;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int col = n0 + wn * (BN / 2) + ni * 32 + 8 * vg + 4 * lg;
                    const float4 o = make_float4(acc_elem(acc[mi][ni][4 * vg + 0]), acc_elem(acc[mi][ni][4 * vg + 1]),
                                                 acc_elem(acc[mi][ni][4 * vg + 2]), acc_elem(acc[mi][ni][4 * vg + 3]));
                    if (row < M && col < N) *reinterpret_cast<float4*>(Cf + (size_t)row * ldc + col) = o;
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
    // the lane index goes through an opaque move: everything derived from it is recomputed here, per
    // tile, instead of being hoisted out of the tile loop and held (or spilled) across the main loop
    // ... and the matrix pipeline gets the distance it needs before its results are read (32 wait states)
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(lane));
    const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lg = lane >> 5;
    const int rrow = lane >> 3, runit = lane & 7;                 // this lane's row (of 8) and unit when rows are read back
    // the fields of this tile's problem, fetched once
    bf16_t* const C = P.C; const int ldc = P.ldc, N = P.N;
    const bf16_t* const bias = P.bias; const bf16_t* const bias2 = P.bias2;
    bf16_t* const cache = (EPI == PEPI_STORE) ? reinterpret_cast<bf16_t*>(P.cache) : nullptr;
    const int32_t* const pos = P.pos; const int S_max = P.S_max, T = P.T;
    char* const wr = patch + li * 128 + lg * 8;                   // this lane's row of the patch when written
    const int wsw = (li >> 1) & 7;
    // cache rows of the wave's strip of BM / 2 tile rows: one look-up per tile when the strip touches at most two sequences
    const bool strip_span = EPI == PEPI_STORE && cache != nullptr && T >= BM / 2;
    CacheSpan span = {0, 0, 0, 0};
    if constexpr (EPI == PEPI_STORE) { if (strip_span) span = cache_span(pos, T, M, m0 + wm * (BM / 2)); }
#pragma unroll
    for (int pr = 0; pr < (NI + 1) / 2; ++pr) {                   // pairs of 32-column blocks; the last one may be single
        const int np2 = (2 * pr + 1 < NI) ? 2 : 1;                // column blocks in this pair
        uint2 bgp[2][4], bup[2][4];                               // bias of this lane's columns, bf16 pairs as loaded
#pragma unroll
        for (int p2 = 0; p2 < 2; ++p2)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) { bgp[p2][vg] = make_uint2(0u, 0u); bup[p2][vg] = make_uint2(0u, 0u); }
        if (bias || (EPI == PEPI_GATEUP && bias2)) {
#pragma unroll
            for (int p2 = 0; p2 < 2; ++p2)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    int gcol = n0 + wn * (BN / 2) + (pr * 2 + p2) * 32 + 8 * vg + 4 * lg;
                    gcol = gcol < N ? gcol : N - 4;                // clamped columns are never stored
                    if (bias) bgp[p2][vg] = *reinterpret_cast<const uint2*>(bias + gcol);
                    if constexpr (EPI == PEPI_GATEUP) { if (bias2) bup[p2][vg] = *reinterpret_cast<const uint2*>(bias2 + gcol); }
                }
        }
        const int gcol = n0 + wn * (BN / 2) + pr * 64 + runit * 8;   // first of the 8 columns this lane stores
        const bool col_ok = gcol < N && runit < 4 * np2;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int r0 = m0 + wm * (BM / 2) + mi * 32;
            int crow[4] = {-1, -1, -1, -1};
            if constexpr (EPI == PEPI_STORE) {
                if (strip_span) {
#pragma unroll
                    for (int it = 0; it < 4; ++it) crow[it] = cache_row(span, T, S_max, M, r0 + it * 8 + rrow);
                } else if (cache) {
                    cache_rows(crow, pos, T, S_max, M, r0, rrow);
                }
            }
            // shared-K holder: the other workgroups' partial sums of this block, three slots per round trip
            float psum[2][4][4];
#pragma unroll
            for (int p2 = 0; p2 < 2; ++p2)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg)
#pragma unroll
                    for (int e = 0; e < 4; ++e) psum[p2][vg][e] = poison;      // NaN when a partial sum never arrived
            if constexpr (SK) {
                for (int c = part0; c < part1; c += 3) {
                    uint2 raw[3][2][4][2];
#pragma unroll
                    for (int cc = 0; cc < 3; ++cc) {
                        const int cs = c + cc < part1 ? c + cc : part1 - 1;      // a repeated slot is loaded but not added
#pragma unroll
                        for (int p2 = 0; p2 < np2; ++p2)
#pragma unroll
                            for (int vg = 0; vg < 4; ++vg) {
                                const float* src = parts + (size_t)cs * (BM * BN) + part_index<BM, BN>(wave, mi, pr * 2 + p2, vg, lane);
                                raw[cc][p2][vg][0] = ld_dev_b64(src); raw[cc][p2][vg][1] = ld_dev_b64(src + 2);
                            }
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int cc = 0; cc < 3; ++cc) {
                        const float w = c + cc < part1 ? 1.f : 0.f;
#pragma unroll
                        for (int p2 = 0; p2 < np2; ++p2)
#pragma unroll
                            for (int vg = 0; vg < 4; ++vg) {
                                psum[p2][vg][0] += w * __uint_as_float(raw[cc][p2][vg][0].x); psum[p2][vg][1] += w * __uint_as_float(raw[cc][p2][vg][0].y);
                                psum[p2][vg][2] += w * __uint_as_float(raw[cc][p2][vg][1].x); psum[p2][vg][3] += w * __uint_as_float(raw[cc][p2][vg][1].y);
                            }
                    }
                }
            }
#pragma unroll
            for (int p2 = 0; p2 < np2; ++p2)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    const int ni = pr * 2 + p2;
                    const uint2 rg = bgp[p2][vg], ru = bup[p2][vg];
                    const float bg[4] = {__uint_as_float(rg.x << 16), __uint_as_float(rg.x & 0xffff0000u),
                                         __uint_as_float(rg.y << 16), __uint_as_float(rg.y & 0xffff0000u)};
                    const float bu[4] = {__uint_as_float(ru.x << 16), __uint_as_float(ru.x & 0xffff0000u),
                                         __uint_as_float(ru.y << 16), __uint_as_float(ru.y & 0xffff0000u)};
                    const float* ps = psum[p2][vg];
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if constexpr (EPI == PEPI_GATEUP)
                            v[e] = silu_bf16out(acc_elem(acc[mi][ni][4 * vg + e]) + bg[e]) * (acc_elem(acc2[mi][ni][4 * vg + e]) + bu[e]);
                        else
                            v[e] = (acc_elem(acc[mi][ni][4 * vg + e]) + ps[e]) + bg[e];
                    }
                    uint2 o; o.x = ppack2(v[0], v[1]); o.y = ppack2(v[2], v[3]);
                    *reinterpret_cast<uint2*>(wr + (((p2 * 4 + vg) ^ wsw) * 16)) = o;
                }
#pragma unroll
            for (int h = 0; h < 2; ++h) {               // two rows in flight at a time: enough to cover the LDS latency
                uint4 val[2];
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) {
                    const int row = (2 * h + i2) * 8 + rrow;
                    val[i2] = *reinterpret_cast<const uint4*>(patch + row * 128 + ((runit ^ ((row >> 1) & 7)) * 16));
                }
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2) {
                    const int it = 2 * h + i2;
                    const int m = r0 + it * 8 + rrow;
                    if (C && col_ok && m < M) *reinterpret_cast<uint4*>(C + (size_t)m * ldc + gcol) = val[i2];
                    if constexpr (EPI == PEPI_STORE) {
                        if (col_ok && crow[it] >= 0) *reinterpret_cast<uint4*>(cache + (size_t)crow[it] * N + gcol) = val[i2];
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);      // keep the accumulator reads of later blocks from piling up in registers
        }
    }
}

template <int BM, int BN, int EPI, int MINB, bool SK>
__global__ void __launch_bounds__(256, MINB) k_prefill_persist(PArgs pa) {
    constexpr int MI = BM / 64, NI = BN / 64;
    constexpr int L = MI + NI;
    __shared__ uint4 lds[persist_lds_bytes<BM, BN>() / 16];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const char* ring = reinterpret_cast<const char*>(lds);
    char* patch = reinterpret_cast<char*>(lds) + DSTAGES * dma_stage_bytes<BM, BN>() + wave * 4096;
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)lds);

    FragAddr<BM, BN> f;
    frag_setup<BM, BN>(f);

    Requester<BM, BN, EPI> q;
    q.w = walk_begin(pa); q.issued = 0; q.phase = 0; q.kt = 0; q.kend = 0;
    q.live = walk_next<BM, BN>(q.w, pa, q.sg);
    if (!q.live) return;                                    // no work for this workgroup (whole workgroup leaves)
    requester_open<BM, BN, EPI>(q, pa, wave, lane);
    for (int i = 0; i < DSTAGES; ++i) {
        issue_all<BM, BN, 0>(requester_next<BM, BN, EPI>(q, lds0, wave));
        requester_advance<BM, BN, EPI>(q, pa, wave, lane);
    }

    Walk cw = walk_begin(pa);
    Seg sg;
    uint32_t done = 0;
    wait_groups<L>((int)q.issued - 1);                      // group 0 has landed
    __builtin_amdgcn_s_barrier();
    bf16x8_t af0[MI], bf0[NI], af1[MI], bf1[NI];

    while (walk_next<BM, BN>(cw, pa, sg)) {
        const PProb& P = pa.p[sg.prob];
        f32x16_t acc[MI][NI];
        f32x16_t acc2[(EPI == PEPI_GATEUP) ? MI : 1][(EPI == PEPI_GATEUP) ? NI : 1];
        const int steps = sg.ke - sg.kb;           // >= 1; whole tiles have >= 2
        read_first_frags<BM, BN>(af0, bf0, ring + (done & (DSTAGES - 1)) * dma_stage_bytes<BM, BN>(), f);
        if (EPI == PEPI_STORE && steps == 1) {
            persist_step<BM, BN, EPI, true, true>(acc, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
        } else {
            persist_step<BM, BN, EPI, true, false>(acc, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
            for (int kt = 2; kt < steps; ++kt)
                persist_step<BM, BN, EPI, false, false>(acc, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
            if constexpr (EPI == PEPI_GATEUP) {
                const int nk2 = P.K2 / DBK;
                persist_step<BM, BN, EPI, false, false>(acc, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
                persist_step<BM, BN, EPI, true, false>(acc2, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
                for (int kt = 2; kt < nk2; ++kt)
                    persist_step<BM, BN, EPI, false, false>(acc2, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
                persist_step<BM, BN, EPI, false, true>(acc2, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
            } else {
                persist_step<BM, BN, EPI, false, true>(acc, af0, bf0, af1, bf1, ring, f, q, pa, lds0, done, wave, lane);
            }
        }
        if constexpr (SK) {
            if (!(sg.kb == 0 && sg.ke == pa.sk_nk)) {
                const int wl = logical_wg();
                if (sg.kb > 0) {
                    // not the holder of this tile's first k-step: hand the partial sums over
                    store_partial<BM, BN>(acc, pa.sk_slots + (size_t)wl * (BM * BN), wave, lane);
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this wave's part has been written
                    __builtin_amdgcn_s_barrier();
                    if (tid == 0) __hip_atomic_store(pa.sk_flags + wl, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    // holder of k = 0 (its last segment): the rest of the tile's k range lies with the
                    // following logical workgroups, which did that part first
                    const int tile_end = (cw.next / pa.sk_nk + 1) * pa.sk_nk;   // cw.next == end of this range, inside the tile
                    int c1 = wl + 1;
                    while (c1 < (int)gridDim.x && sk_unit_begin(pa, c1) < tile_end) ++c1;
                    uint32_t* gave_up = reinterpret_cast<uint32_t*>(lds) + (persist_lds_bytes<BM, BN>() / 4 - 1);   // last word of wave 3's patch: free here
                    if (tid == 0) {
                        bool ok = true;
                        for (int c = wl + 1; c < c1; ++c)
                            if (sk_unit_begin(pa, c + 1) > sk_unit_begin(pa, c)) ok = sk_wait_flag(pa.sk_flags + c, pa.err, pa.sk_spin_limit) && ok;
                        *gave_up = ok ? 0u : 1u;
                    }
                    __builtin_amdgcn_s_barrier();
                    const float poison = *gave_up ? __uint_as_float(0x7fc00000u) : 0.f;
                    __builtin_amdgcn_s_barrier();                 // everyone has read the word before wave 3 reuses its patch
                    // (the launcher sizes the grid so that no range is empty: every slot in [wl + 1, c1) is fresh)
                    wave_epilogue<BM, BN, EPI, true>(acc, acc2, P, pa.M, sg.m0, sg.n0, patch, wave, lane, pa.sk_slots, wl + 1, c1, poison);
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // partial sums have been read
                    __builtin_amdgcn_s_barrier();
                    if (tid == 0)
                        for (int c = wl + 1; c < c1; ++c) __hip_atomic_store(pa.sk_flags + c, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                continue;
            }
        }
        wave_epilogue<BM, BN, EPI>(acc, acc2, P, pa.M, sg.m0, sg.n0, patch, wave, lane);
    }
}

// Fast-path rule: K in 64-row steps, N in 128-column tiles, any M >= 1.
bool prefill_shape_ok(int64_t M, int64_t K, int64_t N) {
    return M >= 1 && M < (1 << 30) && K >= 64 && (K % 64) == 0 && N >= 128 && (N % 128) == 0 &&
           K < (1 << 24) && N < (1 << 24);
}

// all problems of one launch have the same K and N (then every tile of the launch grid is a real one)
static bool one_shape(const PArgs& a) {
    for (int i = 1; i < a.nprob; ++i)
        if (a.p[i].K != a.p[0].K || a.p[i].N != a.p[0].N) return false;
    return true;
}

template <int BM, int BN, int EPI, int MINB>
static int launch_persist(PArgs a, hipStream_t s, bool share_k = false) {
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n_max = 0;
    for (int i = 0; i < a.nprob; ++i) { const int t = (a.p[i].N + BN - 1) / BN; if (t > a.tiles_n_max) a.tiles_n_max = t; }
    const int total = a.tiles_m * a.tiles_n_max * a.nprob;
    // row tiles per group of the tile walk (a group's tiles are visited row-fastest): 8, and 2 for the gate/up kernel,
    // whose tiles carry two B operands (measured 393 -> 373 us on the benchmark's layer)
    a.group_m = EPI == PEPI_GATEUP ? 2 : 8;
    a.sk_spin_limit = g_wait_limit < (1u << 20) ? g_wait_limit : (1u << 22);     // these polls sleep longer than the decode ones
    a.trace = g_trace_buffer;
    a.sk = 0; a.sk_nk = 0;
    int grid = 0;
    if (share_k && EPI == PEPI_STORE && BM == 256 && (BN == 256 || BN == 192) && a.sk_slots && one_shape(a)) {
        // shared-K walk: equal k-step ranges, at least 8 steps each, one workgroup per slot of the chip
        a.sk = 1; a.sk_nk = a.p[0].K / 32;
        const long long units = (long long)total * a.sk_nk;
        long long g = units / 8 < 256 * MINB ? units / 8 : 256 * MINB;
        g &= ~7ll;
        if (g < 8) { a.sk = 0; }
        grid = (int)g;
        // More rows than columns: the A operand is the big one.  Column tiles of one row block then follow each other in
        // the walk, so that the workgroups that hold them (neighbours on one XCD) read the same rows of A at the same time
        // and share them in that L2; otherwise row tiles of one column block do (they share B).
        if (a.sk && a.M > a.p[0].N) a.group_m = 1;
    }
    if (!a.sk) {
        const int per_xcd = (total + 7) / 8;
        const int slots = per_xcd < 32 * MINB ? per_xcd : 32 * MINB;      // workgroups per XCD
        grid = 8 * slots;
    }
    if constexpr (EPI == PEPI_STORE && BM == 256 && (BN == 256 || BN == 192)) {
        if (a.sk) {
            // the only prefill launch that keeps state in the workspace (flags, error word): make sure the control block is valid
            if (int pst = ws_prepare(reinterpret_cast<char*>(a.sk_flags) - kHeaderBytes, s); pst != LR_OK) return pst;
            hipLaunchKernelGGL((k_prefill_persist<BM, BN, EPI, MINB, true>), dim3((unsigned)grid), dim3(256), 0, s, a);
            return launch_status("prefill gemm");
        }
    }
    hipLaunchKernelGGL((k_prefill_persist<BM, BN, EPI, MINB, false>), dim3((unsigned)grid), dim3(256), 0, s, a);
    return launch_status("prefill gemm");
}

// Tile shape of a plain launch, from a small cost model fitted to measurements on this chip, in units of "one
// 256 x 256 tile on one CU": the 256-row kernels (one workgroup per CU) take one unit per round for 256
// columns and 0.75 for 192; the 128 x 128 kernel needs 0.46 for its quarter-size tile when every tile has a CU
// to itself, and 0.64 per round of two tiles per CU otherwise.  Big-N products with short K (the
// reconstruction x V) go to 256 x 256; the rank-space products (N = 384, 1536: multiples of 192 but poor
// fits for 256) to 256 x 192, which wastes no matrix work on columns past N; small ones to 128 x 128.
static int pick_tile(const PArgs& a) {
    long t256 = 0, t192 = 0, t128 = 0;
    for (int i = 0; i < a.nprob; ++i) {
        t256 += (long)((a.M + 255) / 256) * ((a.p[i].N + 255) / 256);
        t192 += (long)((a.M + 255) / 256) * ((a.p[i].N + 191) / 192);
        t128 += (long)((a.M + 127) / 128) * ((a.p[i].N + 127) / 128);
    }
    const double c256 = (double)((t256 + 255) / 256);
    const double c192 = 0.75 * (double)((t192 + 255) / 256);
    const double c128 = t128 <= 256 ? 0.46 : 0.64 * (double)((t128 + 511) / 512);
    if (c192 < c256 && c192 < c128) return 192;
    return c256 <= c128 ? 256 : 128;
}

// A product with a very long K and so few 256 x 256 tiles that half the CUs would get none (h U_d of
// the MLP) shares its K range between workgroups instead: every CU gets the same number of k-steps.
// Measured on this chip (M = 8192): 8192 x 11008 x 768 takes 236 us as 128 x 128 tiles and about 175 us
// shared; with K = 4096 the hand-over of partial tiles and the lost L2 reuse (workgroups of one XCD
// are no longer at the same k) cost more than the better balance brings, so those stay tiled.
static bool want_share_k(const PArgs& a) {
    if (!a.sk_slots || !one_shape(a) || g_device_shared) return false;     // the hand-over needs all workgroups resident
    const long t256 = (long)a.nprob * ((a.M + 255) / 256) * ((a.p[0].N + 255) / 256);
    const long nk = a.p[0].K / 32;
    return t256 <= 128 && t256 * nk / 256 >= 96;
}

// The tile the dispatcher would pick for `n` products C[M, N] = A[M, K] * B[K, N] launched together (plain
// epilogue), and whether they would share K between workgroups.  Pure host logic (no device needed).
static int split_k_chunks(const PArgs& a);
void prefill_plan_query(int64_t M, int64_t K, int64_t N, int n, bool gateup, int* bm, int* bn, int* share_k) {
    PArgs a;
    memset(&a, 0, sizeof(a));
    a.M = (int)M; a.nprob = n < 1 ? 1 : (n > kMaxPProb ? kMaxPProb : n);
    for (int i = 0; i < a.nprob; ++i) { a.p[i].K = (int)K; a.p[i].N = (int)N; a.p[i].C = reinterpret_cast<bf16_t*>(sizeof(float)); }
    a.sk_slots = reinterpret_cast<float*>(sizeof(float));      // "a shared-K area exists"; never dereferenced here
    *share_k = 0;
    if (gateup) { *bm = 128; *bn = 128; return; }
    if (const int split = split_k_chunks(a); split >= 2) { *share_k = split; *bm = 128; *bn = 128; return; }
    if (want_share_k(a)) { *share_k = 1; *bm = 256; *bn = (N % 192 == 0) ? 192 : 256; return; }
    const int t = pick_tile(a);
    *bm = t == 128 ? 128 : 256; *bn = t;
}

// One launch adds the partial matrices of every product of a split-K launch: blockIdx.y is the product,
// C[m, n] = sum over `split` partial matrices (fp32, `stride` floats apart) in chunk order, rounded to bf16 once.
struct RProb {
    const float* part;
    bf16_t* C;
    size_t stride;
    int ldc, N, split;
};
struct RArgs {
    int M;
    RProb p[kMaxPProb / 2];
};

__global__ void __launch_bounds__(256) k_prefill_reduce(const RArgs a) {
    const RProb& r = a.p[blockIdx.y];
    const int N = r.N, split = r.split;
    const size_t total = (size_t)a.M * (size_t)(N / 4);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t m = i / (size_t)(N / 4);
        const int n = 4 * (int)(i - m * (size_t)(N / 4));
        const float* src = r.part + m * (size_t)N + n;
        float4 acc = *reinterpret_cast<const float4*>(src);
        for (int sp = 1; sp < split; ++sp) {
            const float4 v = *reinterpret_cast<const float4*>(src + (size_t)sp * r.stride);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<uint2*>(r.C + m * (size_t)r.ldc + n) = make_uint2(ppack2(acc.x, acc.y), ppack2(acc.z, acc.w));
    }
}

// Few rows and a long K (a rank-space product x U or h U_d of a prompt of some hundred tokens: 24..192 tiles of 128 x 128
// for 512 workgroup slots, each with hundreds of k-steps): the K range is cut into `split` chunks that run as separate
// products of ONE launch and leave fp32 partial sums in the workspace tail (the area of the shared-K partial tiles, unused by
// such a launch); a small second launch adds them in chunk order (deterministic) and rounds once.  Returns how many chunks
// would be used (0 or 1: not worth it or not possible).
static int split_k_chunks(const PArgs& a) {
    if (!a.sk_slots || a.nprob < 1) return 0;
    long t128 = 0, n_sum = 0;
    for (int i = 0; i < a.nprob; ++i) {
        const PProb& p = a.p[i];
        if (p.bias || p.cache || !p.C || p.K != a.p[0].K || (p.N & 3)) return 0;
        t128 += (long)((a.M + 127) / 128) * ((p.N + 127) / 128);
        n_sum += p.N;
    }
    if (t128 > 192) return 0;                                   // enough tiles to fill the chip as they are
    long split = 512 / t128;
    const long by_k = a.p[0].K / 512, by_prob = kMaxPProb / a.nprob;
    const long by_mem = (long)(kSkSlotBytes / ((size_t)a.M * (size_t)n_sum * 4));
    if (by_k < split) split = by_k;
    if (by_prob < split) split = by_prob;
    if (by_mem < split) split = by_mem;
    if (split > 8) split = 8;
    return split >= 2 ? (int)split : 0;
}

static int launch_split_k(const PArgs& a, int split, hipStream_t s) {
    const int K = a.p[0].K;
    const int chunk = ((K / 64 + split - 1) / split) * 64;
    PArgs b = a;
    b.nprob = 0;
    size_t off[kMaxPProb];
    int used[kMaxPProb];
    size_t o = 0;
    for (int i = 0; i < a.nprob; ++i) { off[i] = o; o += (size_t)split * (size_t)a.M * (size_t)a.p[i].N; used[i] = 0; }
    for (int sp = 0; sp < split; ++sp)
        for (int i = 0; i < a.nprob; ++i) {
            const int k0 = sp * chunk, kc = K - k0 < chunk ? K - k0 : chunk;
            if (kc <= 0) continue;
            PProb& p = b.p[b.nprob++];
            p = a.p[i];
            p.A = a.p[i].A + k0; p.B = a.p[i].B + (size_t)k0 * (size_t)a.p[i].N; p.K = kc;
            p.C = nullptr; p.Cf = a.sk_slots + off[i] + (size_t)sp * (size_t)a.M * (size_t)a.p[i].N; p.ldc = a.p[i].N;
            used[i] = sp + 1;
        }
    int st = launch_persist<128, 128, PEPI_PARTIAL, 2>(b, s, false);
    if (st != LR_OK) return st;
    RArgs r;
    r.M = a.M;
    size_t blocks = 1;
    for (int i = 0; i < a.nprob; ++i) {
        r.p[i].part = a.sk_slots + off[i]; r.p[i].C = a.p[i].C; r.p[i].stride = (size_t)a.M * (size_t)a.p[i].N;
        r.p[i].ldc = a.p[i].ldc; r.p[i].N = a.p[i].N; r.p[i].split = used[i];
        const size_t b = ((size_t)a.M * (size_t)(a.p[i].N / 4) + 255) / 256;
        if (b > blocks) blocks = b;
    }
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_prefill_reduce, dim3((unsigned)blocks, (unsigned)a.nprob), dim3(256), 0, s, r);
    return launch_status("prefill split-K reduction");
}

int prefill_launch(const PArgs& a, int epi, hipStream_t s) {
    if (a.M <= 0 || a.nprob <= 0) return LR_OK;
    if (epi == PEPI_STORE) {
        const int split = split_k_chunks(a);
        if (split >= 2) return launch_split_k(a, split, s);
    }
    if (epi == PEPI_GATEUP) return launch_persist<128, 128, PEPI_GATEUP, 2>(a, s);
    if (want_share_k(a)) {
        // 192-wide tiles when they cover the columns exactly: more, aligned pieces of the K range per row block
        // (N = 768: four column tiles x two halves of K = eight workgroups per row block, all on one XCD)
        if (a.p[0].N % 192 == 0) return launch_persist<256, 192, PEPI_STORE, 1>(a, s, true);
        return launch_persist<256, 256, PEPI_STORE, 1>(a, s, true);
    }
    switch (pick_tile(a)) {
        case 192: return launch_persist<256, 192, PEPI_STORE, 1>(a, s);
        case 256: return launch_persist<256, 256, PEPI_STORE, 1>(a, s);
        default: return launch_persist<128, 128, PEPI_STORE, 2>(a, s);
    }
}

}  // namespace lr
