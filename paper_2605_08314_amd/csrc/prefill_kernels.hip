// Prefill-phase GEMM (bf16 MFMA, LDS-staged): C[M, N] = A[M, K] * B[K, N] with A, B, C row-major.
//
// Tile: BM x 128 x 64 per workgroup of 4 waves (2 x 2), each wave (BM/2) x 64 built from
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

namespace lr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int PBN = 128, PBK = 64;

__host__ __device__ constexpr int plane_units(int rows) { return rows + rows / 8 + 1; }
__device__ __forceinline__ int unit_of(int plane, int chunk, int row) { return chunk * plane + row + (row >> 3); }

template <int BM> constexpr int main_units() { return 8 * plane_units(BM) + 8 * plane_units(PBN); }
template <int BM> constexpr int epi_units() { return BM * (PBN + 8) * 2 / 16; }
template <int BM> constexpr int lds_units() { return main_units<BM>() > epi_units<BM>() ? main_units<BM>() : epi_units<BM>(); }

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

// One K loop: acc[mi][ni] += (B tile)^T x (A tile)^T over k in [0, K).
template <int BM>
__device__ __forceinline__ void gemm_loop(f32x16_t (&acc)[BM / 64][2], const bf16_t* __restrict__ A, int lda,
                                          const bf16_t* __restrict__ B, int N, int K, int M, int m0, int n0, uint4* lds) {
    constexpr int MI = BM / 64;
    constexpr int NA = BM / 32;                 // 16-byte chunks of A per thread and k-step
    constexpr int PA = plane_units(BM), PB = plane_units(PBN);
    uint4* As = lds;
    uint4* Bs = lds + 8 * PA;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lg = lane >> 5;
    const int cg = tid & 15, rg = tid >> 4;     // B loader: column group (8 columns), row group (4 k-rows)

    uint4 ra[NA], rb[4];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            const int m = m0 + row;
            if (m < M) ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)m * lda + k0 + kc * 8);
            else ra[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        const bf16_t* bp = B + (size_t)(k0 + rg * 4) * N + n0 + cg * 8;
#pragma unroll
        for (int a = 0; a < 4; ++a) rb[a] = *reinterpret_cast<const uint4*>(bp + (size_t)a * N);
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kc = c & 7;
            As[unit_of(PA, kc, row)] = ra[i];
        }
        const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&rb[0]);
        const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&rb[1]);
        const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&rb[2]);
        const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&rb[3]);
        uint2* Bs2 = reinterpret_cast<uint2*>(Bs);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint32_t sel = (b & 1) ? 0x07060302u : 0x05040100u;
            uint2 v;
            v.x = __builtin_amdgcn_perm(r1[b >> 1], r0[b >> 1], sel);    // k rows 4rg+0, 4rg+1 of column b
            v.y = __builtin_amdgcn_perm(r3[b >> 1], r2[b >> 1], sel);    // k rows 4rg+2, 4rg+3
            Bs2[unit_of(PB, rg >> 1, cg * 8 + b) * 2 + (rg & 1)] = v;
        }
    };

    const int nk = K / PBK;
    load_tiles(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();                 // everyone finished reading the previous tile
        store_tiles();
        __syncthreads();
        if (kt + 1 < nk) load_tiles((kt + 1) * PBK);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8_t af[MI], bf[2];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) af[mi] = frag_of(As[unit_of(PA, 2 * kk + lg, wm * (BM / 2) + mi * 32 + li)]);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) bf[ni] = frag_of(Bs[unit_of(PB, 2 * kk + lg, wn * 64 + ni * 32 + li)]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ni], af[mi], acc[mi][ni], 0, 0, 0);
        }
    }
}

template <int BM, int EPI, int MINB>
__global__ void __launch_bounds__(256, MINB) k_prefill_gemm(PArgs pa) {
    constexpr int MI = BM / 64;
    __shared__ uint4 lds[lds_units<BM>()];
    // tile order: each XCD (workgroups are dealt round-robin to the 8 XCDs) walks a contiguous range
    // of tiles, n fastest, so the A rows of a tile row stay in that XCD's L2 while B streams past.
    const int per_prob = pa.tiles_m * pa.tiles_n_max;
    const int total = per_prob * pa.nprob;
    int id = blockIdx.x;
    {
        const int chunk = (total + 7) / 8;
        const int swz = (id & 7) * chunk + (id >> 3);
        if ((total & 7) == 0) id = swz;
    }
    const int prob = id / per_prob;
    const int rem = id - prob * per_prob;
    const int tm = rem / pa.tiles_n_max, tn = rem - tm * pa.tiles_n_max;
    const PProb& P = pa.p[prob];
    if (tn * PBN >= P.N) return;
    const int m0 = tm * BM, n0 = tn * PBN, M = pa.M;

    f32x16_t acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    gemm_loop<BM>(acc, P.A, P.lda, P.B, P.N, P.K, M, m0, n0, lds);

    f32x16_t acc2[(EPI == PEPI_GATEUP) ? MI : 1][2];
    if constexpr (EPI == PEPI_GATEUP) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[mi][ni][v] = 0.f;
        gemm_loop<BM>(acc2, P.A2, P.lda2, P.B2, P.N, P.K2, M, m0, n0, lds);
    }

    // ---- epilogue: registers -> bf16 staging tile in LDS -> coalesced 16-byte row stores
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lg = lane >> 5;
    constexpr int CS = PBN + 8;                       // staging row stride in bf16
    __syncthreads();                                  // main-loop LDS no longer needed
    bf16_t* Cs = reinterpret_cast<bf16_t*>(lds);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int row = wm * (BM / 2) + mi * 32 + li;                 // token row inside the tile
                const int col = wn * 64 + ni * 32 + 8 * vg + 4 * lg;          // first of 4 consecutive columns
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[mi][ni][4 * vg + e];
                if constexpr (EPI == PEPI_GATEUP) {
                    float bg[4] = {0.f, 0.f, 0.f, 0.f}, bu[4] = {0.f, 0.f, 0.f, 0.f};
                    if (P.bias) { for (int e = 0; e < 4; ++e) bg[e] = bf16_to_f32(P.bias[n0 + col + e]); }
                    if (P.bias2) { for (int e = 0; e < 4; ++e) bu[e] = bf16_to_f32(P.bias2[n0 + col + e]); }
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = silu_f32(v[e] + bg[e]) * (acc2[mi][ni][4 * vg + e] + bu[e]);
                } else {
                    if (P.bias) { for (int e = 0; e < 4; ++e) v[e] += bf16_to_f32(P.bias[n0 + col + e]); }
                }
                uint2 o; o.x = ppack2(v[0], v[1]); o.y = ppack2(v[2], v[3]);
                *reinterpret_cast<uint2*>(Cs + row * CS + col) = o;
            }
    __syncthreads();
    constexpr int CHUNKS = BM * (PBN / 8);            // 16-byte chunks in the tile
#pragma unroll 4
    for (int c = tid; c < CHUNKS; c += 256) {
        const int row = c >> 4, ch = c & 15;
        const int m = m0 + row;
        if (m >= M) continue;
        const uint4 val = *reinterpret_cast<const uint4*>(Cs + row * CS + ch * 8);
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

template <int BM, int EPI, int MINB>
static int launch_cfg(PArgs a, hipStream_t s) {
    a.tiles_m = (a.M + BM - 1) / BM;
    const int total = a.tiles_m * a.tiles_n_max * a.nprob;
    hipLaunchKernelGGL((k_prefill_gemm<BM, EPI, MINB>), dim3((unsigned)total), dim3(256), 0, s, a);
    return launch_status("prefill gemm");
}

// BM = 256 unless that leaves the 256 CUs visibly under-filled (few tiles) and 128 fills them better.
static int pick_bm(const PArgs& a, int force) {
    if (force == 128 || force == 256) return force;
    auto waste = [&](int bm) {
        const long tiles = (long)((a.M + bm - 1) / bm) * a.tiles_n_max * a.nprob;
        const long slots = 256L * (bm == 128 ? 2 : 2);    // resident tiles per round
        const long rounds = (tiles + slots - 1) / slots;
        return (double)(rounds * slots) / (double)tiles * (bm == 128 ? 1.15 : 1.0);   // 128-row tiles reuse B less
    };
    return waste(128) < waste(256) ? 128 : 256;
}

int prefill_launch(const PArgs& a, int epi, hipStream_t s) {
    if (a.M <= 0 || a.nprob <= 0) return LR_OK;
    static int force_bm = -1;
    if (force_bm < 0) { const char* v = getenv("LOWRANK_PREFILL_BM"); force_bm = v ? atoi(v) : 0; }
    if (epi == PEPI_GATEUP) {
        const int bm = (force_bm == 256) ? 256 : 128;
        if (bm == 256) return launch_cfg<256, PEPI_GATEUP, 1>(a, s);
        return launch_cfg<128, PEPI_GATEUP, 2>(a, s);
    }
    if (pick_bm(a, force_bm) == 128) return launch_cfg<128, PEPI_STORE, 2>(a, s);
    return launch_cfg<256, PEPI_STORE, 2>(a, s);
}

}  // namespace lr
