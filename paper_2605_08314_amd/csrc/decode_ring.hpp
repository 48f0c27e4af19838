// Decode phase, up to 16 token rows: descriptors of the streaming kernel whose factor bytes travel
// global memory -> LDS ring -> matrix cores, requested far ahead of the stage they belong to.
//
// A call is a chain of stages separated by device-wide barriers (t += x U | y = t V ..., four for the
// packed MLP).  The factor bytes do not depend on any activation, so the wait at a barrier need not stop
// the HBM stream: in every workgroup four "producer" waves do nothing but issue direct-to-LDS loads of the
// workgroup's tiles, in the order in which they will be used and across stage borders, as far ahead as
// their rings have room; four "consumer" waves take the blocks out of the rings, multiply, reduce and run
// the epilogues and the device-wide barriers.  Producer p serves consumer p alone (blocks p, p + 4, ... of
// every tile) through a ring of its own and two LDS counters (blocks landed / blocks released); no
// workgroup barrier is involved, so one late block delays one wave, not eight.
//
// The order of tiles and blocks is a pure function of the descriptors, the workgroup index and p;
// producer, consumer and the host-side checker walk it with the same code (PairWalk).
#pragma once
#include "decode.hpp"

namespace lr {

constexpr int kRingStages = 4;
constexpr int kRingProbs = 4;
constexpr int kRingConsumers = 4;                    // consumer waves = blocks per round
constexpr int kRingProducers = 4;                    // producer wave p feeds consumer wave p
constexpr int kRingChunkBytes = 32 * 64 * 2;         // one block: 32 rows x 64 columns of bf16
constexpr int kRingLdsBytes = 156 * 1024;           // rings + activation regions + reduction scratch
constexpr int kRingMaxDepth = 8, kRingMinDepth = 3;  // blocks per pair ring: as many as the rest leaves room for
constexpr int kRingRedStride = 68;                   // floats per row of a wave's partial tile (64 + 4: rows fall into different banks)

// how a stage reads its activation rows
enum { RA_BF16_PLAIN = 0,    // bf16, written before the launch or finalised earlier in it: plain loads
       RA_F32_COHERENT = 1,  // fp32 accumulators other workgroups of this launch added into (epoch-parity area)
       RA_BF16_COHERENT = 2  // bf16 rows other workgroups of this launch stored (hidden rows)
};

struct RStage {
    DProb p[kRingProbs];
    int nprob, total_tiles;
    int epi;          // EPI_*
    int a_kind;       // RA_*
    int finalise;     // EPI_ATOMIC: partial tiles to slots + bf16 finalisation by the last K-slice (larger row counts)
};

struct RingArgs {
    FusedCommon fc;
    int nstages, M;
    int depth;        // blocks each pair's LDS ring holds (kRingMinDepth..kRingMaxDepth)
    int wmax;         // cap of that window
    int window0;      // blocks a producer may have in flight at kernel start (grows by one per landed block up to depth)
    int a_bytes;      // bytes of one consumer wave's activation region (behind the rings)
    int red_bufs;     // 2: the reduction scratch alternates between tiles; 1: one scratch, one more consumer sync per tile
    int a_rows;       // activation rows kept in LDS: the power of two >= M (MFMA row j reads row j mod a_rows)
    RStage st[kRingStages];
};

// One workgroup tile as the rings see it: nb1 blocks of 32 rows of W starting at row 32 * kb0, then nb2 blocks
// of W2 from its row 0 (gate/up stages); block b belongs to pair b % 4.
struct RingTile {
    int pi;           // problem index inside the stage
    int lt;           // tile index inside the problem
    int n0;           // first column
    int kb0, nb1, nb2;
};

__host__ __device__ inline RingTile ring_tile(const RStage& st, int tile) {
    RingTile t;
    int pi = 0;
    for (int i = 1; i < kRingProbs; ++i)
        if (i < st.nprob && tile >= st.p[i].tile_begin) pi = i;
    const DProb& P = st.p[pi];
    t.pi = pi;
    t.lt = tile - P.tile_begin;
    const int tn = t.lt % P.tiles_n, tk = t.lt / P.tiles_n;
    t.n0 = tn * 64;
    t.kb0 = tk * (P.KS >> 5);
    int kb1 = t.kb0 + (P.KS >> 5);
    if (kb1 > (P.K >> 5)) kb1 = P.K >> 5;
    t.nb1 = kb1 - t.kb0;
    t.nb2 = st.epi == EPI_GATEUP ? (P.K2 >> 5) : 0;
    return t;
}

// Position of pair p in its sequence of blocks: stages in order, the workgroup's tiles of a stage
// (wg, wg + grid, ...) in order, the pair's blocks of a tile (p, p + 4, ...) in order; tiles with fewer
// than p + 1 blocks are passed over.
struct PairWalk {
    int s, tile, b;
    RingTile t;
};

__host__ __device__ inline void pair_walk_settle(PairWalk& w, const RingArgs& ra, int wg, int grid, int p) {
    while (w.s < ra.nstages) {
        if (w.tile >= ra.st[w.s].total_tiles) { ++w.s; w.tile = wg; continue; }
        w.t = ring_tile(ra.st[w.s], w.tile);
        if (p < w.t.nb1 + w.t.nb2) break;
        w.tile += grid;
    }
    w.b = p;
}
__host__ __device__ inline void pair_walk_begin(PairWalk& w, const RingArgs& ra, int wg, int grid, int p) {
    w.s = 0; w.tile = wg;
    pair_walk_settle(w, ra, wg, grid, p);
}
__host__ __device__ inline bool pair_walk_live(const PairWalk& w, const RingArgs& ra) { return w.s < ra.nstages; }
__host__ __device__ inline void pair_walk_next(PairWalk& w, const RingArgs& ra, int wg, int grid, int p) {
    w.b += kRingConsumers;
    if (w.b < w.t.nb1 + w.t.nb2) return;
    w.tile += grid;
    pair_walk_settle(w, ra, wg, grid, p);
}

// Whether the streaming kernel can run this chain (host); sets ra.depth, ra.a_bytes, ra.red_bufs.  Fills `why` on refusal.
bool ring_args_ok(RingArgs& ra, int grid, const char** why);
// Walks every pair's sequence on the host: every block inside its matrix, every block of every tile visited once.
bool ring_walk_check(const RingArgs& ra, int grid, const char** why);
int decode_launch_ring(const RingArgs& ra, int grid, hipStream_t s);

}  // namespace lr
