// Decode phase, up to 16 token rows: the streaming kernel (see decode_ring.hpp for the idea).
//
// Workgroup = 8 waves: waves 0..3 consume, waves 4..7 produce; producer p serves consumer p.
// LDS: four rings of `depth` blocks (32 rows x 64 columns as in memory: 128-byte rows) | four activation
// regions (a consumer wave's own columns of the tile's activation rows, bf16) | reduction scratch | counters.
//
// Producer p: 4 x global_load_lds_dwordx4 (8 rows x 128 bytes each) per block, as long as its ring has a free
// slot (blocks requested - blocks released < depth); nothing else is in its vector-memory queue, so "my oldest
// block has landed" is one s_waitcnt vmcnt(4 * (blocks in flight - 1)) (requests complete in order), after
// which it publishes the count of landed blocks in LDS.
// Consumer p: waits for that count, ds_read_b64_tr_b16 turns the block's rows into the column-major MFMA
// operand (lane (j, g): column 16 * cb + j, rows 8g..8g+7), one 16-byte LDS read fetches the activation operand,
// four v_mfma_f32_16x16x32_bf16 per block; then it publishes the count of released blocks.
// The consumers meet once per tile (their partial tiles are added through LDS) at a counter in LDS.
//
// No loop below waits without a bound: a wait that exceeds its spin limit sets the workspace's error word and
// goes on (wrong results, reported by lowrank_workspace_status), so every wave reaches the end of the kernel.
#include <stdlib.h>
#include "decode_device.hpp"
#include "decode_ring.hpp"

namespace lr {

typedef short rs16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) rs16x4_t lds_rs16x4_t;

// 64 lanes x 16 bytes: global (src, per lane) -> LDS (dst + 16 * lane, dst wave-uniform); counted by vmcnt.
// The builtin (not inline assembly) so that the compiler knows this is a load: it may then overwrite the address
// registers while the request is in flight, where it would drain the queue before touching an opaque statement's operands.
__device__ __forceinline__ void ring_dma16(char* dst, const char* src) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
}
__device__ __forceinline__ void ring_drain_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void ring_drain_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// at most 4 * n vector-memory instructions of this wave still in flight
__device__ __forceinline__ void ring_wait_blocks(uint32_t n) {
    switch (n) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt vmcnt(20)" ::: "memory"); break;
        case 6: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
        default: asm volatile("s_waitcnt vmcnt(28)" ::: "memory"); break;
    }
}
static_assert(kRingMaxDepth - 1 <= 7, "ring_wait_blocks covers at most 7 later blocks");

// counters in LDS (uint32 words)
enum { RF_READY = 0,      // [4] blocks of pair p that have landed
       RF_FREED = 4,      // [4] blocks consumer p has released
       RF_SYNC = 8,       // arrivals at the consumers' meeting points
       RF_FIN = 9,        // consumer waves that have stored their share of a partial tile
       RF_OPEN = 10,      // stages whose device-wide barrier consumer wave 0 has seen complete
       RF_ARRIVE = 11,    // [3] consumer waves that have finished stage s
       RF_WORDS = 16 };
constexpr uint32_t kLdsSpinLimit = 1u << 24;

__device__ __forceinline__ uint32_t flag_load(const uint32_t* f) { return __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ void flag_store(uint32_t* f, uint32_t v) { __hip_atomic_store(f, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ uint32_t flag_add(uint32_t* f) { return __hip_atomic_fetch_add(f, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

// wave-uniform wait until *f >= want; returns the value seen
__device__ __forceinline__ uint32_t flag_wait(const uint32_t* f, uint32_t want, uint32_t* err) {
    uint32_t v, spins = 0;
    while (true) {
        v = __builtin_amdgcn_readfirstlane(flag_load(f));
        if (v >= want) break;
        if (++spins > kLdsSpinLimit) {
            if ((threadIdx.x & 63) == 0) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    asm volatile("" ::: "memory");
    return v;
}

// ---- producer ----------------------------------------------------------------------------------------
// The producers read and write their LDS counters through inline assembly: the compiler, which tracks direct-to-LDS
// loads, would otherwise drain the whole request queue (s_waitcnt vmcnt(0)) in front of every LDS access that it
// cannot prove distinct from the loads' destination.
__device__ __forceinline__ uint32_t pflag_load(uint32_t lds_addr) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr) : "memory");
    return __builtin_amdgcn_readfirstlane(v);
}
__device__ __forceinline__ void pflag_store(uint32_t lds_addr, uint32_t v) {
    asm volatile("ds_write_b32 %0, %1" :: "v"(lds_addr), "v"(v) : "memory");
}
struct ProducerState {
    uint32_t issued, landed, freed, slot, window, wmax, depth, spins;
    uint32_t freed_addr, ready_addr;
    uint32_t* err;
};

// the oldest block in flight has landed: publish it
__device__ __forceinline__ void producer_retire(ProducerState& ps) {
    ring_wait_blocks(ps.issued - ps.landed - 1);
    ++ps.landed;
    pflag_store(ps.ready_addr, ps.landed);
    if (ps.window < ps.wmax) ++ps.window;
    ps.spins = 0;
}

// Returns once the ring has a free slot and the window allows another request (false: gave up, see the spin limit).
// While there is no room it retires blocks in flight, oldest first; with nothing in flight it looks at the consumer's
// counter now and then.
__device__ __forceinline__ bool producer_make_room(ProducerState& ps) {
    while (true) {
        if (ps.issued - ps.freed >= ps.depth) ps.freed = pflag_load(ps.freed_addr);
        if (ps.issued - ps.freed < ps.depth && ps.issued - ps.landed < ps.window) return true;
        if (ps.landed < ps.issued) { producer_retire(ps); continue; }
        if (++ps.spins > kLdsSpinLimit) {
            if ((threadIdx.x & 63) == 0) __hip_atomic_store(ps.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

__device__ __forceinline__ void producer_run(const RingArgs& ra, int p, int lane, char* ring_lds, uint32_t* flags) {
    const int wg = blockIdx.x, grid = gridDim.x;
    ProducerState ps;
    ps.issued = 0; ps.landed = 0; ps.freed = 0; ps.slot = 0; ps.spins = 0;
    ps.depth = (uint32_t)ra.depth;
    // Blocks in flight are limited by a window that starts at half the ring and grows by one per landed block, so
    // that the first requests of all workgroups at kernel start are the blocks that are needed first.
    ps.wmax = (uint32_t)ra.wmax < ps.depth ? (uint32_t)ra.wmax : ps.depth;
    ps.window = (uint32_t)ra.window0 < ps.wmax ? (uint32_t)ra.window0 : ps.wmax;
    ps.err = &ra.fc.ctrl->error;
    char* ring0 = ring_lds + (size_t)p * ps.depth * kRingChunkBytes;
    const uint32_t flags_lds = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) uint32_t*)flags);
    ps.freed_addr = flags_lds + 4u * (RF_FREED + p);
    ps.ready_addr = flags_lds + 4u * (RF_READY + p);
    // Request i of a block (rows 8i..8i+7) stores the 16-byte pieces of a row in the order piece ^ 2i, which spreads the
    // four row groups that one transposing read touches over all banks (rows are 128 bytes: half the bank space).
    const size_t lane_row = (size_t)(lane >> 3);
    bool ok = true;
    for (int s = 0; s < ra.nstages && ok; ++s) {
        const RStage& st = ra.st[s];
        // Requests of the next stage do not start while this pair's blocks of the current stage are in flight: they
        // would compete with blocks that the whole device is waiting for.
        while (ps.landed < ps.issued) producer_retire(ps);
        for (int tile = wg; tile < st.total_tiles && ok; tile += grid) {
            const RingTile t = ring_tile(st, tile);
            const DProb& P = st.p[t.pi];
            const size_t rowbytes = (size_t)P.N * 2u;
            const size_t lane_off = lane_row * rowbytes + (size_t)t.n0 * 2u;
            const char* base1 = reinterpret_cast<const char*>(P.W) + (size_t)(32 * t.kb0) * rowbytes + lane_off;
            const char* base2 = reinterpret_cast<const char*>(t.nb2 ? P.W2 : P.W) + lane_off;
            const int nb = t.nb1 + t.nb2;
            for (int b = p; b < nb; b += kRingConsumers) {
                if (!producer_make_room(ps)) { ok = false; break; }
                const char* src = b < t.nb1 ? base1 + (size_t)(32 * b) * rowbytes : base2 + (size_t)(32 * (b - t.nb1)) * rowbytes;
                char* dst = ring0 + (size_t)ps.slot * kRingChunkBytes;
#pragma unroll
                for (int i = 0; i < 4; ++i) ring_dma16(dst + 1024 * i, src + (size_t)(8 * i) * rowbytes + (size_t)(((lane & 7) ^ (2 * i)) * 16));
                ++ps.issued;
                ps.slot = ps.slot + 1 == ps.depth ? 0u : ps.slot + 1;
            }
        }
    }
    while (ps.landed < ps.issued) producer_retire(ps);
    ring_drain_vm();
}

// ---- consumer ----------------------------------------------------------------------------------------
// This wave's columns of the tile's activation rows -> its LDS region as bf16, row stride ASW elements: local
// block lb (block wave + 4 lb of the tile) occupies columns [32 lb, 32 lb + 32).  Rows M..a_rows-1 are zero.
// No branch surrounds a load (indices are clamped instead), so the loads of a batch are all in flight together.
template <int KIND>
__device__ __forceinline__ void ring_load_a(char* aw, const DProb& P, const RingTile& t, int wave, int nbw, int M, int a_rows, int ASW, size_t shift) {
    const int lane = threadIdx.x & 63;
    const int GT = 4 * nbw;                                   // 8-element groups per row
    const int items = a_rows * GT;
    const char* A1 = reinterpret_cast<const char*>(P.A) + (KIND == RA_F32_COHERENT ? shift : 0);
    const char* A2 = reinterpret_cast<const char*>(t.nb2 ? P.A2 : P.A) + (KIND == RA_F32_COHERENT ? shift : 0);
    constexpr int ES = KIND == RA_F32_COHERENT ? 4 : 2;
    constexpr int UB = KIND == RA_F32_COHERENT ? 4 : 8;       // items per lane and batch
    const int lda1 = __builtin_amdgcn_readfirstlane(P.lda), lda2 = __builtin_amdgcn_readfirstlane(t.nb2 ? P.lda2 : P.lda);
    for (int it0 = lane; it0 < items; it0 += 64 * UB) {
        uint4 v[UB];
        uint2 wv[KIND == RA_F32_COHERENT ? UB : 1][4];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            int it = it0 + 64 * u;
            it = it < items ? it : items - 1;
            int m = it / GT;
            const int rem = it - m * GT;
            m = m < M ? m : M - 1;
            const int b = wave + 4 * (rem >> 2), c = rem & 3;
            const bool first = b < t.nb1;
            const char* base = first ? A1 : A2;
            const size_t ld = (size_t)(first ? lda1 : lda2);
            const size_t col = (size_t)(first ? 32 * (t.kb0 + b) : 32 * (b - t.nb1)) + (size_t)(8 * c);
            const char* src = base + ((size_t)m * ld + col) * ES;
            if constexpr (KIND == RA_BF16_PLAIN) {
                v[u] = *reinterpret_cast<const uint4*>(src);
            } else if constexpr (KIND == RA_BF16_COHERENT) {
                const uint2 a = ld_coherent_b64(src), b2 = ld_coherent_b64(src + 8);
                v[u] = make_uint4(a.x, a.y, b2.x, b2.y);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) wv[u][q] = ld_coherent_b64(src + 8 * q);
            }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int it = it0 + 64 * u;
            if (it < items) {
                const int m = it / GT, rem = it - m * GT;
                if constexpr (KIND == RA_F32_COHERENT) {
                    v[u] = make_uint4(pack2(__uint_as_float(wv[u][0].x), __uint_as_float(wv[u][0].y)), pack2(__uint_as_float(wv[u][1].x), __uint_as_float(wv[u][1].y)),
                                      pack2(__uint_as_float(wv[u][2].x), __uint_as_float(wv[u][2].y)), pack2(__uint_as_float(wv[u][3].x), __uint_as_float(wv[u][3].y)));
                }
                if (m >= M) v[u] = make_uint4(0u, 0u, 0u, 0u);
                *reinterpret_cast<uint4*>(aw + ((size_t)m * ASW + 8 * rem) * 2) = v[u];
            }
        }
    }
}

__device__ __forceinline__ void consumers_meet(uint32_t* flags, uint32_t& meetings, uint32_t* err) {
    ring_drain_lds();                                         // this wave's LDS writes are done
    if ((threadIdx.x & 63) == 0) flag_add(flags + RF_SYNC);
    ++meetings;
    flag_wait(flags + RF_SYNC, meetings * kRingConsumers, err);
}

__device__ __forceinline__ void consumer_run(const RingArgs& ra, int wave, int lane, char* lds, uint32_t* flags) {
    const int tid = threadIdx.x;                              // 0..255
    const int j = lane & 15, g = lane >> 4;
    const int wg = blockIdx.x, G = gridDim.x;
    const uint32_t depth = (uint32_t)ra.depth;
    const int M = ra.M, a_rows = ra.a_rows;
    uint32_t* err = &ra.fc.ctrl->error;
    const char* ring = lds + (size_t)wave * depth * kRingChunkBytes;
    char* aw = lds + (size_t)kRingConsumers * depth * kRingChunkBytes + (size_t)wave * ra.a_bytes;
    float* red0 = reinterpret_cast<float*>(lds + (size_t)kRingConsumers * depth * kRingChunkBytes + (size_t)kRingConsumers * ra.a_bytes);
    const int red_floats = kRingConsumers * 2 * a_rows * kRingRedStride;

    // {epoch, dirty extents} of the control block: read once per wave, after the first tile's activation loads have been
    // issued (vector-memory results return in order, so an earlier device-coherent read would hold those loads back).
    uint32_t ctl_e = 0;
    uint2 ctl_d = make_uint2(0u, 0u);
    bool have_ctl = false;
    auto load_ctl = [&]() {
        if (!have_ctl) {
            ctl_e = ld_agent(&ra.fc.ctrl->epoch);
            ctl_d = ld_coherent_b64(&ra.fc.ctrl->dirty[0]);
            have_ctl = true;
        }
    };
    // The control block comes through a device-coherent load that takes a microsecond or two; nothing may wait for it
    // before the first tile's blocks have been multiplied, so every use of the parity goes through an opaque copy that
    // the compiler cannot hoist to the top of the kernel.
    auto snapshot = [&]() -> CtrlSnap {
        uint32_t e = ctl_e, d0 = ctl_d.x, d1 = ctl_d.y;
        asm volatile("" : "+v"(e), "+v"(d0), "+v"(d1));
        CtrlSnap c;
        c.epoch = e; c.p = e & 1u; c.dirty_other = c.p ? d0 : d1;
        return c;
    };
    auto parity = [&]() -> uint32_t { return snapshot().p; };
    LR_STAMP_TO(ra.fc.trace, 0);

    uint32_t seq = 0, seen = 0, slot = 0, meetings = 0, tiles_done = 0;
    // this lane's source word of a transposing read (column block cb = 0): row 8g + (lane % 16) / 4 of the block, 8 bytes
    // lane % 4 of the 32-byte column group; the group of column block cb sits at position cb ^ g of its row (see the producer)
    const int boff = (8 * g + ((lane & 15) >> 2)) * 128 + (lane & 3) * 8;

    for (int s = 0; s < ra.nstages; ++s) {
        const RStage& st = ra.st[s];
        bool waited = (s == 0);
        for (int tile = wg; tile < st.total_tiles; tile += G) {
            const RingTile t = ring_tile(st, tile);
            const DProb& P = st.p[t.pi];
            if (!waited) {
                if (wave == 0) {
                    // lane i < kSlots watches slot i of the previous stage's barrier
                    const uint32_t* slots = ra.fc.ctrl->cnt[parity()][s - 1];
                    const uint32_t want = (uint32_t)lane < (uint32_t)kSlots ? ((uint32_t)G + kSlots - 1 - lane) / kSlots : 0u;
                    const uint32_t* pslot = slots + ((uint32_t)lane < (uint32_t)kSlots ? lane : 0) * kSlotStride;
                    uint32_t spins = 0;
                    while (true) {
                        const bool ok = ld_agent(pslot) >= want;
                        if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
                        if (++spins > kSpinLimit) {
                            if (lane == 0) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    if (lane == 0) flag_store(flags + RF_OPEN, (uint32_t)s);
                    if (s == 1) fused_publish(ra.fc, snapshot());
                } else {
                    flag_wait(flags + RF_OPEN, (uint32_t)s, err);
                }
                LR_STAMP_TO(ra.fc.trace, 3 * s);
                waited = true;
            }
            const int nb = t.nb1 + t.nb2;
            const int nbw = nb > wave ? (nb - wave + kRingConsumers - 1) / kRingConsumers : 0;
            const int ASW = 32 * nbw + 8;
            if (st.a_kind == RA_BF16_PLAIN) ring_load_a<RA_BF16_PLAIN>(aw, P, t, wave, nbw, M, a_rows, ASW, 0);
            else if (st.a_kind == RA_F32_COHERENT) ring_load_a<RA_F32_COHERENT>(aw, P, t, wave, nbw, M, a_rows, ASW, (size_t)parity() * ra.fc.acc_bytes);
            else ring_load_a<RA_BF16_COHERENT>(aw, P, t, wave, nbw, M, a_rows, ASW, 0);
            load_ctl();

            f32x4_t acc[2][4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) acc[mt][cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            const char* arow = aw + (size_t)(j & (a_rows - 1)) * ASW * 2 + 16 * g;

            for (int lb = 0; lb < nbw; ++lb) {
                if (seen <= seq) seen = flag_wait(flags + RF_READY + wave, seq + 1, err);
                const char* chunk = ring + slot * kRingChunkBytes + boff;
                bf16x8_t bv[4];
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) {
                    union { struct { rs16x4_t lo, hi; } h; bf16x8_t v; } x;
                    x.h.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_rs16x4_t*)(chunk + (cb ^ g) * 32));
                    x.h.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_rs16x4_t*)(chunk + (cb ^ g) * 32 + 4 * 128));
                    bv[cb] = x.v;
                }
                const uint4 a4 = *reinterpret_cast<const uint4*>(arow + 64 * lb);
                const bf16x8_t av = as_bf16x8(a4.x, a4.y, a4.z, a4.w);
                ring_drain_lds();                               // the block has been read: its slot may be refilled
                ++seq;
                slot = slot + 1 == depth ? 0u : slot + 1;
                if (lane == 0) flag_store(flags + RF_FREED + wave, seq);
                if (wave + kRingConsumers * lb < t.nb1) {
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) acc[0][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv[cb], acc[0][cb], 0, 0, 0);
                } else {
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) acc[1][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv[cb], acc[1][cb], 0, 0, 0);
                }
            }

            // ---- cross-wave reduction and epilogue ----
            float* red = red0 + (ra.red_bufs == 2 ? (tiles_done & 1u) * red_floats : 0);
            const int nmat = st.epi == EPI_GATEUP ? 2 : 1;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                if (mt < nmat) {
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (4 * g + v < a_rows)
                                red[((wave * 2 + mt) * a_rows + 4 * g + v) * kRingRedStride + 16 * cb + j] = acc[mt][cb][v];
                }
            consumers_meet(flags, meetings, err);
            {
                const int m = tid >> 4, c4 = (tid & 15) * 4;
                const int n = t.n0 + c4;
                if (m < M) {
                    float val[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        if (mt >= nmat) continue;
                        float4 sum = *reinterpret_cast<const float4*>(&red[((0 * 2 + mt) * a_rows + m) * kRingRedStride + c4]);
#pragma unroll
                        for (int w = 1; w < kRingConsumers; ++w) {
                            const float4 o = *reinterpret_cast<const float4*>(&red[((w * 2 + mt) * a_rows + m) * kRingRedStride + c4]);
                            sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
                        }
                        val[mt][0] = sum.x; val[mt][1] = sum.y; val[mt][2] = sum.z; val[mt][3] = sum.w;
                    }
                    if (st.epi == EPI_ATOMIC) {
                        if (st.finalise) {
                            float* ps = P.part + (size_t)(P.tile_begin + t.lt) * (16 * 64) + (size_t)m * 64 + c4;
                            st_coherent_b64(ps, make_uint2(__float_as_uint(val[0][0]), __float_as_uint(val[0][1])));
                            st_coherent_b64(ps + 2, make_uint2(__float_as_uint(val[0][2]), __float_as_uint(val[0][3])));
                        } else {
                            // returning atomics, consumed below: performed before this workgroup's arrival is counted
                            float* c = reinterpret_cast<float*>(reinterpret_cast<char*>(P.C) + (size_t)parity() * ra.fc.acc_bytes) + (size_t)m * P.ldc + n;
                            const float r0 = unsafeAtomicAdd(c, val[0][0]), r1 = unsafeAtomicAdd(c + 1, val[0][1]);
                            const float r2 = unsafeAtomicAdd(c + 2, val[0][2]), r3 = unsafeAtomicAdd(c + 3, val[0][3]);
                            asm volatile("" ::"v"(r0), "v"(r1), "v"(r2), "v"(r3));
                        }
                    } else if (st.epi == EPI_STORE) {
                        if (P.bias) {
                            float bv[4];
                            load_bf16_row<4>(bv, P.bias + n);
#pragma unroll
                            for (int b = 0; b < 4; ++b) val[0][b] += bv[b];
                        }
                        if (P.Y) store_bf16_row<4>(P.Y + (size_t)m * P.N + n, val[0]);
                        if (P.cache) {
                            const int bi = m / P.T, sq = m - bi * P.T;
                            const int64_t pp = (int64_t)P.pos[bi] + sq;
                            if (pp >= 0 && pp < P.S_max)
                                store_bf16_row<4>(reinterpret_cast<bf16_t*>(P.cache) + ((size_t)bi * P.S_max + (size_t)pp) * P.N + n, val[0]);
                        }
                    } else {
                        float bg[4] = {0.f, 0.f, 0.f, 0.f}, bu[4] = {0.f, 0.f, 0.f, 0.f}, hv[4];
                        if (P.bias) load_bf16_row<4>(bg, P.bias + n);
                        if (P.bias2) load_bf16_row<4>(bu, P.bias2 + n);
#pragma unroll
                        for (int b = 0; b < 4; ++b) hv[b] = silu_f32(val[0][b] + bg[b]) * (val[1][b] + bu[b]);
                        st_coherent_b64(P.Y + (size_t)m * P.N + n, make_uint2(pack2(hv[0], hv[1]), pack2(hv[2], hv[3])));
                    }
                }
            }
            if (st.epi == EPI_ATOMIC && st.finalise) {
                // The consumer wave that stores its share of the partial tile last counts the tile's K-slice in; the
                // K-slice of this column tile that is counted last adds all slices in slice order and writes bf16.
                ring_drain_vm();
                uint32_t mine = 0;
                if (lane == 0) mine = flag_add(flags + RF_FIN);
                mine = __builtin_amdgcn_readfirstlane(mine);
                if ((mine & (kRingConsumers - 1)) == kRingConsumers - 1) {
                    const int tn = t.lt % P.tiles_n;
                    const uint32_t slices = (uint32_t)((P.K + P.KS - 1) / P.KS);
                    uint32_t old = 0;
                    if (lane == 0) old = __hip_atomic_fetch_add(ra.fc.ctrl->tcnt[parity()] + P.ctile_begin + tn, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    old = __builtin_amdgcn_readfirstlane(old);
                    if (old == slices - 1u) {
                        const size_t sl_sz = (size_t)16 * 64, step = (size_t)P.tiles_n * sl_sz;
                        for (int it = lane; it < M * 16; it += 64) {
                            const int m = it >> 4, c4 = 4 * (it & 15);
                            const float* src = P.part + (size_t)(P.tile_begin + tn) * sl_sz + (size_t)m * 64 + c4;
                            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
                            for (uint32_t sl0 = 0; sl0 < slices; sl0 += 8) {
                                uint2 a[8], b[8];
#pragma unroll
                                for (uint32_t u = 0; u < 8; ++u) {
                                    const uint32_t sl = sl0 + u < slices ? sl0 + u : slices - 1;
                                    a[u] = ld_coherent_b64(src + (size_t)sl * step); b[u] = ld_coherent_b64(src + (size_t)sl * step + 2);
                                }
#pragma unroll
                                for (uint32_t u = 0; u < 8; ++u)
                                    if (sl0 + u < slices) {
                                        s0 += __uint_as_float(a[u].x); s1 += __uint_as_float(a[u].y);
                                        s2 += __uint_as_float(b[u].x); s3 += __uint_as_float(b[u].y);
                                    }
                            }
                            st_coherent_b64(P.Y + (size_t)m * P.ldy + t.n0 + c4, make_uint2(pack2(s0, s1), pack2(s2, s3)));
                        }
                    }
                }
            }
            ++tiles_done;
            if (ra.red_bufs != 2) consumers_meet(flags, meetings, err);      // one scratch: all have read it before the next tile writes it
        }
        LR_STAMP_TO(ra.fc.trace, 3 * s + 1);
        load_ctl();
        if (s + 1 < ra.nstages) {
            if (s == 0) {
                // clear what the previous call left in the other accumulator area and the other parity's counters
                const CtrlSnap cs = snapshot();
                const uint32_t par = cs.p;
                const uint32_t n4 = (cs.dirty_other + 3u) >> 2;
                float4* other = reinterpret_cast<float4*>(ra.fc.acc0 + (size_t)(1u - par) * ra.fc.acc_bytes);
                for (uint32_t i = (uint32_t)wg * 256u + (uint32_t)tid; i < n4; i += (uint32_t)G * 256u) other[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (wg == 0) {
                    for (uint32_t i = tid; i < (uint32_t)(kBarriers * kSlots); i += 256u)
                        ra.fc.ctrl->cnt[1u - par][i / kSlots][(i % kSlots) * kSlotStride] = 0u;
                    for (uint32_t i = tid; i < (uint32_t)kTileCounters; i += 256u) ra.fc.ctrl->tcnt[1u - par][i] = 0u;
                }
            }
            // the consumer wave that finishes the stage last signals the workgroup's arrival
            ring_drain_vm();                                    // this wave's stores and atomics of the stage have been performed
            uint32_t mine = 0;
            if (lane == 0) mine = flag_add(flags + RF_ARRIVE + s);
            mine = __builtin_amdgcn_readfirstlane(mine);
            if (mine == kRingConsumers - 1 && lane == 0)
                __hip_atomic_fetch_add(ra.fc.ctrl->cnt[parity()][s] + (wg % kSlots) * kSlotStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            LR_STAMP_TO(ra.fc.trace, 3 * s + 2);
        }
    }
    // workgroup 0 always owns tile 0 of every stage, so its wave 0 has published the epoch after its first wait
}

__global__ void __launch_bounds__(64 * (kRingConsumers + kRingProducers)) k_decode_ring(RingArgs ra) {
    __shared__ __attribute__((aligned(1024))) char lds[kRingLdsBytes];
    __shared__ uint32_t flags[RF_WORDS];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid < RF_WORDS) flags[tid] = 0u;
    {
        // Touch every cache line of the kernel arguments at once.  The walks below read the descriptors through chains of
        // dependent scalar loads (stage -> problem -> pointers); each first touch of a line is a trip to memory, and with
        // this the trips overlap instead of adding up.
        const __attribute__((address_space(4))) uint32_t* ka = (const __attribute__((address_space(4))) uint32_t*)__builtin_amdgcn_kernarg_segment_ptr();
        uint32_t acc = 0;
#pragma unroll
        for (int off = 0; off < (int)sizeof(RingArgs); off += 64) acc += ka[off / 4];
        asm volatile("" ::"s"(acc));
    }
    __syncthreads();                                            // the only workgroup barrier of the kernel
    if (wave >= kRingConsumers) {
        producer_run(ra, wave - kRingConsumers, lane, lds, flags);
    } else {
        consumer_run(ra, wave, lane, lds, flags);
    }
}

// ---- host ------------------------------------------------------------------------------------------

bool ring_args_ok(RingArgs& ra, int grid, const char** why) {
    *why = "";
    if (ra.M < 1 || ra.M > 16) { *why = "more than 16 token rows"; return false; }
    if (ra.nstages < 2 || ra.nstages > kRingStages || ra.nstages - 1 > kBarriers) { *why = "stage count"; return false; }
    if (grid < 1) { *why = "grid"; return false; }
    if (ra.a_rows < 1 || ra.a_rows > 16 || (ra.a_rows & (ra.a_rows - 1)) != 0) { *why = "activation rows"; return false; }
    if (ra.M > ra.a_rows) { *why = "activation rows"; return false; }
    int nb_max = 1;
    for (int s = 0; s < ra.nstages; ++s) {
        const RStage& st = ra.st[s];
        if (st.nprob < 1 || st.nprob > kRingProbs || st.total_tiles < 1) { *why = "problem count"; return false; }
        for (int i = 0; i < st.nprob; ++i) {
            const DProb& P = st.p[i];
            if (P.N % 64 || P.K % 32 || P.KS % 32 || P.KS < 32 || P.tiles_n != P.N / 64) { *why = "tile shape"; return false; }
            int kt = P.KS < P.K ? P.KS : P.K;
            if (st.epi == EPI_GATEUP) { if (P.K2 % 32) { *why = "tile shape"; return false; } kt = P.K + P.K2; }
            if (kt / 32 > nb_max) nb_max = kt / 32;
        }
    }
    const int nbw = (nb_max + kRingConsumers - 1) / kRingConsumers;
    const size_t a_bytes = ((size_t)ra.a_rows * (size_t)(32 * nbw + 8) * 2 + 255) & ~(size_t)255;
    const size_t red1 = (size_t)kRingConsumers * 2 * ra.a_rows * kRingRedStride * 4;
    for (int bufs = 2; bufs >= 1; --bufs) {
        const size_t rest = (size_t)kRingConsumers * a_bytes + (size_t)bufs * red1;
        if (rest >= (size_t)kRingLdsBytes) continue;
        const size_t depth = ((size_t)kRingLdsBytes - rest) / ((size_t)kRingConsumers * kRingChunkBytes);
        if (depth >= (size_t)(bufs == 2 ? 5 : kRingMinDepth)) {
            ra.depth = (int)(depth > (size_t)kRingMaxDepth ? (size_t)kRingMaxDepth : depth);
            {
                const char* e = getenv("LOWRANK_RING_DEPTH");      // measurement overrides
                if (e && *e && atoi(e) >= kRingMinDepth && atoi(e) < ra.depth) ra.depth = atoi(e);
                e = getenv("LOWRANK_RING_WINDOW");
                ra.window0 = (e && *e && atoi(e) >= 1) ? atoi(e) : 4;
                e = getenv("LOWRANK_RING_WMAX");
                ra.wmax = (e && *e && atoi(e) >= 1) ? atoi(e) : 64;
            }
            ra.a_bytes = (int)a_bytes;
            ra.red_bufs = bufs;
            return true;
        }
    }
    *why = "activation rows leave no room for the rings";
    return false;
}

bool ring_walk_check(const RingArgs& ra, int grid, const char** why) {
    *why = "";
    long long want_blocks = 0;
    for (int s = 0; s < ra.nstages; ++s) {
        // the tiles of a stage are the tiles of its problems, back to back
        const RStage& st = ra.st[s];
        int expect = 0;
        for (int i = 0; i < st.nprob; ++i) {
            const DProb& P = st.p[i];
            if (P.tile_begin != expect) { *why = "tile_begin"; return false; }
            const int tk = (P.K + P.KS - 1) / P.KS;
            if (st.epi != EPI_ATOMIC && P.KS < P.K) { *why = "full-K stage with a split"; return false; }
            expect += P.tiles_n * (st.epi == EPI_ATOMIC ? tk : 1);
            want_blocks += (long long)P.tiles_n * (P.K / 32 + (st.epi == EPI_GATEUP ? P.K2 / 32 : 0));
        }
        if (expect != st.total_tiles) { *why = "total_tiles"; return false; }
    }
    // every pair's sequence: inside the matrices, in order, and together exactly the blocks of all tiles
    long long blocks = 0;
    for (int wg = 0; wg < grid; ++wg)
        for (int p = 0; p < kRingConsumers; ++p) {
            PairWalk w;
            pair_walk_begin(w, ra, wg, grid, p);
            int last_s = -1, last_tile = -1, last_b = -1;
            while (pair_walk_live(w, ra)) {
                const RStage& st = ra.st[w.s];
                if (w.tile % grid != wg || w.tile < 0 || w.tile >= st.total_tiles) { *why = "tile owner"; return false; }
                const bool same = w.s == last_s && w.tile == last_tile;
                if (w.s < last_s || (w.s == last_s && w.tile < last_tile) || (same && w.b <= last_b)) { *why = "walk order"; return false; }
                last_s = w.s; last_tile = w.tile; last_b = w.b;
                const DProb& P = st.p[w.t.pi];
                if (w.b % kRingConsumers != p || w.b < 0 || w.b >= w.t.nb1 + w.t.nb2 || w.t.nb1 < 1) { *why = "block index"; return false; }
                const bool first = w.b < w.t.nb1;
                const long long row0 = first ? 32ll * (w.t.kb0 + w.b) : 32ll * (w.b - w.t.nb1);
                const long long rows = first ? P.K : P.K2;
                if ((first ? (const void*)P.W : (const void*)P.W2) == nullptr) { *why = "null matrix"; return false; }
                if (row0 < 0 || row0 + 32 > rows || w.t.n0 < 0 || w.t.n0 + 64 > P.N) { *why = "block outside its matrix"; return false; }
                // the consumer's activation region holds this block's columns
                const int nbw = (w.t.nb1 + w.t.nb2 - p + kRingConsumers - 1) / kRingConsumers;
                if ((size_t)ra.a_rows * (size_t)(32 * nbw + 8) * 2 > (size_t)ra.a_bytes) { *why = "activation region"; return false; }
                if (++blocks > (1ll << 26)) { *why = "walk does not end"; return false; }
                pair_walk_next(w, ra, wg, grid, p);
            }
        }
    if (blocks != want_blocks) { *why = "blocks visited"; return false; }
    const size_t lds = (size_t)kRingConsumers * ra.depth * kRingChunkBytes + (size_t)kRingConsumers * ra.a_bytes +
                       (size_t)ra.red_bufs * kRingConsumers * 2 * ra.a_rows * kRingRedStride * 4;
    if (ra.depth < kRingMinDepth || ra.depth > kRingMaxDepth || lds > (size_t)kRingLdsBytes) { *why = "LDS layout"; return false; }
    return true;
}

int decode_launch_ring(const RingArgs& ra_in, int grid, hipStream_t s) {
    RingArgs ra = ra_in;
    const char* why = "";
    if (!ring_args_ok(ra, grid, &why)) { set_error("streaming decode kernel refused: %s", why); return LR_ERR_UNSUPPORTED; }
    const char* chk = getenv("LOWRANK_DECODE_CHECK");
    if (chk && *chk && atoi(chk) != 0 && !ring_walk_check(ra, grid, &why)) {
        set_error("streaming decode kernel: plan check failed: %s", why);
        return LR_ERR_UNSUPPORTED;
    }
    const char* dry = getenv("LOWRANK_DECODE_DRYRUN");
    if (dry && *dry && atoi(dry) != 0) return LR_OK;      // host-side tests of the plan: nothing is launched
    hipLaunchKernelGGL(k_decode_ring, dim3((unsigned)grid), dim3(64 * (kRingConsumers + kRingProducers)), 0, s, ra);
    return launch_status("decode (streaming)");
}

}  // namespace lr
