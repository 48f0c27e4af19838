// Launcher of the fused two-stage decode kernel (lowrank_linear, lowrank_qkv).
#include <stdlib.h>
#include <mutex>
#include "decode_device.hpp"

namespace lr {

template <int MB, int C1, int C2, int NP>
static int launch_f2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int grid, hipStream_t s) {
    Fused2Args<NP> fa;
    fa.fc = fc;
    for (int i = 0; i < NP; ++i) { fa.s1.p[i] = s1.p[i]; fa.s2.p[i] = s2.p[i]; }
    fa.s1.nprob = s1.nprob; fa.s1.M = s1.M; fa.s1.total_tiles = s1.total_tiles;
    fa.s2.nprob = s2.nprob; fa.s2.M = s2.M; fa.s2.total_tiles = s2.total_tiles;
    // eight waves; up to 16 rows each wave is two weight blocks ahead (measured against three in one run: the O projection
    // 8.96 against 9.25 us at one row and 0.2-0.3 us less up to 16 rows, QKV unchanged; one block ahead loses 0.7 us on QKV),
    // from 17 rows on three; the same in both stages (3 / 2, 2 / 3, 1 / 2, 2 / 1 measured: no better or worse)
    constexpr int PF = MB == 1 ? 2 : 3, NW = 8;
    void (*kern)(Fused2Args<NP>) = k_decode_fused2<MB, C1, C2, PF, PF, NP, NW>;
    if (!decode_grid_is_resident((const void*)kern, 64 * NW, grid)) return LR_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NW), 0, s, fa);
    return launch_status("fused decode (two stages)");
}

template <int MB, int NP>
static int launch_f2_cpl(const FusedCommon& fc, const DStage& s1, const DStage& s2, int c1, int c2, int grid, hipStream_t s) {
    if (c1 == 4 && c2 == 4) return launch_f2<MB, 4, 4, NP>(fc, s1, s2, grid, s);
    set_error("bad decode tile configuration");
    return LR_ERR_UNSUPPORTED;
}

int decode_launch_fused2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int cpl1, int cpl2, int grid, hipStream_t s) {
    if (s1.M <= 0) return LR_OK;
    const bool small = s1.nprob <= 4 && s2.nprob <= 4;
    if (s1.M <= 16) return small ? launch_f2_cpl<1, 4>(fc, s1, s2, cpl1, cpl2, grid, s) : launch_f2_cpl<1, 8>(fc, s1, s2, cpl1, cpl2, grid, s);
    return small ? launch_f2_cpl<2, 4>(fc, s1, s2, cpl1, cpl2, grid, s) : launch_f2_cpl<2, 8>(fc, s1, s2, cpl1, cpl2, grid, s);
}

// Whether `grid` workgroups of this very kernel (threads per workgroup as launched, static LDS only) can be resident at the
// same time on an otherwise idle device: the runtime's occupancy figure for the kernel times the number of compute units.
// Queried once per kernel; sets the error message when it does not fit.
bool decode_grid_is_resident(const void* kernel, int threads, int grid) {
    struct Seen { const void* k; int per_cu; };
    static Seen seen[64];
    static int n_seen = 0;
    static std::mutex mu;                                        // entry points may be called from several host threads
    std::lock_guard<std::mutex> lock(mu);
    int per_cu = -1;
    for (int i = 0; i < n_seen; ++i)
        if (seen[i].k == kernel) per_cu = seen[i].per_cu;
    if (per_cu < 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, 0) != hipSuccess) { (void)hipGetLastError(); n = 1; }   // (no figure: trust the launch bounds)
        per_cu = n;
        if (n_seen < 64) seen[n_seen++] = Seen{kernel, per_cu};
    }
    const int cus = decode_resident_grid();
    if ((long)per_cu * (cus > 0 ? cus : 1) >= grid) return true;
    set_error("a fused decode launch of %d workgroups cannot be resident on this device (%d per compute unit x %d); "
              "use lowrank_configure(LR_CFG_DEVICE_SHARED, 1) for one launch per stage", grid, per_cu, cus);
    return false;
}

int decode_resident_grid() {
    // A fused launch needs every workgroup resident at the same time.  Each fused kernel is compiled for at least one
    // workgroup per CU, so one per CU is resident -- provided nothing else occupies CUs, which the caller vouches for
    // (lowrank_configure(LR_CFG_DEVICE_SHARED, 1) withdraws that and selects one launch per stage).
    if (g_device_shared) return 0;
    static int cached = 0;
    if (cached > 0) return cached;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 0;
    cached = cus;
    return cached;
}

}  // namespace lr
