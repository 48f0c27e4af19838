// Launcher of the fused two-stage decode kernel (lowrank_linear, lowrank_qkv).
#include <stdlib.h>
#include "decode_device.hpp"

namespace lr {

template <int MB, int C1, int C2, int NP>
static int launch_f2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int grid, int nw, bool t16, hipStream_t s) {
    Fused2Args<NP> fa;
    fa.fc = fc;
    for (int i = 0; i < NP; ++i) { fa.s1.p[i] = s1.p[i]; fa.s2.p[i] = s2.p[i]; }
    fa.s1.nprob = s1.nprob; fa.s1.M = s1.M; fa.s1.total_tiles = s1.total_tiles;
    fa.s2.nprob = s2.nprob; fa.s2.M = s2.M; fa.s2.total_tiles = s2.total_tiles;
    if (t16) {
        if (nw == 8) hipLaunchKernelGGL((k_decode_fused2<MB, C1, C2, 3, NP, 8, true>), dim3((unsigned)grid), dim3(512), 0, s, fa);
        else hipLaunchKernelGGL((k_decode_fused2<MB, C1, C2, 3, NP, 4, true>), dim3((unsigned)grid), dim3(256), 0, s, fa);
    } else {
        if (nw == 8) hipLaunchKernelGGL((k_decode_fused2<MB, C1, C2, 3, NP, 8, false>), dim3((unsigned)grid), dim3(512), 0, s, fa);
        else hipLaunchKernelGGL((k_decode_fused2<MB, C1, C2, 3, NP, 4, false>), dim3((unsigned)grid), dim3(256), 0, s, fa);
    }
    return launch_status("fused decode (two stages)");
}

template <int MB, int NP>
static int launch_f2_cpl(const FusedCommon& fc, const DStage& s1, const DStage& s2, int c1, int c2, int grid, int nw, bool t16, hipStream_t s) {
    if (c1 == 4 && c2 == 4) return launch_f2<MB, 4, 4, NP>(fc, s1, s2, grid, nw, t16, s);
    set_error("bad decode tile configuration");
    return LR_ERR_UNSUPPORTED;
}

int decode_launch_fused2(const FusedCommon& fc, const DStage& s1, const DStage& s2, int cpl1, int cpl2,
                         int grid, int nw, bool t16, hipStream_t s) {
    if (s1.M <= 0) return LR_OK;
    const bool small = s1.nprob <= 4 && s2.nprob <= 4;
    if (s1.M <= 16) return small ? launch_f2_cpl<1, 4>(fc, s1, s2, cpl1, cpl2, grid, nw, t16, s)
                                 : launch_f2_cpl<1, 8>(fc, s1, s2, cpl1, cpl2, grid, nw, t16, s);
    return small ? launch_f2_cpl<2, 4>(fc, s1, s2, cpl1, cpl2, grid, nw, t16, s)
                 : launch_f2_cpl<2, 8>(fc, s1, s2, cpl1, cpl2, grid, nw, t16, s);
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
