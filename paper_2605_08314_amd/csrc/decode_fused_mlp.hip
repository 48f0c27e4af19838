// Launcher of the fused four-stage decode kernel (lowrank_packed_mlp).
#include "decode_device.hpp"

namespace lr {

// Weight blocks a wave requests ahead in each of the four stages, on eight waves per workgroup.  Up to 16 rows: three, and two in
// the gate/up stage (against three there: 26.7 / 31.2 / 32.8 us at 1 / 8 / 16 rows instead of 26.9 / 31.6 / 33.3; four: no gain).
// From 17 rows on (two 16-row blocks per wave) the gate/up stage, with its two accumulator sets, has registers for two blocks
// ahead (three spill: 46 us at 32 rows); the other stages keep two or three, which covers a wave's whole share of their
// tiles, so that those bytes stream while the barrier in front of the stage is pending.  Measured at 17 / 24 / 32 rows:
// 34.6 / 36.5 / 39.3 us, against 37.5 / 39.3 / 41.7 with one block ahead in every stage and 42.5 / 43.9 / 45.4 with three
// blocks on four waves (the most that configuration's registers allowed on eight).
template <int MB, int CA, int CC, int CD>
static int launch_mlp(const FusedMlpArgs& fa, int grid, bool t16, hipStream_t s) {
    constexpr int NW = 8;
    void (*kern)(FusedMlpArgs) = nullptr;
    if constexpr (MB == 1) kern = t16 ? k_decode_fused_mlp<MB, CA, CC, CD, 3, 2, 3, 3, NW, true> : k_decode_fused_mlp<MB, CA, CC, CD, 3, 2, 3, 3, NW, false>;
    else kern = t16 ? k_decode_fused_mlp<MB, CA, CC, CD, 2, 2, 3, 3, NW, true> : k_decode_fused_mlp<MB, CA, CC, CD, 2, 2, 3, 3, NW, false>;
    if (!decode_grid_is_resident((const void*)kern, 64 * NW, grid)) return LR_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * NW), 0, s, fa);
    return launch_status("fused decode (packed MLP)");
}

template <int MB>
static int launch_mlp_cpl(const FusedMlpArgs& fa, int ca, int cc, int cd, int grid, bool t16, hipStream_t s) {
    if (cd != 4 || ca != 4 || cc != 4) { set_error("bad decode tile configuration"); return LR_ERR_UNSUPPORTED; }
    return launch_mlp<MB, 4, 4, 4>(fa, grid, t16, s);
}

int decode_launch_fused_mlp(const FusedMlpArgs& fa, int cpl_a, int cpl_c, int cpl_d, int grid, bool t16, hipStream_t s) {
    if (fa.a.M <= 0) return LR_OK;
    if (fa.a.M <= 16) return launch_mlp_cpl<1>(fa, cpl_a, cpl_c, cpl_d, grid, t16, s);
    return launch_mlp_cpl<2>(fa, cpl_a, cpl_c, cpl_d, grid, t16, s);
}

}  // namespace lr
