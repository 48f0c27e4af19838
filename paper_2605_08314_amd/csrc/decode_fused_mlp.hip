// Launcher of the fused four-stage decode kernel (lowrank_packed_mlp).
#include "decode_device.hpp"

namespace lr {

// Weight blocks a wave requests ahead (PF) and waves per workgroup (NW).  Up to 16 rows: three blocks, eight waves.  From 17
// rows on (two 16-row blocks per wave) three blocks ahead no longer fit the registers of eight waves, and four waves leave
// every SIMD with a single wave; one block ahead on eight waves still keeps 32 KB per compute unit in flight, twice what
// saturates it (measured at 17 / 24 / 32 rows: 38.3 / 39.9 / 42.8 us against 42.5 / 43.9 / 45.4 with three blocks on four waves).
template <int MB, int CA, int CC, int CD>
static int launch_mlp(const FusedMlpArgs& fa, int grid, bool t16, hipStream_t s) {
    constexpr int PF = MB == 1 ? 3 : 1, NW = 8;
    void (*kern)(FusedMlpArgs) = t16 ? k_decode_fused_mlp<MB, CA, CC, CD, PF, NW, true> : k_decode_fused_mlp<MB, CA, CC, CD, PF, NW, false>;
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
