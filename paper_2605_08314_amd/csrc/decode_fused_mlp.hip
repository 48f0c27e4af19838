// Launcher of the fused four-stage decode kernel (lowrank_packed_mlp).
#include "decode_device.hpp"

namespace lr {

template <int MB, int CA, int CC, int CD>
static int launch_mlp(const FusedMlpArgs& fa, int grid, int nw, bool t16, hipStream_t s) {
    void (*kern)(FusedMlpArgs) = t16 ? (nw == 8 ? k_decode_fused_mlp<MB, CA, CC, CD, 3, 8, true> : k_decode_fused_mlp<MB, CA, CC, CD, 3, 4, true>)
                                     : (nw == 8 ? k_decode_fused_mlp<MB, CA, CC, CD, 3, 8, false> : k_decode_fused_mlp<MB, CA, CC, CD, 3, 4, false>);
    if (!decode_grid_is_resident((const void*)kern, 64 * nw, grid)) return LR_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * nw), 0, s, fa);
    return launch_status("fused decode (packed MLP)");
}

template <int MB>
static int launch_mlp_cpl(const FusedMlpArgs& fa, int ca, int cc, int cd, int grid, int nw, bool t16, hipStream_t s) {
    if (cd != 4 || ca != 4 || cc != 4) { set_error("bad decode tile configuration"); return LR_ERR_UNSUPPORTED; }
    return launch_mlp<MB, 4, 4, 4>(fa, grid, nw, t16, s);
}

int decode_launch_fused_mlp(const FusedMlpArgs& fa, int cpl_a, int cpl_c, int cpl_d, int grid, int nw, bool t16, hipStream_t s) {
    if (fa.a.M <= 0) return LR_OK;
    if (fa.a.M <= 16) return launch_mlp_cpl<1>(fa, cpl_a, cpl_c, cpl_d, grid, nw, t16, s);
    return launch_mlp_cpl<2>(fa, cpl_a, cpl_c, cpl_d, grid, nw, t16, s);
}

}  // namespace lr
