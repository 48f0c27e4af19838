// Launchers of the per-stage decode kernels (one launch per stage).
#include "decode_device.hpp"

namespace lr {

template <int MB, int CPL>
static int launch_stage_cfg(const DStage& st, bool a_f32, int epi, hipStream_t s) {
    const dim3 grid((unsigned)st.total_tiles), block(256);
    constexpr int PF = 3;
    if (epi == EPI_ATOMIC) {
        if (a_f32) hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_ATOMIC, PF>), grid, block, 0, s, st);
        else       hipLaunchKernelGGL((k_decode_stage<MB, CPL, false, EPI_ATOMIC, PF>), grid, block, 0, s, st);
    } else if (epi == EPI_STORE) {
        if (a_f32) hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_STORE, PF>), grid, block, 0, s, st);
        else       hipLaunchKernelGGL((k_decode_stage<MB, CPL, false, EPI_STORE, PF>), grid, block, 0, s, st);
    } else {
        if (!a_f32) { set_error("gate/up stage expects the fp32 rank-space input"); return LR_ERR_UNSUPPORTED; }
        hipLaunchKernelGGL((k_decode_stage<MB, CPL, true, EPI_GATEUP, PF>), grid, block, 0, s, st);
    }
    return launch_status("decode stage");
}

int decode_launch_stage(const DStage& st, int cpl, bool a_f32, int epi, hipStream_t s) {
    if (st.total_tiles <= 0 || st.M <= 0) return LR_OK;
    const int mb = st.M <= 16 ? 1 : 2;
    if (mb == 1 && cpl == 4) return launch_stage_cfg<1, 4>(st, a_f32, epi, s);
    if (mb == 2 && cpl == 4) return launch_stage_cfg<2, 4>(st, a_f32, epi, s);
    set_error("bad decode tile configuration");
    return LR_ERR_UNSUPPORTED;
}

}  // namespace lr
