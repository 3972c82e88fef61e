// Matrix-core backward kernel of the Renderer with a chain wave and a weights wave per ray (see
// lp_mfma_bwd_ws.h): shapes it covers and their instantiations.
#include "lp_mfma_bwd_ws.h"

#include <cstdlib>

namespace lp {

bool bwd_ws_supported(const GridDev& g, const MlpDev& m)
{
    static const bool off = [] { const char* e = std::getenv("LP_BWD_ONE_WAVE"); return e && e[0] == '1'; }();
    if (off) return false;
    return g.kind == LP_GRID_VOXEL && g.C == 16 && m.dims[0] == 16 && m.n_feat == 3 && m.feat_act == 0 && m.n_layers == 3 && m.dims[1] == 64 &&
           m.dims[2] == 64 && (g.dtype == LP_F32 || g.dtype == LP_BF16 || g.dtype == LP_F16);
}

hipError_t launch_bwd_mfma_ws(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                              hipStream_t stream)
{
    if (!bwd_ws_supported(g, m)) return hipErrorInvalidValue;
    // grids stored in bf16 / fp16 take the contraction as a run-time branch (as in the one-wave kernels)
    if (g.dtype == LP_BF16) return launch_bwd_ws<LP_GRID_VOXEL, 16, 64, false, LP_BF16>(g, m, rays, io, n_cu, stream);
    if (g.dtype == LP_F16) return launch_bwd_ws<LP_GRID_VOXEL, 16, 64, false, LP_F16>(g, m, rays, io, n_cu, stream);
    return g.contract > 0.0 ? launch_bwd_ws<LP_GRID_VOXEL, 16, 64, true>(g, m, rays, io, n_cu, stream)
                            : launch_bwd_ws<LP_GRID_VOXEL, 16, 64, false>(g, m, rays, io, n_cu, stream);
}

}  // namespace lp

extern "C" lp_status lp_diag_ws_phases(unsigned long long* cycles)
{
    if (!cycles) return LP_ERR_INVALID_ARG;
#ifdef LP_WS_PHASES
    if (hipMemcpyFromSymbol(cycles, HIP_SYMBOL(lp::g_ws_phase_cycles), sizeof(unsigned long long) * 32) != hipSuccess)
        return LP_ERR_HIP;
    static const unsigned long long zeros[32] = {};
    if (hipMemcpyToSymbol(HIP_SYMBOL(lp::g_ws_phase_cycles), zeros, sizeof(zeros)) != hipSuccess) return LP_ERR_HIP;
    return LP_OK;
#else
    return LP_ERR_UNSUPPORTED;
#endif
}
