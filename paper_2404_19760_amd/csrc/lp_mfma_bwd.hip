// Matrix-core backward kernel of the Renderer: dispatch and most instantiations (see
// lp_mfma_bwd.h).
#include "lp_mfma_bwd.h"

namespace lp {

namespace {

template <int KIND>
hipError_t dispatch_bwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                         hipStream_t stream)
{
    const int C = m.dims[0], CG = g.C, H = m.dims[1], NH = m.n_layers - 1;
    // grids stored in bf16 / fp16: plain inputs; the contraction is a run-time branch of these kernels
#define LP_CASE(c, h, nh)                                                                                  \
    if (C == c && CG == c && H == h && NH == nh && g.dtype != LP_F32)               \
        return g.dtype == LP_BF16 ? launch_bwd<KIND, c, h, nh, false, c, LP_BF16>(g, m, rays, io, n_cu, stream) \
                                  : launch_bwd<KIND, c, h, nh, false, c, LP_F16>(g, m, rays, io, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    if (g.dtype != LP_F32 && CG == C) return hipErrorInvalidValue;   // (the decoder kernels read any storage type)
#define LP_CASE(c, cg, h, nh)                                                                     \
    if (C == c && CG == cg && H == h && NH == nh)                                                 \
        return g.contract > 0.0 ? launch_bwd<KIND, c, h, nh, true, cg>(g, m, rays, io, n_cu, stream) \
                                : launch_bwd<KIND, c, h, nh, false, cg>(g, m, rays, io, n_cu, stream);
    LP_CASE(16, 16, 32, 1) LP_CASE(16, 16, 64, 1) LP_CASE(32, 32, 32, 1) LP_CASE(32, 32, 64, 1)
    LP_CASE(16, 16, 32, 2) LP_CASE(16, 16, 64, 2) LP_CASE(32, 32, 32, 2) LP_CASE(32, 32, 64, 2)
#undef LP_CASE
    // 16 grid channels + direction inputs (the two-MLP decoder merged into one MLP of 32 inputs);
    // with contract coordinates, and the widest variant on a triplane: the other translation unit
    if (C == 32 && CG == 16 && (g.contract > 0.0 || (KIND == LP_GRID_TRIPLANE && H == 64 && NH == 2)))
        return launch_bwd_mfma_b(g, m, rays, io, n_cu, stream);
#define LP_CASE(h, nh) \
    if (C == 32 && CG == 16 && H == h && NH == nh) \
        return launch_bwd<KIND, 32, h, nh, false, 16, kAnyDtype>(g, m, rays, io, n_cu, stream);
    LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2)
    if constexpr (KIND == LP_GRID_VOXEL) { LP_CASE(64, 2) }
#undef LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace

// one workgroup of 4 waves per compute unit, rounded up to a multiple of the 8 XCDs
int mfma_bwd_records(int n_cu) { return ((n_cu + 7) / 8 * 8) * kWaves; }

hipError_t launch_bwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                           hipStream_t stream)
{
    if (bwd_ws_supported(g, m)) return launch_bwd_mfma_ws(g, m, rays, io, n_cu, stream);
    if (g.kind == LP_GRID_HASH) return launch_bwd_mfma_hash(g, m, rays, io, n_cu, stream);
    if (g.kind == LP_GRID_HEXPLANE) return launch_bwd_mfma_hexplane(g, m, rays, io, n_cu, stream);
    return g.kind == LP_GRID_VOXEL ? dispatch_bwd<LP_GRID_VOXEL>(g, m, rays, io, n_cu, stream)
                                   : dispatch_bwd<LP_GRID_TRIPLANE>(g, m, rays, io, n_cu, stream);
}

}  // namespace lp
