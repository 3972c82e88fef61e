// Matrix-core backward kernel of the Renderer: the instantiations that are built without the
// VGPR-form build flag (see lp_mfma_bwd.h): direction inputs with contract coordinates, and
// direction inputs with two hidden layers of width 64 on a triplane.
#include "lp_mfma_bwd.h"

namespace lp {

namespace {

template <int KIND>
hipError_t dispatch_b(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                      hipStream_t stream)
{
    const int H = m.dims[1], NH = m.n_layers - 1;
    if (g.contract > 0.0) {
#define LP_CASE(h, nh) \
    if (H == h && NH == nh) return launch_bwd<KIND, 32, h, nh, true, 16, kAnyDtype>(g, m, rays, io, n_cu, stream);
        LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2) LP_CASE(64, 2)
#undef LP_CASE
        return hipErrorInvalidValue;
    }
    if constexpr (KIND == LP_GRID_TRIPLANE) {
        if (H == 64 && NH == 2) return launch_bwd<KIND, 32, 64, 2, false, 16, kAnyDtype>(g, m, rays, io, n_cu, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_bwd_mfma_b(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                             hipStream_t stream)
{
    if (m.dims[0] != 32 || g.C != 16) return hipErrorInvalidValue;
    return g.kind == LP_GRID_VOXEL ? dispatch_b<LP_GRID_VOXEL>(g, m, rays, io, n_cu, stream)
                                   : dispatch_b<LP_GRID_TRIPLANE>(g, m, rays, io, n_cu, stream);
}

}  // namespace lp
