// Matrix-core backward kernel of the Renderer over a hash table (Section 3.2 names hash tables among
// the structures h): the instantiations of lp_mfma_bwd.h for it.  The storage type and the
// contraction are run-time branches, so that one set of kernels serves every table.
#include "lp_mfma_bwd.h"

namespace lp {

hipError_t launch_bwd_mfma_hash(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                                hipStream_t stream)
{
    const int C = m.dims[0], H = m.dims[1], NH = m.n_layers - 1;
#define LP_CASE(c, h, nh)                         \
    if (C == c && g.C == c && H == h && NH == nh) \
        return launch_bwd<LP_GRID_HASH, c, h, nh, false, c, kAnyDtype>(g, m, rays, io, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    // 16 grid channels + direction inputs (the two-MLP decoder merged into one MLP of 32 inputs)
#define LP_CASE(h, nh)                             \
    if (C == 32 && g.C == 16 && H == h && NH == nh) \
        return launch_bwd<LP_GRID_HASH, 32, h, nh, false, 16, kAnyDtype>(g, m, rays, io, n_cu, stream);
    LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2) LP_CASE(64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace lp
