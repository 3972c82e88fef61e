// Splatter backward on the matrix cores: the instantiations for 32-channel triplanes (see
// lp_splat_mfma_bwd.h).
#include "lp_splat_mfma_bwd.h"

namespace lp {

hipError_t launch_splat_mfma_bwd_triplane32(const GridDev& tgt, const MlpDev& m, const RaysDev& rays,
                                            const SplatDev& sp, const BwdIo& io, int n_cu, hipStream_t stream)
{
    return by_extras<LP_GRID_TRIPLANE, 2>(tgt, m, rays, sp, io, n_cu, stream);
}

}  // namespace lp
