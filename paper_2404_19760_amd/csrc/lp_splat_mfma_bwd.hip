// Splatter backward on the matrix cores: dispatch, and the instantiations for voxel grids and
// 16-channel triplanes (see lp_splat_mfma_bwd.h).
#include "lp_splat_mfma_bwd.h"

namespace lp {

hipError_t launch_splat_mfma_bwd(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp,
                                 const BwdIo& io, int n_cu, hipStream_t stream)
{
    if (tgt.kind == LP_GRID_VOXEL)
        return tgt.C == 16 ? by_extras<LP_GRID_VOXEL, 1>(tgt, m, rays, sp, io, n_cu, stream)
                           : by_extras<LP_GRID_VOXEL, 2>(tgt, m, rays, sp, io, n_cu, stream);
    return tgt.C == 16 ? by_extras<LP_GRID_TRIPLANE, 1>(tgt, m, rays, sp, io, n_cu, stream)
                       : launch_splat_mfma_bwd_triplane32(tgt, m, rays, sp, io, n_cu, stream);
}

}  // namespace lp
