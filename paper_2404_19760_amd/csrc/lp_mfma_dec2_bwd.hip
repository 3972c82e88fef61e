// Backward of the Renderer with the two-chain decoder: launcher and instantiations (see
// lp_mfma_dec2_bwd.h).
#include "lp_mfma_dec2_bwd.h"

namespace lp {

namespace {

// record layout of one chain: a 3-layer MLP in -> 64 -> 64 -> out
MlpDev chain_mlp(int in, int out)
{
    MlpDev m = {};
    m.n_layers = 3;
    m.dims[0] = in; m.dims[1] = kH; m.dims[2] = kH; m.dims[3] = out;
    int off = 0;
    for (int l = 0; l < 3; ++l) {
        m.w_off[l] = off; off += m.dims[l] * m.dims[l + 1];
        m.b_off[l] = off; off += m.dims[l + 1];
    }
    m.param_total = off;
    return m;
}

template <int KIND>
hipError_t dispatch(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const BwdIo& io, int n_cu,
                    hipStream_t stream)
{
    const MlpDev ms = chain_mlp(g.C, 1), mv = chain_mlp(g.C + d.E, 3);
    if (io.ws_stride < ms.param_total || io.ws_stride < mv.param_total) return hipErrorInvalidValue;
    const bool cc = g.contract > 0.0;
    if (g.C == 16)
        return cc ? launch_dec2_bwd_t<KIND, 16, true>(g, d, ms, mv, rays, io, n_cu, stream)
                  : launch_dec2_bwd_t<KIND, 16, false>(g, d, ms, mv, rays, io, n_cu, stream);
    if (g.C == 32)
        return cc ? launch_dec2_bwd_t<KIND, 32, true>(g, d, ms, mv, rays, io, n_cu, stream)
                  : launch_dec2_bwd_t<KIND, 32, false>(g, d, ms, mv, rays, io, n_cu, stream);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_dec2_bwd(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const BwdIo& io, int n_cu,
                           hipStream_t stream)
{
    return g.kind == LP_GRID_VOXEL ? dispatch<LP_GRID_VOXEL>(g, d, rays, io, n_cu, stream)
                                   : dispatch<LP_GRID_TRIPLANE>(g, d, rays, io, n_cu, stream);
}

}  // namespace lp
