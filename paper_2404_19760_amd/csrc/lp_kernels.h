// Kernels and host-side launchers shared between the translation units of the library.
#pragma once
#include "lp_device.h"

namespace lp {

// ---- generic scalar kernels (lp_generic.hip) ---------------------------------------
__global__ void fwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays, FwdOut out);
__global__ void bwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays, BwdIo io, int tiles_per_block);
__global__ void reduce_params_kernel(MlpDev m, BwdIo io, int n_records);

// ---- matrix-core kernels (lp_mfma_fwd.hip / lp_mfma_bwd.hip) -------------------------
// Shapes covered: C in {16, 32}, one or two hidden layers of equal width in {32, 64}.
bool mfma_supported(const GridDev& g, const MlpDev& m);
// Number of partial-sum records (one per wave) the backward writes for `n_cu` compute units.
int mfma_bwd_records(int n_cu);
// Launchers return hipSuccess or the failing HIP error; shape must be supported.
hipError_t launch_fwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out,
                           int n_cu, hipStream_t stream);
hipError_t launch_bwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io,
                           int n_cu, hipStream_t stream);

}  // namespace lp
