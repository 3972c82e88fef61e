// placeholder until the matrix-core kernels land
#include "lp_kernels.h"
namespace lp {
bool mfma_supported(const GridDev&, const MlpDev&) { return false; }
int mfma_bwd_records(int n_cu) { return 4 * n_cu; }
hipError_t launch_fwd_mfma(const GridDev&, const MlpDev&, const RaysDev&, const FwdOut&, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_mfma(const GridDev&, const MlpDev&, const RaysDev&, const BwdIo&, int, hipStream_t) { return hipErrorNotSupported; }
}
