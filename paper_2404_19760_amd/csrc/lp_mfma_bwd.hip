// placeholder until the matrix-core backward lands
#include "lp_kernels.h"
namespace lp {
int mfma_bwd_records(int n_cu) { return 0 * n_cu; }
hipError_t launch_bwd_mfma(const GridDev&, const MlpDev&, const RaysDev&, const BwdIo&, int, hipStream_t) { return hipErrorNotSupported; }
}
