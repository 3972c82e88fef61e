// Kernels and host-side launchers shared between the translation units of the library.
#pragma once
#include "lp_device.h"

namespace lp {

// ---- generic scalar kernels (lp_generic.hip) ---------------------------------------
__global__ void fwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays, FwdOut out);
__global__ void bwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays, BwdIo io, int tiles_per_block);
constexpr int kGenericCellColumns = 16;  // LDS columns of the generic backward kernel that hold the lanes' cells
constexpr int kReduceThreads = 1024;  // block size of reduce_params_kernel; one block per 64 parameters
__global__ void reduce_params_kernel(MlpDev m, BwdIo io, int n_records);
__global__ void splat_fwd_generic_kernel(GridDev tgt, MlpDev m, RaysDev rays, SplatDev sp);
__global__ void splat_normalise_kernel(float* theta, const float* theta_w, long long cells, int C);
__global__ void fill_zero_kernel(float* p, long long n);
__global__ void splat_bwd_generic_kernel(GridDev tgt, MlpDev m, RaysDev rays, SplatDev sp, BwdIo io,
                                         int tiles_per_block);

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
// the part of it that lp_mfma_bwd_b.hip builds with other flags (direction inputs with contract
// coordinates or with two 64-wide hidden layers on a triplane)
hipError_t launch_bwd_mfma_b(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io,
                             int n_cu, hipStream_t stream);
// its instantiations for hash tables (lp_mfma_bwd_hash.hip)
hipError_t launch_bwd_mfma_hash(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io,
                                int n_cu, hipStream_t stream);

// its instantiations for HexPlanes (lp_mfma_bwd_hexplane.hip)
hipError_t launch_bwd_mfma_hexplane(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io,
                                    int n_cu, hipStream_t stream);

// the shapes that run as a pair of waves per ray (lp_mfma_bwd_ws.hip)
bool bwd_ws_supported(const GridDev& g, const MlpDev& m);
hipError_t launch_bwd_mfma_ws(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io,
                              int n_cu, hipStream_t stream);

// ---- naive Splatter forward, wavefront per ray (lp_splat_fast.hip): 16 or 32 channels ----
bool splat_naive_supported(const GridDev& tgt);
hipError_t launch_splat_naive(const GridDev& tgt, const RaysDev& rays, const SplatDev& sp, int n_cu,
                              hipStream_t stream);

// ---- Splatter forward with an MLP on the matrix cores (lp_splat_mfma.hip) ----------------
// Shapes covered: prior and target with the same 16 or 32 fp32 channels, no contraction; one or
// two hidden layers of width 64; pixel feature + direction encoding of at most 48 inputs.
bool splat_mfma_supported(const GridDev& tgt, const MlpDev& m, const SplatDev& sp);
hipError_t launch_splat_mfma(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp,
                             int n_cu, hipStream_t stream);
// backward of the same shapes (lp_splat_mfma_bwd.hip): one record of partial sums per wave,
// mfma_bwd_records(n_cu) of them, added up by reduce_params_kernel (launched by this call)
hipError_t launch_splat_mfma_bwd(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp,
                                 const BwdIo& io, int n_cu, hipStream_t stream);
// the part of it for 32-channel triplanes (lp_splat_mfma_bwd_t32.hip, built with other flags)
hipError_t launch_splat_mfma_bwd_triplane32(const GridDev& tgt, const MlpDev& m, const RaysDev& rays,
                                            const SplatDev& sp, const BwdIo& io, int n_cu, hipStream_t stream);

// ---- the two-MLP decoder as ONE block-structured MLP (lp_decoder.hip) ------------------
// Combined layer l has the opacity MLP's rows first, then the feature MLP's; a shallower MLP
// is carried through the extra layers by identity blocks (exact behind a ReLU); the first
// layer's columns are the grid channels, the direction encoding, zero padding.
struct DecLayout {
    int L, Ls, Lv;                   // layers: combined, opacity, feature
    int dims_s[LP_MAX_LAYERS + 1], dims_v[LP_MAX_LAYERS + 1];
    int C, E;                        // grid channels, direction-encoding width
    const float* Ws[LP_MAX_LAYERS]; const float* bs[LP_MAX_LAYERS];
    const float* Wv[LP_MAX_LAYERS]; const float* bv[LP_MAX_LAYERS];
    float* dWs[LP_MAX_LAYERS]; float* dbs[LP_MAX_LAYERS];  // backward only
    float* dWv[LP_MAX_LAYERS]; float* dbv[LP_MAX_LAYERS];
};
// layer widths of the merged MLP: dims[0] = in_width (>= C + E), dims[L] = 1 + n_feat
void dec_combined_dims(const DecLayout& d, int in_width, int dims[LP_MAX_LAYERS + 1]);
// packed[i] = value of combined parameter i (layout of MlpDev::w_off / b_off); grads, if not
// NULL, is zeroed (param_total floats)
hipError_t launch_dec_pack(const DecLayout& d, const MlpDev& m, float* packed, float* grads, hipStream_t stream);
// adds the combined gradient `grads` into the two MLPs' gradient buffers of `d`
hipError_t launch_dec_unpack(const DecLayout& d, const MlpDev& m, const float* grads, hipStream_t stream);

// ---- two-MLP decoder with two 3-layer MLPs of width 64 as two chains (lp_mfma_dec2*.hip) ----
// Device pointers of the two MLPs (three layers each; opacity [64][C], [64][64], [1][64];
// feature [64][C+E], [64][64], [3][64]) and, for the backward, of their gradients.
struct Dec2Dev {
    const float* Ws[3]; const float* bs[3];
    const float* Wv[3]; const float* bv[3];
    float* dWs[3]; float* dbs[3];
    float* dWv[3]; float* dbv[3];
    int E;   // width of the direction encoding (at most 32)
    int feat_act;   // 0: sigmoid features, 1: identity
};
// grids of 16 / 32 channels, both MLPs with two hidden layers of 64, three features (sigmoid or identity)
bool dec2_supported(const GridDev& g, const DecLayout& d, int n_feat, int feat_act);
Dec2Dev dec2_view(const DecLayout& d, int feat_act);
hipError_t launch_dec2_fwd(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const FwdOut& out, int n_cu,
                           hipStream_t stream);
// backward: ACCUMULATES into io.d_grid and into d's gradient pointers; io.ws holds
// mfma_bwd_records(n_cu) records of io.ws_stride floats (at least either MLP's parameter count);
// io.dW / io.db are not used
hipError_t launch_dec2_bwd(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const BwdIo& io, int n_cu,
                           hipStream_t stream);

}  // namespace lp
