// Naive Splatter forward (Section 3.3 "Splatter": every point of a pixel's ray pushes the pixel's
// feature vector into the cell that contains it), wavefront per ray.
//
// The push is the Renderer's backward scatter with a feature gradient that is constant along
// the ray, so it runs on the same machinery: a step is 32 points; lane (col, grp) of the step
// places point slot col and publishes its corner weights and cell offset in LDS; then the lanes
// turn into channels, walk 16 consecutive points each, sum the weights of runs that stay in one
// cell and issue one atomic add per corner on whole 64-byte lines (value = pixel feature times
// summed weight).  The weight sums go to the one-channel structure the same way, one lane per
// corner.  Ray groups are visited in scrambled order like the Renderer's backward (atomic adds
// of neighbouring rays queue up at the same L2 channel).
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"
#include "lp_splat_common.h"

namespace lp {

namespace {

constexpr int kWaves = 4;

template <int KIND, int C, bool CC>
__global__ __launch_bounds__(kWaves * 64) void splat_naive_kernel(GridDev tgt, RaysDev rays, SplatDev sp,
                                                                  long long group_mul)
{
    __shared__ float info_all[kWaves][32 * 16];
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* info = info_all[wave];

    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    const RaySchedule sched = ray_schedule(n_groups * kWaves, kWaves);
    const int S = rays.S;
    for (long long seq = sched.first; seq < sched.end; seq += sched.stride) {
        const long long ray = ((seq / kWaves) * group_mul % n_groups) * kWaves + seq % kWaves;
        if (ray >= rays.M) continue;
        const RayGeom q = load_ray_geom(rays, ray);
        // the pixel's feature of this lane's channel (16 channels: both halves of a lane group)
        const float v = sp.feats[(size_t)ray * C + (col & (C - 1))];
        f32x16 val;
#pragma unroll
        for (int r = 0; r < 16; ++r) val[r] = v;
        for (int j0 = 0; j0 < S; j0 += kBwdStep) {
            const int j = j0 + slot_to_sample(col);
            const Cell3 c = sample_cell<CC>(tgt, q, min(j, S - 1));
            wave_lds_fence();
            if (grp == 0) {
                float* rec = info + col * 16;
                write_scatter_record<KIND, C, true>(rec, tgt, c);
                if (j >= S) {  // a point past the end of the ray pushes nothing
#pragma unroll
                    for (int k = 0; k < (KIND == LP_GRID_TRIPLANE ? 12 : 8); ++k) rec[k] = 0.0f;
                }
            }
            wave_lds_fence();
            scatter_channels<KIND, C>(tgt, sp.theta, q.scene, info, val, col, grp);
            scatter_weights<KIND, C>(tgt, sp.theta_w, q.scene, info, col, grp);
        }
    }
}

template <int KIND, int C, bool CC>
hipError_t launch(const GridDev& tgt, const RaysDev& rays, const SplatDev& sp, int n_cu, hipStream_t stream)
{
    long long blocks = 4LL * n_cu;   // small kernel: four workgroups per compute unit
    const long long need = (rays.M + kWaves - 1) / kWaves;
    if (blocks > need) blocks = need;
    blocks = (blocks + 7) / 8 * 8;
    const long long n_groups = need;
    const long long group_mul = splat_group_multiplier(n_groups);
    hipLaunchKernelGGL((splat_naive_kernel<KIND, C, CC>), dim3((unsigned)blocks), dim3(kWaves * 64), 0, stream, tgt,
                       rays, sp, group_mul);
    return hipGetLastError();
}

template <int KIND>
hipError_t dispatch(const GridDev& tgt, const RaysDev& rays, const SplatDev& sp, int n_cu, hipStream_t stream)
{
    const bool cc = tgt.contract > 0.0;
    if (tgt.C == 16) return cc ? launch<KIND, 16, true>(tgt, rays, sp, n_cu, stream) : launch<KIND, 16, false>(tgt, rays, sp, n_cu, stream);
    if (tgt.C == 32) return cc ? launch<KIND, 32, true>(tgt, rays, sp, n_cu, stream) : launch<KIND, 32, false>(tgt, rays, sp, n_cu, stream);
    return hipErrorInvalidValue;
}

}  // namespace

bool splat_naive_supported(const GridDev& tgt)
{
    if (tgt.kind != LP_GRID_VOXEL && tgt.kind != LP_GRID_TRIPLANE && tgt.kind != LP_GRID_HASH) return false;
    if (tgt.C != 16 && tgt.C != 32) return false;
    if (tgt.kind == LP_GRID_HASH) {   // a table whose size is a power of two (`mod size` is a mask in this kernel)
        const unsigned long long T = tgt.hash_size;
        return T != 0 && (T & (T - 1)) == 0 && T * tgt.C < (1ull << 30);
    }
    const unsigned long long n0 = (unsigned long long)tgt.N[0], n1 = (unsigned long long)tgt.N[1], n2 = (unsigned long long)tgt.N[2];
    if (tgt.kind == LP_GRID_VOXEL) return n0 * n1 * n2 * tgt.C < (1ull << 30);   // 32-bit byte offsets in a scene
    return n0 * n1 * tgt.C < (1ull << 30) && n1 * n2 * tgt.C < (1ull << 30) && n2 * n0 * tgt.C < (1ull << 30);
}

hipError_t launch_splat_naive(const GridDev& tgt, const RaysDev& rays, const SplatDev& sp, int n_cu,
                              hipStream_t stream)
{
    if (tgt.kind == LP_GRID_HASH) return dispatch<LP_GRID_HASH>(tgt, rays, sp, n_cu, stream);
    return tgt.kind == LP_GRID_VOXEL ? dispatch<LP_GRID_VOXEL>(tgt, rays, sp, n_cu, stream)
                                     : dispatch<LP_GRID_TRIPLANE>(tgt, rays, sp, n_cu, stream);
}

}  // namespace lp
