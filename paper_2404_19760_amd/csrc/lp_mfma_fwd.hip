// Matrix-core forward kernel of the Renderer (Eq. (1), Section 3.3; fused as in Section 3.4).
//
// A workgroup is 4 wavefronts sharing the MLP weights in LDS (bf16 hi/lo MFMA A operands).
// A wavefront marches ONE ray at a time, 64 consecutive samples per step: lanes (i, g) sample
// and interpolate the g-th half of the channels of samples i and 32 + i, the MLP runs on the
// matrix cores for the 64 samples (two N blocks of 32), then lane l owns sample l of the step
// for the density / colour heads and the emission-absorption update, where the transmittance
// prefix is a wave-level scan of sigma * Delta.  Nothing per sample is written to memory.
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"

namespace lp {

namespace {

constexpr int kWaves = 4;

// NB = N blocks of 32 samples per step.  NB = 2: lane l owns sample l of the 64-sample step.
// NB = 1 (half the registers, two waves per SIMD for the wide MLPs): both lane groups hold the
// decoder outputs of sample (lane & 31); group 0 alone accumulates.
template <int KIND, int C, int H, int NH, int NB, bool CC, int CG, int GT>
__global__ __launch_bounds__(kWaves * 64) void fwd_mfma_kernel(GridDev g, MlpDev m, RaysDev rays, FwdOut out)
{
    constexpr int kStep = 32 * NB;
    extern __shared__ uint4 lds[];
    stage_mlp<C, H, NH, false, NB, CG>(lds, m);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const RaySchedule sched = ray_schedule(rays.M, kWaves);
    const int S = rays.S;
    const bool identity = m.feat_act != 0;   // rendered features without the sigmoid (two-MLP decoder only)

    for (long long ray = sched.first; ray < sched.end; ray += sched.stride) {
        RayGeom q = load_ray_geom(rays, ray);
        if constexpr (CG != C) set_direction_inputs(m, q);
        float tau = 0.0f;                                              // optical depth of earlier steps
        float acc_r = 0.0f, acc_g = 0.0f, acc_b = 0.0f, acc_d = 0.0f;  // per-lane partial sums

        for (int j0 = 0; j0 < S; j0 += kStep) {
            struct { float z[4]; } a;
            if constexpr (NB == 2) {
                forward_outputs<KIND, C, H, NH, CC, CG, GT>(g, lds, q, j0, S, lane, a.z);
            } else {
                StepActs<C, H, NH, NB> full;
                forward_step<KIND, C, H, NH, false, NB, false, CC, CG, GT>(g, lds, q, j0, S, lane, full);
#pragma unroll
                for (int k = 0; k < 4; ++k) a.z[k] = full.z[k];
            }

            // heads and emission-absorption update; the lane owns sample j0 + pos
            const int pos = lane & (kStep - 1);
            const int j = j0 + pos;
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const float sd = j < S ? fast_softplus(a.z[0]) * q.delta : 0.0f;
            const float incl = group_scan_incl<kStep>(sd, pos);
            const float Tprev = __expf(-(tau + (incl - sd)));
            const float w = (NB == 2 || lane < 32) ? Tprev * one_minus_exp_neg(sd) : 0.0f;
            acc_r += w * feature_head(a.z[1], identity);
            acc_g += w * feature_head(a.z[2], identity);
            acc_b += w * feature_head(a.z[3], identity);
            acc_d += w * t;
            tau += __shfl(incl, kStep - 1, kStep);
        }

        acc_r = wave_sum(acc_r);
        acc_g = wave_sum(acc_g);
        acc_b = wave_sum(acc_b);
        acc_d = wave_sum(acc_d);
        if (lane == 0) {
            const float T = __expf(-tau);
            out.rgb[3 * ray + 0] = acc_r + T * out.bg[0];
            out.rgb[3 * ray + 1] = acc_g + T * out.bg[1];
            out.rgb[3 * ray + 2] = acc_b + T * out.bg[2];
            if (out.alpha) out.alpha[ray] = one_minus_exp_neg(tau);
            if (out.depth) out.depth[ray] = acc_d;
            if (out.cache) out.cache[ray] = tau;
        }
    }
}

template <int KIND, int C, int H, int NH, int NB, bool CC, int CG, int GT = LP_F32>
hipError_t launch_fwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                      hipStream_t stream)
{
    constexpr int kLdsBytes = MlpLds<C, H, NH, false, NB>::bytes(kWaves);
    auto kernel = fwd_mfma_kernel<KIND, C, H, NH, NB, CC, CG, GT>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    // persistent grid: as many workgroups as fit a compute unit's registers, a multiple of the 8 XCDs, no more than the rays need
    long long blocks = 3LL * n_cu;
    const long long need = (rays.M + kWaves - 1) / kWaves;
    if (blocks > need) blocks = need;
    blocks = (blocks + 7) / 8 * 8;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, m, rays, out);
    return hipGetLastError();
}

template <int KIND>
hipError_t dispatch_fwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                        hipStream_t stream)
{
    const int C = m.dims[0], CG = g.C, H = m.dims[1], NH = m.n_layers - 1;
    // grids stored in bf16 / fp16: plain inputs; the contraction is a run-time branch of these kernels
#define LP_CASE(c, h, nh)                                                                                     \
    if (C == c && CG == c && H == h && NH == nh && g.dtype != LP_F32)                  \
        return g.dtype == LP_BF16 ? launch_fwd<KIND, c, h, nh, 2, false, c, LP_BF16>(g, m, rays, out, n_cu, stream) \
                                  : launch_fwd<KIND, c, h, nh, 2, false, c, LP_F16>(g, m, rays, out, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    if (g.dtype != LP_F32 && CG == C) return hipErrorInvalidValue;   // (the decoder kernels read any storage type)
#define LP_CASE(c, cg, h, nh)                                                                          \
    if (C == c && CG == cg && H == h && NH == nh)                                                      \
        return g.contract > 0.0 ? launch_fwd<KIND, c, h, nh, 2, true, cg>(g, m, rays, out, n_cu, stream) \
                                : launch_fwd<KIND, c, h, nh, 2, false, cg>(g, m, rays, out, n_cu, stream);
    LP_CASE(16, 16, 32, 1) LP_CASE(16, 16, 64, 1) LP_CASE(32, 32, 32, 1) LP_CASE(32, 32, 64, 1)
    LP_CASE(16, 16, 32, 2) LP_CASE(16, 16, 64, 2) LP_CASE(32, 32, 32, 2) LP_CASE(32, 32, 64, 2)
#undef LP_CASE
    // 16 grid channels + direction inputs (the two-MLP decoder merged into one MLP of 32 inputs)
#define LP_CASE(h, nh)                                                                                  \
    if (C == 32 && CG == 16 && H == h && NH == nh)                                                      \
        return g.contract > 0.0 ? launch_fwd<KIND, 32, h, nh, 2, true, 16, kAnyDtype>(g, m, rays, out, n_cu, stream) \
                                : launch_fwd<KIND, 32, h, nh, 2, false, 16, kAnyDtype>(g, m, rays, out, n_cu, stream);
    LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2) LP_CASE(64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

// hash tables: the storage type and the contraction are run-time branches of one set of kernels
hipError_t dispatch_fwd_hash(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                             hipStream_t stream)
{
    const int C = m.dims[0], H = m.dims[1], NH = m.n_layers - 1;
#define LP_CASE(c, h, nh)                         \
    if (C == c && g.C == c && H == h && NH == nh) \
        return launch_fwd<LP_GRID_HASH, c, h, nh, 2, false, c, kAnyDtype>(g, m, rays, out, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    // 16 table channels + direction inputs (the two-MLP decoder merged into one MLP of 32 inputs)
#define LP_CASE(h, nh)                             \
    if (C == 32 && g.C == 16 && H == h && NH == nh) \
        return launch_fwd<LP_GRID_HASH, 32, h, nh, 2, false, 16, kAnyDtype>(g, m, rays, out, n_cu, stream);
    LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2) LP_CASE(64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

// HexPlanes: likewise one set of kernels
hipError_t dispatch_fwd_hexplane(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                                 hipStream_t stream)
{
    const int C = m.dims[0], H = m.dims[1], NH = m.n_layers - 1;
#define LP_CASE(c, h, nh)                         \
    if (C == c && g.C == c && H == h && NH == nh) \
        return launch_fwd<LP_GRID_HEXPLANE, c, h, nh, 2, false, c, kAnyDtype>(g, m, rays, out, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    // 16 plane channels + direction inputs (the two-MLP decoder merged into one MLP of 32 inputs)
#define LP_CASE(h, nh)                             \
    if (C == 32 && g.C == 16 && H == h && NH == nh) \
        return launch_fwd<LP_GRID_HEXPLANE, 32, h, nh, 2, false, 16, kAnyDtype>(g, m, rays, out, n_cu, stream);
    LP_CASE(32, 1) LP_CASE(64, 1) LP_CASE(32, 2) LP_CASE(64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace

bool mfma_supported(const GridDev& g, const MlpDev& m)
{
    if (g.kind != LP_GRID_VOXEL && g.kind != LP_GRID_TRIPLANE && g.kind != LP_GRID_HASH && g.kind != LP_GRID_HEXPLANE)
        return false;
    // inputs: all of them grid channels (16 or 32), or 16 grid channels + 16 direction inputs
    const bool plain = m.n_enc == 0 && m.dims[0] == g.C && (g.C == 16 || g.C == 32);
    const bool with_dir = m.n_enc > 0 && g.C == 16 && m.dims[0] == 32 && m.n_enc <= 16;
    if (!plain && !with_dir) return false;
        if (m.n_feat != 3 || m.dims[m.n_layers] != 4) return false;
    if (m.n_layers != 2 && m.n_layers != 3) return false;
    const int H = m.dims[1];
    if (H != 32 && H != 64) return false;
    if (m.n_layers == 3 && m.dims[2] != H) return false;
    // 32-bit byte offsets inside one scene's tensor (below 4 GiB), 16-byte aligned tensors
    const unsigned long long n0 = (unsigned long long)g.N[0], n1 = (unsigned long long)g.N[1], n2 = (unsigned long long)g.N[2];
    const unsigned long long per_scene = n0 * n1 * n2 * g.C;  // voxel tensor of one scene
    if (g.kind == LP_GRID_VOXEL) {
        if (per_scene >= (1ull << 30)) return false;
        if ((uintptr_t)g.data[0] & 15u) return false;
    } else if (g.kind == LP_GRID_HASH) {
        // a table whose size is a power of two (`mod size` is a mask in these kernels)
        const unsigned long long T = (unsigned long long)g.hash_size;
        if (T == 0 || (T & (T - 1)) != 0 || T * g.C >= (1ull << 30)) return false;
        if ((uintptr_t)g.data[0] & 15u) return false;
    } else {
        if (n0 * n1 * g.C >= (1ull << 30) || n1 * n2 * g.C >= (1ull << 30) || n2 * n0 * g.C >= (1ull << 30)) return false;
        for (int p = 0; p < 3; ++p)
            if ((uintptr_t)g.data[p] & 15u) return false;
        if (g.kind == LP_GRID_HEXPLANE) {   // the space-time planes under the same limits
            const unsigned long long nt = (unsigned long long)g.NT;
            if (n0 * nt * g.C >= (1ull << 30) || n1 * nt * g.C >= (1ull << 30) || n2 * nt * g.C >= (1ull << 30))
                return false;
            for (int p = 0; p < 3; ++p)
                if ((uintptr_t)g.data_t[p] & 15u) return false;
        }
    }
    return true;
}

hipError_t launch_fwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                           hipStream_t stream)
{
    if (g.kind == LP_GRID_HASH) return dispatch_fwd_hash(g, m, rays, out, n_cu, stream);
    if (g.kind == LP_GRID_HEXPLANE) return dispatch_fwd_hexplane(g, m, rays, out, n_cu, stream);
    return g.kind == LP_GRID_VOXEL ? dispatch_fwd<LP_GRID_VOXEL>(g, m, rays, out, n_cu, stream)
                                   : dispatch_fwd<LP_GRID_TRIPLANE>(g, m, rays, out, n_cu, stream);
}

}  // namespace lp
