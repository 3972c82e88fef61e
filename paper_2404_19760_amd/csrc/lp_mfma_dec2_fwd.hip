// Forward of the Renderer with the paper's two-MLP decoder at its experimental size (see
// lp_mfma_dec2.h): the forward kernel of the single-MLP path with two MLP chains per step.
#include "lp_mfma_dec2.h"

namespace lp {

namespace {

using namespace dec2;

template <int KIND, int C, bool CC>
__global__ __launch_bounds__(kWaves * 64) void dec2_fwd_kernel(GridDev g, Dec2Dev d, RaysDev rays, FwdOut out)
{
    using L = Lds<C, false, 2>;
    constexpr int kStep = 64, KS1 = C / 16;
    extern __shared__ uint4 lds[];
    stage_decoder<C, false, 2>(lds, d);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const float* bias_s = reinterpret_cast<const float*>(lds + L::S + L::Chain::BIAS);
    const float* bias_v = reinterpret_cast<const float*>(lds + L::WAVE + wave * L::W_UNITS + L::W_BIAS);
    const RaySchedule sched = ray_schedule(rays.M, kWaves);
    const int S = rays.S;

    for (long long ray = sched.first; ray < sched.end; ray += sched.stride) {
        const RayGeom q = load_ray_geom(rays, ray);
        ray_direction_bias<C, false, 2>(lds, d, q, lane, wave);
        float tau = 0.0f;                                              // optical depth of earlier steps
        float acc_r = 0.0f, acc_g = 0.0f, acc_b = 0.0f, acc_d = 0.0f;  // per-lane partial sums

        for (int j0 = 0; j0 < S; j0 += kStep) {
            Frag fh[2][KS1], fl[2][KS1];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const Cell3 c = sample_cell<CC>(g, q, min(j0 + 32 * nb + col, S - 1));
                sample_features<KIND, C, C, kAnyDtype>(g, q, c, grp, fh[nb], fl[nb]);
            }
            // the chains' outputs occupy different rows (opacity: 0, features: 1..3)
            float zs[4], zv[4];
            mlp_outputs<C, kH, 2>(lds + L::S, bias_s, lane, fh, fl, zs);
            __builtin_amdgcn_sched_barrier(0);
            mlp_outputs<C, kH, 2>(lds + L::V, bias_v, lane, fh, fl, zv);

            // heads and emission-absorption update; the lane owns sample j0 + lane
            const int j = j0 + lane;
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const float sd = j < S ? fast_softplus(zs[0]) * q.delta : 0.0f;
            const float incl = group_scan_incl<kStep>(sd, lane);
            const float Tprev = __expf(-(tau + (incl - sd)));
            const float w = Tprev * one_minus_exp_neg(sd);
            acc_r += w * feature_head(zv[1], d.feat_act != 0);
            acc_g += w * feature_head(zv[2], d.feat_act != 0);
            acc_b += w * feature_head(zv[3], d.feat_act != 0);
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

template <int KIND, int C, bool CC>
hipError_t launch(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const FwdOut& out, int n_cu,
                  hipStream_t stream)
{
    constexpr int kLdsBytes = Lds<C, false, 2>::END * 16;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    auto kernel = dec2_fwd_kernel<KIND, C, CC>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    long long blocks = 2LL * n_cu;
    const long long need = (rays.M + kWaves - 1) / kWaves;
    if (blocks > need) blocks = need;
    blocks = (blocks + 7) / 8 * 8;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, d, rays, out);
    return hipGetLastError();
}

template <int KIND>
hipError_t dispatch(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const FwdOut& out, int n_cu,
                    hipStream_t stream)
{
    const bool cc = g.contract > 0.0;
    if (g.C == 16) return cc ? launch<KIND, 16, true>(g, d, rays, out, n_cu, stream) : launch<KIND, 16, false>(g, d, rays, out, n_cu, stream);
    if (g.C == 32) return cc ? launch<KIND, 32, true>(g, d, rays, out, n_cu, stream) : launch<KIND, 32, false>(g, d, rays, out, n_cu, stream);
    return hipErrorInvalidValue;
}

}  // namespace

bool dec2_supported(const GridDev& g, const DecLayout& d, int n_feat, int feat_act)
{
    if (g.kind != LP_GRID_VOXEL && g.kind != LP_GRID_TRIPLANE) return false;
    if (g.C != 16 && g.C != 32) return false;
    if (n_feat != 3 || (feat_act != 0 && feat_act != 1)) return false;
    if (d.Ls != 3 || d.Lv != 3 || d.E > dec2::kMaxDir) return false;
    if (d.dims_s[0] != g.C || d.dims_s[1] != kH || d.dims_s[2] != kH || d.dims_s[3] != 1) return false;
    if (d.dims_v[0] != g.C + d.E || d.dims_v[1] != kH || d.dims_v[2] != kH || d.dims_v[3] != 3) return false;
    // 32-bit byte offsets inside one scene's tensor, 16-byte aligned tensors (as the single-MLP kernels)
    const unsigned long long n0 = (unsigned long long)g.N[0], n1 = (unsigned long long)g.N[1], n2 = (unsigned long long)g.N[2];
    if (g.kind == LP_GRID_VOXEL) {
        if (n0 * n1 * n2 * g.C >= (1ull << 30) || ((uintptr_t)g.data[0] & 15u)) return false;
    } else {
        if (n0 * n1 * g.C >= (1ull << 30) || n1 * n2 * g.C >= (1ull << 30) || n2 * n0 * g.C >= (1ull << 30)) return false;
        for (int p = 0; p < 3; ++p)
            if ((uintptr_t)g.data[p] & 15u) return false;
    }
    return true;
}

Dec2Dev dec2_view(const DecLayout& d, int feat_act)
{
    Dec2Dev v;
    for (int l = 0; l < 3; ++l) {
        v.Ws[l] = d.Ws[l]; v.bs[l] = d.bs[l];
        v.Wv[l] = d.Wv[l]; v.bv[l] = d.bv[l];
        v.dWs[l] = d.dWs[l]; v.dbs[l] = d.dbs[l];
        v.dWv[l] = d.dWv[l]; v.dbv[l] = d.dbv[l];
    }
    v.E = d.E;
    v.feat_act = feat_act;
    return v;
}

hipError_t launch_dec2_fwd(const GridDev& g, const Dec2Dev& d, const RaysDev& rays, const FwdOut& out, int n_cu,
                           hipStream_t stream)
{
    return g.kind == LP_GRID_VOXEL ? dispatch<LP_GRID_VOXEL>(g, d, rays, out, n_cu, stream)
                                   : dispatch<LP_GRID_TRIPLANE>(g, d, rays, out, n_cu, stream);
}

}  // namespace lp
