// Splatter forward with an MLP on the matrix cores (Section 3.3 "Splatter": each point of a
// pixel's ray pushes g_s(pixel feature, prior structure sampled at the point, encoded
// direction) into the target structure), wavefront per ray.
//
// A step is 32 points.  The MLP runs transposed like the Renderer's (hidden layers D = W X with
// the points along N); its inputs are ordered for the kernel: first the prior's channels
// (gathered per point), then the per-ray inputs (pixel feature, direction encoding, zeros up to
// a multiple of 16), whose operand fragments are built once per ray.  The last layer is taken
// with the roles swapped, V = H^T Wout^T (points along M, channels along N), which leaves lane =
// channel and registers = 16 consecutive points: the layout the run-merging scatter of the
// Renderer's backward works on, so the push shares that code.
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"
#include "lp_splat_common.h"

namespace lp {

namespace {

constexpr int kWaves = 4;
constexpr int kHidden = 64;

// KSP K-steps of prior channels (16 each), KSE K-steps of per-ray inputs
template <int KSP, int KSE, int NH>
struct SplatLds {
    using W = MlpLds<16 * (KSP + KSE), kHidden, NH, false, 1>;
    static constexpr int BIAS_OUT = W::END;            // 32 floats
    static constexpr int INFO = BIAS_OUT + 8;          // per wave 32 records of 16 dwords
    static constexpr int UNITS = INFO + kWaves * 128;
};

template <int KSP, int KSE, int NH, int CO>
__device__ __forceinline__ void stage_splat_mlp(uint4* lds, const MlpDev& m, int n_in)
{
    using S = SplatLds<KSP, KSE, NH>;
    using L = typename S::W;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH, CP = 16 * KSP;
    auto hidden_col = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto block_row = [](int mb, int i) { return 32 * mb + i; };
    const int n_extra = n_in + m.n_enc;
    // kernel input (s, g, e) -> column of the first layer: the caller's order is pixel feature,
    // prior channels, direction encoding
    stage_operand(lds + L::A1, m.W[0], MB, KS1, m.dims[0], block_row, [=](int s, int gg, int e) {
        if (s < KSP) return n_in + 16 * s + 8 * gg + e;
        const int x = 16 * (s - KSP) + 8 * gg + e;
        return x < n_in ? x : x < n_extra ? CP + x : -1;
    });
    if constexpr (NH == 2) stage_operand(lds + L::A2, m.W[1], MB, KSH, kHidden, block_row, hidden_col);
    // last layer as the B operand of the swapped product: "row" i = output channel (16 channels:
    // a second copy in rows 16..31, both halves of a lane group scatter)
    stage_operand(lds + L::A3, m.W[NH], 1, KSH, kHidden, [](int, int i) { return i & (CO - 1); }, hidden_col);
    float* sbias = reinterpret_cast<float*>(lds + L::BIAS);
    for (int i = threadIdx.x; i < kHidden; i += blockDim.x) {
        sbias[i] = m.b[0][i];
        sbias[kHidden + i] = NH == 2 ? m.b[1][i] : 0.0f;
    }
    float* bias_out = reinterpret_cast<float*>(lds + S::BIAS_OUT);
    if (threadIdx.x < 32) bias_out[threadIdx.x] = m.b[NH][threadIdx.x & (CO - 1)];
}

template <int KIND, int KSP, int KSE, int NH>
__global__ __launch_bounds__(kWaves * 64) void splat_mfma_kernel(GridDev tgt, MlpDev m, RaysDev rays,
                                                                    SplatDev sp, long long group_mul)
{
    constexpr int CO = 16 * KSP;  // the target has the prior's channel count
    using SL = SplatLds<KSP, KSE, NH>;
    using L = typename SL::W;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    __shared__ uint4 lds[SL::UNITS];
    stage_splat_mlp<KSP, KSE, NH, CO>(lds, m, sp.n_in);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* info = reinterpret_cast<float*>(lds + SL::INFO + wave * 128);
    const float* sbias = reinterpret_cast<const float*>(lds + L::BIAS);
    const float bias_out = reinterpret_cast<const float*>(lds + SL::BIAS_OUT)[col];
    const int n_in = sp.n_in, n_extra = sp.n_in + m.n_enc;

    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    const RaySchedule sched = ray_schedule(n_groups * kWaves, kWaves);
    const int S = rays.S;
    for (long long seq = sched.first; seq < sched.end; seq += sched.stride) {
        const long long ray = ((seq / kWaves) * group_mul % n_groups) * kWaves + seq % kWaves;
        if (ray >= rays.M) continue;
        const RayGeom q = load_ray_geom(rays, ray);
        // per-ray inputs as operand fragments: element e of K-step s is input 16 s + 8 grp + e
        Frag eh[KSE], el[KSE];
        {
            const float d[3] = {q.dx, q.dy, q.dz};
#pragma unroll
            for (int s = 0; s < KSE; ++s) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int k = 16 * s + 8 * grp + e;
                    x[e] = k < n_in ? sp.feats[(size_t)ray * n_in + k] : k < n_extra ? dir_encoding(d, k - n_in) : 0.0f;
                }
                split8(x, eh[s], el[s]);
            }
        }
        for (int j0 = 0; j0 < S; j0 += kBwdStep) {
            const int j = j0 + slot_to_sample(col);
            const int jj = min(j, S - 1);
            Frag fh[1][KS1], fl[1][KS1];
            {
                const Cell3 cp = sample_cell<false>(sp.prior, q, jj);
#pragma unroll
                for (int s = 0; s < KSP; ++s) {
                    float feat[8];
                    gather_half<KIND, CO, 8, LP_F32>(sp.prior, q.scene, cp, 16 * s + 8 * grp, feat);
                    split8(feat, fh[0][s], fl[0][s]);
                }
#pragma unroll
                for (int s = 0; s < KSE; ++s) { fh[0][KSP + s] = eh[s]; fl[0][KSP + s] = el[s]; }
            }
            const Cell3 ct = sample_cell<false>(tgt, q, jj);
            wave_lds_fence();
            if (grp == 0) {
                float* rec = info + col * 16;
                write_scatter_record<KIND, CO>(rec, tgt, ct);
                if (j >= S) {  // a point past the end of the ray pushes nothing
#pragma unroll
                    for (int k = 0; k < (KIND == LP_GRID_VOXEL ? 8 : 12); ++k) rec[k] = 0.0f;
                }
            }
            Frag lh[1][KSH], ll[1][KSH];
            {
                f32x16 acc[MB][1];
                init_bias<MB, 1>(acc, sbias, grp);
                layer_mfma<MB, KS1, 1>(acc, lds + L::A1, lane, fh, fl);
                to_operands<MB, true, 1>(acc, lh, ll);
                if constexpr (NH == 2) {
                    init_bias<MB, 1>(acc, sbias + kHidden, grp);
                    layer_mfma<MB, KSH, 1>(acc, lds + L::A2, lane, lh, ll);
                    to_operands<MB, true, 1>(acc, lh, ll);
                }
            }
            // V[point][channel]: the hidden activations are the A operand as they stand
            f32x16 v;
#pragma unroll
            for (int r = 0; r < 16; ++r) v[r] = bias_out;
#pragma unroll
            for (int s = 0; s < KSH; ++s) {
                Frag wh, wl;
                load_operand(lds + L::A3 + s * 128, lane, wh, wl);
                v = mfma3(lh[0][s], ll[0][s], wh, wl, v);
            }
            wave_lds_fence();
            scatter_channels<KIND, CO>(tgt, sp.theta, q.scene, info, v, col, grp);
            scatter_weights<KIND, CO>(tgt, sp.theta_w, q.scene, info, col, grp);
        }
    }
}

template <int KIND, int KSP, int KSE, int NH>
hipError_t launch(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, int n_cu,
                  hipStream_t stream)
{
    long long blocks = 2LL * n_cu;
    const long long need = (rays.M + kWaves - 1) / kWaves;
    if (blocks > need) blocks = need;
    blocks = (blocks + 7) / 8 * 8;
    hipLaunchKernelGGL((splat_mfma_kernel<KIND, KSP, KSE, NH>), dim3((unsigned)blocks), dim3(kWaves * 64), 0, stream,
                       tgt, m, rays, sp, splat_group_multiplier(need));
    return hipGetLastError();
}

template <int KIND, int KSP, int KSE>
hipError_t by_layers(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, int n_cu,
                     hipStream_t stream)
{
    return m.n_layers == 2 ? launch<KIND, KSP, KSE, 1>(tgt, m, rays, sp, n_cu, stream)
                           : launch<KIND, KSP, KSE, 2>(tgt, m, rays, sp, n_cu, stream);
}

template <int KIND, int KSP>
hipError_t by_extras(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, int n_cu,
                     hipStream_t stream)
{
    const int n_extra = sp.n_in + m.n_enc;
    if (n_extra <= 16) return by_layers<KIND, KSP, 1>(tgt, m, rays, sp, n_cu, stream);
    if (n_extra <= 32) return by_layers<KIND, KSP, 2>(tgt, m, rays, sp, n_cu, stream);
    return by_layers<KIND, KSP, 3>(tgt, m, rays, sp, n_cu, stream);
}

template <int KIND>
hipError_t by_channels(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, int n_cu,
                       hipStream_t stream)
{
    return tgt.C == 16 ? by_extras<KIND, 1>(tgt, m, rays, sp, n_cu, stream)
                       : by_extras<KIND, 2>(tgt, m, rays, sp, n_cu, stream);
}

}  // namespace

bool splat_mfma_supported(const GridDev& tgt, const MlpDev& m, const SplatDev& sp)
{
    if (m.n_layers != 2 && m.n_layers != 3) return false;
    for (int l = 1; l < m.n_layers; ++l)
        if (m.dims[l] != kHidden) return false;
    if (!sp.has_prior || sp.prior.C != tgt.C || sp.prior.dtype != LP_F32) return false;
    if (tgt.contract > 0.0 || sp.prior.contract > 0.0) return false;
    if (sp.n_in + m.n_enc > 48) return false;
    return splat_naive_supported(tgt) && splat_naive_supported(sp.prior);
}

hipError_t launch_splat_mfma(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp,
                             int n_cu, hipStream_t stream)
{
    return tgt.kind == LP_GRID_VOXEL ? by_channels<LP_GRID_VOXEL>(tgt, m, rays, sp, n_cu, stream)
                                     : by_channels<LP_GRID_TRIPLANE>(tgt, m, rays, sp, n_cu, stream);
}

}  // namespace lp
