// Splatter forward with an MLP on the matrix cores (Section 3.3 "Splatter": each point of a
// pixel's ray pushes g_s(pixel feature, prior structure sampled at the point, encoded
// direction) into the target structure), wavefront per ray.
//
// A step is 32 points.  The MLP runs transposed like the Renderer's (hidden layers D = W X with
// the points along N).  The pixel feature and the direction encoding are the same for every
// point of a ray, so their part of the first layer, W1[:, per-ray inputs] x, is evaluated once per
// ray and joins the bias; a step's first layer then contracts the prior's channels (gathered
// per point) only.  The last layer is taken
// with the roles swapped, V = H^T Wout^T (points along M, channels along N), which leaves lane =
// channel and registers = 16 consecutive points: the layout the run-merging scatter of the
// Renderer's backward works on, so the push shares that code.  Contract coordinates are a
// run-time branch in the point placement (uniform over the launch).
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"
#include "lp_splat_common.h"

namespace lp {

namespace {

constexpr int kWaves = 4;
constexpr int kHidden = 64;

// LDS layout in 16-byte units.  KSP K-steps of prior channels (16 each), KSE K-steps of per-ray
// inputs (pixel feature, direction encoding, zeros); element e of lane group g in K-step s is
// input 16 s + 8 g + e of its kind.
template <int KSP, int KSE, int NH>
struct SplatLds {
    static constexpr int MB = kHidden / 32, KSH = kHidden / 16;
    static constexpr int A1P = 0;                                   // W1, prior columns   [MB][KSP]
    static constexpr int A1E = A1P + MB * KSP * 128;                // W1, per-ray columns [MB][KSE]
    static constexpr int A2 = A1E + MB * KSE * 128;                 // W2   [MB][KSH]  (NH == 2)
    static constexpr int A3 = A2 + (NH == 2 ? MB * KSH * 128 : 0);  // Wout as B operand [1][KSH]
    static constexpr int BIAS = A3 + KSH * 128;                     // floats b1[64] b2[64] bout[32]
    static constexpr int WAVE = BIAS + (2 * kHidden + 32) / 4;      // per-wave areas
    // a wave's area: 32 scatter records of 16 dwords, the ray's first-layer bias, its 48 inputs
    static constexpr int W_INFO = 0, W_BIAS = 128, W_X = W_BIAS + kHidden / 4, W_UNITS = W_X + 48 / 4;
    static constexpr int UNITS = WAVE + kWaves * W_UNITS;
    static_assert(UNITS * 16 <= 64 * 1024, "static LDS of a workgroup");
};

template <int KSP, int KSE, int NH, int CO>
__device__ __forceinline__ void stage_splat_mlp(uint4* lds, const MlpDev& m, int n_in)
{
    using L = SplatLds<KSP, KSE, NH>;
    constexpr int MB = L::MB, KSH = L::KSH, CP = 16 * KSP;
    auto hidden_col = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto block_row = [](int mb, int i) { return 32 * mb + i; };
    const int n_extra = n_in + m.n_enc;
    // the caller's column order is pixel feature, prior channels, direction encoding
    stage_operand(lds + L::A1P, m.W[0], MB, KSP, m.dims[0], block_row,
                  [=](int s, int gg, int e) { return n_in + 16 * s + 8 * gg + e; });
    stage_operand(lds + L::A1E, m.W[0], MB, KSE, m.dims[0], block_row, [=](int s, int gg, int e) {
        const int x = 16 * s + 8 * gg + e;
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
    if (threadIdx.x < 32) sbias[2 * kHidden + threadIdx.x] = m.b[NH][threadIdx.x & (CO - 1)];
}

template <int KIND, int KSP, int KSE, int NH>
__global__ __launch_bounds__(kWaves * 64) void splat_mfma_kernel(GridDev tgt, MlpDev m, RaysDev rays, SplatDev sp,
                                                                 long long group_mul)
{
    constexpr int CO = 16 * KSP;  // the target has the prior's channel count
    using L = SplatLds<KSP, KSE, NH>;
    constexpr int MB = L::MB, KSH = L::KSH;
    __shared__ uint4 lds[L::UNITS];
    stage_splat_mlp<KSP, KSE, NH, CO>(lds, m, sp.n_in);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint4* wave_area = lds + L::WAVE + wave * L::W_UNITS;
    float* info = reinterpret_cast<float*>(wave_area + L::W_INFO);
    float* ray_bias = reinterpret_cast<float*>(wave_area + L::W_BIAS);
    float* ray_x = reinterpret_cast<float*>(wave_area + L::W_X);
    const float* sbias = reinterpret_cast<const float*>(lds + L::BIAS);
    const float bias_out = sbias[2 * kHidden + col];
    const int n_in = sp.n_in, n_extra = sp.n_in + m.n_enc;

    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    const RaySchedule sched = ray_schedule(n_groups * kWaves, kWaves);
    const int S = rays.S;
    for (long long seq = sched.first; seq < sched.end; seq += sched.stride) {
        const long long ray = ((seq / kWaves) * group_mul % n_groups) * kWaves + seq % kWaves;
        if (ray >= rays.M) continue;
        const RayGeom q = load_ray_geom(rays, ray);
        // ---- the ray's inputs x (pixel feature, direction encoding, zeros), one per lane, and its
        //      first-layer bias b1 + W1[:, per-ray inputs] x ----
        {
            const float d[3] = {q.dx, q.dy, q.dz};
            const float x_lane = lane < n_in ? sp.feats[(size_t)ray * n_in + lane]
                                             : lane < n_extra ? dir_encoding(d, lane - n_in) : 0.0f;
            wave_lds_fence();
            if (lane < 48) ray_x[lane] = x_lane;
            wave_lds_fence();
            f32x16 acc[MB][1];
            init_bias<MB, 1>(acc, sbias, grp);
            Frag eh[1][KSE], el[1][KSE];
#pragma unroll
            for (int s = 0; s < KSE; ++s) {
                float x[8];
                *reinterpret_cast<f32x4*>(x) = *reinterpret_cast<const f32x4*>(ray_x + 16 * s + 8 * grp);
                *reinterpret_cast<f32x4*>(x + 4) = *reinterpret_cast<const f32x4*>(ray_x + 16 * s + 8 * grp + 4);
                split8(x, eh[0][s], el[0][s]);
            }
            layer_mfma<MB, KSE, 1>(acc, lds + L::A1E, lane, eh, el);
            if (col == 0) {  // every column holds the same values
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) ray_bias[32 * mb + d_row(r, grp)] = acc[mb][0][r];
            }
            wave_lds_fence();
        }
        for (int j0 = 0; j0 < S; j0 += kBwdStep) {
            const int j = j0 + slot_to_sample(col);
            const int jj = min(j, S - 1);
            Frag fh[1][KSP], fl[1][KSP];
            {
                const Cell3 cp = sample_cell_any(sp.prior, q, jj);
#pragma unroll
                for (int s = 0; s < KSP; ++s) {
                    float feat[8];
                    gather_half<KIND, CO, 8, LP_F32>(sp.prior, q.scene, cp, 16 * s + 8 * grp, feat);
                    split8(feat, fh[0][s], fl[0][s]);
                }
            }
            const Cell3 ct = sample_cell_any(tgt, q, jj);
            wave_lds_fence();
            if (grp == 0) {
                float* rec = info + col * 16;
                write_scatter_record<KIND, CO, true>(rec, tgt, ct);
                if (j >= S) {  // a point past the end of the ray pushes nothing
#pragma unroll
                    for (int k = 0; k < (KIND == LP_GRID_VOXEL ? 8 : 12); ++k) rec[k] = 0.0f;
                }
            }
            Frag lh[1][KSH], ll[1][KSH];
            {
                f32x16 acc[MB][1];
                init_bias<MB, 1>(acc, ray_bias, grp);
                layer_mfma<MB, KSP, 1>(acc, lds + L::A1P, lane, fh, fl);
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
    if (tgt.kind != LP_GRID_VOXEL && tgt.kind != LP_GRID_TRIPLANE) return false;   // (hash tables: generic kernels)
    if (m.n_layers != 2 && m.n_layers != 3) return false;
    for (int l = 1; l < m.n_layers; ++l)
        if (m.dims[l] != kHidden) return false;
    if (!sp.has_prior || sp.prior.C != tgt.C || sp.prior.dtype != LP_F32) return false;
    if (tgt.contract != sp.prior.contract) return false;
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
