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

namespace lp {

namespace {

constexpr int kWaves = 4;

template <int C, int H, int NH>
struct FwdLds {
    static constexpr int MB = H / 32;   // 32-row blocks of a hidden layer's outputs
    static constexpr int KS1 = C / 16;  // K-steps over the input channels
    static constexpr int KSH = H / 16;  // K-steps over a hidden layer's outputs
    // offsets in uint4 (16 B) units; each (block, K-step) is 64 hi + 64 lo entries
    static constexpr int A1 = 0;
    static constexpr int A2 = A1 + MB * KS1 * 128;
    static constexpr int A3 = A2 + (NH == 2 ? MB * KSH * 128 : 0);
    static constexpr int BIAS = A3 + KSH * 128;           // floats: b1[H] b2[H] b3[4]
    static constexpr int BYTES = BIAS * 16 + (2 * H + 4) * 4;
};

// relu + split of the D registers of one layer into the next layer's B operands
template <int MB>
__device__ __forceinline__ void activate(const f32x16 (&acc)[MB][2], Frag (&bh)[2][2 * MB], Frag (&bl)[2][2 * MB])
{
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int s = 0; s < 2 * MB; ++s) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaxf(acc[s / 2][nb][8 * (s % 2) + e], 0.0f);
            split8(v, bh[nb][s], bl[nb][s]);
        }
}

template <int KIND, int C, int H, int NH>
__global__ __launch_bounds__(kWaves * 64) void fwd_mfma_kernel(GridDev g, MlpDev m, RaysDev rays, FwdOut out)
{
    using L = FwdLds<C, H, NH>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    extern __shared__ uint4 lds[];
    float* sbias = reinterpret_cast<float*>(lds + L::BIAS);

    // ---- stage the weights as MFMA A operands (once per workgroup) ----
    stage_operand(lds + L::A1, m.W[0], MB, KS1, C,
                  [](int mb, int i) { return 32 * mb + i; },
                  [](int s, int gg, int e) { return k_input<C>(s, gg, e); });
    if constexpr (NH == 2)
        stage_operand(lds + L::A2, m.W[1], MB, KSH, H,
                      [](int mb, int i) { return 32 * mb + i; },
                      [](int s, int gg, int e) { return k_hidden(s, gg, e); });
    // last layer: rows 0..3 and 4..7 both carry the 4 outputs, so that both lane groups of a
    // column hold them (D rows 4g + p)
    stage_operand(lds + L::A3, m.W[NH], 1, KSH, H,
                  [](int, int i) { return i < 8 ? (i & 3) : -1; },
                  [](int s, int gg, int e) { return k_hidden(s, gg, e); });
    for (int i = threadIdx.x; i < H; i += blockDim.x) {
        sbias[i] = m.b[0][i];
        sbias[H + i] = NH == 2 ? m.b[1][i] : 0.0f;
    }
    if (threadIdx.x < 4) sbias[2 * H + threadIdx.x] = m.b[NH][threadIdx.x];
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const RaySchedule sched = ray_schedule(rays.M, kWaves);
    const int S = rays.S;

    for (long long ray = sched.first; ray < sched.end; ray += sched.stride) {
        const float ox = rays.origins[3 * ray + 0], oy = rays.origins[3 * ray + 1], oz = rays.origins[3 * ray + 2];
        const float dx = rays.dirs[3 * ray + 0], dy = rays.dirs[3 * ray + 1], dz = rays.dirs[3 * ray + 2];
        const float near = rays.near[ray];
        const float delta = (rays.far[ray] - near) / (float)S;
        const int scene = rays.scene ? rays.scene[ray] : 0;

        float tau = 0.0f;                       // optical depth of all earlier steps (wave-uniform)
        float acc_r = 0.0f, acc_g = 0.0f, acc_b = 0.0f, acc_d = 0.0f;  // per-lane partial sums

        for (int j0 = 0; j0 < S; j0 += 64) {
            // ---- sample + interpolate: B operands of layer 1 ----
            Frag bh1[2][KS1], bl1[2][KS1];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int j = min(j0 + 32 * nb + col, S - 1);
                const float t = near + ((float)j + 0.5f) * delta;
                const Cell3 c = locate3(g, ox + t * dx, oy + t * dy, oz + t * dz);
                float feat[C / 2];
                gather_half<KIND, C, C / 2>(g, scene, c, grp * (C / 2), feat);
#pragma unroll
                for (int s = 0; s < KS1; ++s) split8(feat + 8 * s, bh1[nb][s], bl1[nb][s]);
            }

            // ---- layer 1 ----
            f32x16 acc[MB][2];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 b = *reinterpret_cast<const f32x4*>(sbias + 32 * mb + 8 * q + 4 * grp);
#pragma unroll
                    for (int p = 0; p < 4; ++p) acc[mb][0][4 * q + p] = acc[mb][1][4 * q + p] = b[p];
                }
#pragma unroll
                for (int s = 0; s < KS1; ++s) {
                    Frag ah, al;
                    load_operand(lds + L::A1 + (mb * KS1 + s) * 128, lane, ah, al);
                    acc[mb][0] = mfma3(ah, al, bh1[0][s], bl1[0][s], acc[mb][0]);
                    acc[mb][1] = mfma3(ah, al, bh1[1][s], bl1[1][s], acc[mb][1]);
                }
            }
            Frag bh[2][KSH], bl[2][KSH];
            activate<MB>(acc, bh, bl);

            // ---- layer 2 (second hidden layer) ----
            if constexpr (NH == 2) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 b = *reinterpret_cast<const f32x4*>(sbias + H + 32 * mb + 8 * q + 4 * grp);
#pragma unroll
                        for (int p = 0; p < 4; ++p) acc[mb][0][4 * q + p] = acc[mb][1][4 * q + p] = b[p];
                    }
#pragma unroll
                    for (int s = 0; s < KSH; ++s) {
                        Frag ah, al;
                        load_operand(lds + L::A2 + (mb * KSH + s) * 128, lane, ah, al);
                        acc[mb][0] = mfma3(ah, al, bh[0][s], bl[0][s], acc[mb][0]);
                        acc[mb][1] = mfma3(ah, al, bh[1][s], bl[1][s], acc[mb][1]);
                    }
                }
                activate<MB>(acc, bh, bl);
            }

            // ---- output layer: 4 rows, replicated for both lane groups ----
            f32x16 o0, o1;
            {
                const f32x4 b = *reinterpret_cast<const f32x4*>(sbias + 2 * H);
#pragma unroll
                for (int r = 0; r < 16; ++r) o0[r] = o1[r] = r < 4 ? b[r] : 0.0f;
#pragma unroll
                for (int s = 0; s < KSH; ++s) {
                    Frag ah, al;
                    load_operand(lds + L::A3 + s * 128, lane, ah, al);
                    o0 = mfma3(ah, al, bh[0][s], bl[0][s], o0);
                    o1 = mfma3(ah, al, bh[1][s], bl[1][s], o1);
                }
            }
            // lane l now owns sample j0 + l: lanes 0..31 from N block 0, lanes 32..63 from block 1
            const float z0 = grp ? o1[0] : o0[0];
            const float z1 = grp ? o1[1] : o0[1];
            const float z2 = grp ? o1[2] : o0[2];
            const float z3 = grp ? o1[3] : o0[3];

            // ---- heads and emission-absorption update ----
            const int j = j0 + lane;
            const float t = near + ((float)j + 0.5f) * delta;
            const float sd = j < S ? fast_softplus(z0) * delta : 0.0f;
            const float incl = wave_scan_incl(sd, lane);
            const float Tprev = __expf(-(tau + (incl - sd)));
            const float w = Tprev * one_minus_exp_neg(sd);
            acc_r += w * fast_logistic(z1);
            acc_g += w * fast_logistic(z2);
            acc_b += w * fast_logistic(z3);
            acc_d += w * t;
            tau += __shfl(incl, 63, 64);
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

template <int KIND, int C, int H, int NH>
hipError_t launch_fwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                      hipStream_t stream)
{
    using L = FwdLds<C, H, NH>;
    auto kernel = fwd_mfma_kernel<KIND, C, H, NH>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, L::BYTES);
    if (e != hipSuccess) return e;
    // persistent grid: two workgroups per compute unit, a multiple of the 8 XCDs, no more than the rays need
    long long blocks = 2LL * n_cu;
    const long long need = (rays.M + kWaves - 1) / kWaves;
    if (blocks > need) blocks = need;
    blocks = (blocks + 7) / 8 * 8;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), L::BYTES, stream, g, m, rays, out);
    return hipGetLastError();
}

template <int KIND>
hipError_t dispatch_fwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                        hipStream_t stream)
{
    const int C = g.C, H = m.dims[1], NH = m.n_layers - 1;
#define LP_CASE(c, h, nh) \
    if (C == c && H == h && NH == nh) return launch_fwd<KIND, c, h, nh>(g, m, rays, out, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace

bool mfma_supported(const GridDev& g, const MlpDev& m)
{
    if (g.C != 16 && g.C != 32) return false;
    if (m.n_layers != 2 && m.n_layers != 3) return false;
    const int H = m.dims[1];
    if (H != 32 && H != 64) return false;
    if (m.n_layers == 3 && m.dims[2] != H) return false;
    // 32-bit element offsets inside one scene's tensor, 16-byte aligned tensors
    const unsigned long long n0 = (unsigned long long)g.N[0], n1 = (unsigned long long)g.N[1], n2 = (unsigned long long)g.N[2];
    const unsigned long long per_scene = n0 * n1 * n2 * g.C;  // voxel tensor of one scene
    if (g.kind == LP_GRID_VOXEL) {
        if (per_scene >= (1ull << 31)) return false;
        if ((uintptr_t)g.data[0] & 15u) return false;
    } else {
        if (n0 * n1 * g.C >= (1ull << 31) || n1 * n2 * g.C >= (1ull << 31) || n2 * n0 * g.C >= (1ull << 31)) return false;
        for (int p = 0; p < 3; ++p)
            if ((uintptr_t)g.data[p] & 15u) return false;
    }
    return true;
}

hipError_t launch_fwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const FwdOut& out, int n_cu,
                           hipStream_t stream)
{
    return g.kind == LP_GRID_VOXEL ? dispatch_fwd<LP_GRID_VOXEL>(g, m, rays, out, n_cu, stream)
                                   : dispatch_fwd<LP_GRID_TRIPLANE>(g, m, rays, out, n_cu, stream);
}

}  // namespace lp
