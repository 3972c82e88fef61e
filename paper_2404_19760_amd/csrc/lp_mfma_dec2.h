// The paper's decoder at the size of its experiments on the matrix cores (Section 3.3: an
// opacity MLP on the grid features and a feature MLP on the grid features and the encoded view
// direction; appendix "Experimental Details": 3-layer MLPs of width 64).
//
// Merged into one block-structured MLP the two would be 128 wide, beyond what a wavefront's
// registers hold.  Here they stay two chains of the single-MLP shape (C inputs, two hidden
// layers of 64) that share the sampled features: the opacity chain's single output sits in row
// 0 of its last layer, the feature chain's three outputs in rows 1..3, so the outputs of the
// two chains add up to the (density, features) vector the compositing code expects.  The view
// direction is the same for every sample of a ray: W1[:, direction inputs] enc(d) is evaluated
// once per ray and joins the feature chain's first-layer bias.
#pragma once
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"

namespace lp {

namespace dec2 {

constexpr int kWaves = 4;
constexpr int kH = 64;

constexpr int kMaxDir = 32;   // direction inputs (two K-steps); four octaves need 27

// LDS layout in 16-byte units: the two chains in the single-MLP layout, the feature chain's
// direction columns of the first layer, then per wave the ray's feature-chain bias (64 floats)
// and its encoded direction (32 floats).
template <int C, bool BWD, int NB>
struct Lds {
    using Chain = MlpLds<C, kH, 2, BWD, NB>;
    static constexpr int KSE = kMaxDir / 16;
    static constexpr int S = 0;                       // opacity chain
    static constexpr int V = Chain::END;              // feature chain
    static constexpr int A1E = V + Chain::END;        // W1 of the feature chain, direction columns [2][KSE]
    static constexpr int WAVE = A1E + 2 * KSE * 128;
    static constexpr int W_BIAS = 0, W_X = kH / 4, W_UNITS = W_X + kMaxDir / 4;
    static constexpr int END = WAVE + kWaves * W_UNITS;
};

// Stages one chain (weights W1 [64][ld1] of which the first C columns are the grid channels,
// W2 [64][64], Wo [n_out][64]) in the single-MLP layout, its outputs in rows first_row .. of
// the last layer (rows 0..3 = rows 4..7, as the single-MLP kernels expect).
template <int C, bool BWD, int NB>
__device__ __forceinline__ void stage_chain(uint4* lds, const float* W1, int ld1, const float* W2, const float* Wo,
                                            const float* b1, const float* b2, const float* bo, int n_out,
                                            int first_row)
{
    using L = MlpLds<C, kH, 2, BWD, NB>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    auto hidden_col = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto block_row = [](int mb, int i) { return 32 * mb + i; };
    auto out_row = [=](int p) { return (p >= first_row && p < first_row + n_out) ? p - first_row : -1; };
    stage_operand(lds + L::A1, W1, MB, KS1, ld1, block_row, [](int s, int gg, int e) { return k_input<C>(s, gg, e); });
    stage_operand(lds + L::A2, W2, MB, KSH, kH, block_row, hidden_col);
    stage_operand(lds + L::A3, Wo, 1, KSH, kH, [=](int, int i) { return i < 8 ? out_row(i & 3) : -1; }, hidden_col);
    if constexpr (BWD) {
        stage_operand_t(lds + L::T3, Wo, MB, 1, kH, block_row, [=](int, int, int e) { return e < 4 ? out_row(e) : -1; });
        stage_operand_t(lds + L::T2, W2, MB, KSH, kH, block_row, hidden_col);
        stage_operand_t(lds + L::T1, W1, 1, KSH, ld1, [](int, int i) { return i & (C - 1); }, hidden_col);
    }
    float* sbias = reinterpret_cast<float*>(lds + L::BIAS);
    for (int i = threadIdx.x; i < kH; i += blockDim.x) {
        sbias[i] = b1[i];
        sbias[kH + i] = b2[i];
    }
    if (threadIdx.x < 4) {
        const int p = out_row(threadIdx.x);
        sbias[2 * kH + threadIdx.x] = p >= 0 ? bo[p] : 0.0f;
    }
}

template <int C, bool BWD, int NB>
__device__ __forceinline__ void stage_decoder(uint4* lds, const Dec2Dev& d)
{
    using L = Lds<C, BWD, NB>;
    stage_chain<C, BWD, NB>(lds + L::S, d.Ws[0], C, d.Ws[1], d.Ws[2], d.bs[0], d.bs[1], d.bs[2], 1, 0);
    stage_chain<C, BWD, NB>(lds + L::V, d.Wv[0], C + d.E, d.Wv[1], d.Wv[2], d.bv[0], d.bv[1], d.bv[2], 3, 1);
    // direction columns of the feature chain's first layer: element e of lane group g in K-step s
    // is direction input 16 s + 8 g + e
    const int E = d.E;
    stage_operand(lds + L::A1E, d.Wv[0], 2, L::KSE, C + E, [](int mb, int i) { return 32 * mb + i; },
                  [=](int s, int gg, int e) { return 16 * s + 8 * gg + e < E ? C + 16 * s + 8 * gg + e : -1; });
}

// The ray's feature-chain bias b1 + W1[:, direction inputs] enc(d) into the wave's LDS area.
template <int C, bool BWD, int NB>
__device__ __forceinline__ void ray_direction_bias(uint4* lds, const Dec2Dev& d, const RayGeom& q, int lane, int wave)
{
    using L = Lds<C, BWD, NB>;
    uint4* area = lds + L::WAVE + wave * L::W_UNITS;
    float* ray_bias = reinterpret_cast<float*>(area + L::W_BIAS);
    float* ray_x = reinterpret_cast<float*>(area + L::W_X);
    const int col = lane & 31, grp = lane >> 5;
    const float dir[3] = {q.dx, q.dy, q.dz};
    const float x_lane = lane < d.E ? dir_encoding(dir, lane) : 0.0f;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane < kMaxDir) ray_x[lane] = x_lane;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    f32x16 acc[2][1];
    init_bias<2, 1>(acc, reinterpret_cast<const float*>(lds + L::V + L::Chain::BIAS), grp);
    Frag eh[1][L::KSE], el[1][L::KSE];
#pragma unroll
    for (int s = 0; s < L::KSE; ++s) {
        float x[8];
        *reinterpret_cast<f32x4*>(x) = *reinterpret_cast<const f32x4*>(ray_x + 16 * s + 8 * grp);
        *reinterpret_cast<f32x4*>(x + 4) = *reinterpret_cast<const f32x4*>(ray_x + 16 * s + 8 * grp + 4);
        split8(x, eh[0][s], el[0][s]);
    }
    layer_mfma<2, L::KSE, 1>(acc, lds + L::A1E, lane, eh, el);
    if (col == 0) {  // every column holds the same values
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) ray_bias[32 * mb + d_row(r, grp)] = acc[mb][0][r];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace dec2

}  // namespace lp
