// The decoder MLP of one 64-sample step on the matrix cores: LDS layout of the weights as
// MFMA A operands, their staging, and the forward pass shared by the forward kernel and the
// recomputing backward kernel (Section 3.4 of the paper: the backward re-runs the forward of
// every sample instead of reading stored activations).
#pragma once
#include "lp_mfma.h"

namespace lp {

// Shapes: C input channels, H hidden width, NH hidden layers (1 or 2), 4 outputs.
// NB = N blocks of 32 samples per step (2 in the forward kernel, 1 in the backward).
template <int C, int H, int NH, bool BWD, int NB = 2>
struct MlpLds {
    static constexpr int MB = H / 32;   // 32-row blocks of a hidden layer
    static constexpr int KS1 = C / 16;  // K-steps over the input channels
    static constexpr int KSH = H / 16;  // K-steps over a hidden layer
    // offsets in uint4 (16 B) units; one (block, K-step) = 64 hi + 64 lo entries = 128 units
    static constexpr int A1 = 0;                                   // W1   [MB][KS1]
    static constexpr int A2 = A1 + MB * KS1 * 128;                 // W2   [MB][KSH]   (NH == 2)
    static constexpr int A3 = A2 + (NH == 2 ? MB * KSH * 128 : 0); // Wout [1][KSH], rows 0..3 = rows 4..7
    static constexpr int FWD_END = A3 + KSH * 128;
    // transposed weights for the input-gradient chain (backward only)
    static constexpr int T3 = FWD_END;                             // Wout^T [MB][1]
    static constexpr int T2 = T3 + (BWD ? MB * 128 : 0);           // W2^T   [MB][KSH]  (NH == 2)
    static constexpr int T1 = T2 + (BWD && NH == 2 ? MB * KSH * 128 : 0);  // W1^T [1][KSH], 32 rows
    static constexpr int W_END = T1 + (BWD ? KSH * 128 : 0);
    static constexpr int BIAS = W_END;                             // floats: b1[H] b2[H] bout[4]
    static constexpr int BIAS_UNITS = (2 * H + 4 + 3) / 4;
    static constexpr int END = BIAS + BIAS_UNITS;                  // first unit after weights and biases
    // per-sample scatter records of a backward wave: 32 NB samples x 16 dwords (weights, corner offsets)
    static constexpr int INFO_UNITS = 32 * NB * 4;
    static constexpr int bytes(int waves) { return (END + (BWD ? waves * INFO_UNITS : 0)) * 16; }
};

// CG = channels of the grid (the gradient of the first CG inputs is scattered); CG < C: the
// other inputs are per-ray direction inputs.
template <int C, int H, int NH, bool BWD, int NB, int CG = C>
__device__ __forceinline__ void stage_mlp(uint4* lds, const MlpDev& m)
{
    using L = MlpLds<C, H, NH, BWD, NB>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    auto hidden_col = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto block_row = [](int mb, int i) { return 32 * mb + i; };
    stage_operand(lds + L::A1, m.W[0], MB, KS1, C, block_row,
                  [](int s, int gg, int e) { return k_input<C>(s, gg, e); });
    if constexpr (NH == 2) stage_operand(lds + L::A2, m.W[1], MB, KSH, H, block_row, hidden_col);
    // output layer: rows 0..3 and 4..7 both carry the 4 outputs, so that both lane groups of a
    // sample column hold them (D rows 4g + p)
    stage_operand(lds + L::A3, m.W[NH], 1, KSH, H, [](int, int i) { return i < 8 ? (i & 3) : -1; }, hidden_col);
    if constexpr (BWD) {
        // A[m][k] = W^T[m][k] = W[k][m]: read W with (row, col) swapped.  stage_operand reads
        // W[row_of * ld + col_of], so pass the transposed roles: "row" = k index, "col" = m index.
        // Wout^T: K = 16 with the 4 outputs at k = 0..3 and again at k = 8..11 (either lane group
        // of the B operand may carry the output gradients)
        stage_operand_t(lds + L::T3, m.W[NH], MB, 1, H,
                        [](int mb, int i) { return 32 * mb + i; },
                        [](int, int, int e) { return e < 4 ? e : -1; });
        if constexpr (NH == 2)
            stage_operand_t(lds + L::T2, m.W[1], MB, KSH, H, [](int mb, int i) { return 32 * mb + i; },
                            [](int s, int gg, int e) { return k_hidden(s, gg, e); });
        // 32 rows: for 16 grid channels a second copy of their 16 rows (the scatter of the
        // backward kernel uses both halves of a lane group)
        stage_operand_t(lds + L::T1, m.W[0], 1, KSH, C, [](int, int i) { return i & (CG - 1); },
                        [](int s, int gg, int e) { return k_hidden(s, gg, e); });
    }
    float* sbias = reinterpret_cast<float*>(lds + L::BIAS);
    for (int i = threadIdx.x; i < H; i += blockDim.x) {
        sbias[i] = m.b[0][i];
        sbias[H + i] = NH == 2 ? m.b[1][i] : 0.0f;
    }
    if (threadIdx.x < 4) sbias[2 * H + threadIdx.x] = m.b[NH][threadIdx.x];
}

// accumulators of a hidden layer start from the bias of the rows each register holds
template <int MB, int NB>
__device__ __forceinline__ void init_bias(f32x16 (&acc)[MB][NB], const float* bias, int grp)
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 b = *reinterpret_cast<const f32x4*>(bias + 32 * mb + 8 * q + 4 * grp);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int p = 0; p < 4; ++p) acc[mb][nb][4 * q + p] = b[p];
        }
}

template <int MB, int NB>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MB][NB])
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.0f;
}

// acc[mb][nb] (+)= A[mb][s] * B[nb][s] over KS K-steps, A from LDS at `a_base`; FRESH starts the
// accumulation from zero instead of adding to acc
template <int MB, int KS, int NB, bool FRESH = false>
__device__ __forceinline__ void layer_mfma(f32x16 (&acc)[MB][NB], const uint4* a_base, int lane,
                                           const Frag (&bh)[NB][KS], const Frag (&bl)[NB][KS])
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            Frag ah, al;
            load_operand(a_base + (mb * KS + s) * 128, lane, ah, al);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[mb][nb] = (FRESH && s == 0) ? mfma3_first(ah, al, bh[nb][s], bl[nb][s])
                                                : mfma3(ah, al, bh[nb][s], bl[nb][s], acc[mb][nb]);
        }
}

// D registers of a layer (optionally through ReLU) -> B operands of the next contraction
template <int MB, bool RELU, int NB>
__device__ __forceinline__ void to_operands(const f32x16 (&acc)[MB][NB], Frag (&bh)[NB][2 * MB], Frag (&bl)[NB][2 * MB])
{
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int s = 0; s < 2 * MB; ++s) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = acc[s / 2][nb][8 * (s % 2) + e];
                v[e] = RELU ? relu_f(x) : x;
            }
            split8(v, bh[nb][s], bl[nb][s]);
        }
}

// Everything the forward of one 64-sample step produces.  The forward kernel uses z only; the
// backward keeps the operand fragments (they are the activations, already split).
template <int C, int H, int NH, int NB>
struct StepActs {
    static constexpr int KS1 = C / 16, KSH = H / 16;
    Frag fh[NB][KS1], fl[NB][KS1];    // interpolated features (layer-1 B operands)
    Frag h1h[NB][KSH], h1l[NB][KSH];  // hidden layer 1 after ReLU
    Frag h2h[NB][KSH], h2l[NB][KSH];  // hidden layer 2 after ReLU (NH == 2)
    float z[4];                       // decoder outputs of the lane's sample: j0 + lane for NB = 2,
                                      // j0 + (lane & 31) in both lane groups for NB = 1
    Cell3 cell[NB];                   // grid cell of sample (lane & 31) of every N block
};

struct RayGeom {
    float ox, oy, oz, dx, dy, dz, near, delta;
    double delta64;
    int scene;
    float time;       // the ray's time (read for a HexPlane only; -inf = none given: clamps onto the first index)
    float extra[16];  // direction inputs of the MLP (only when the MLP has more inputs than the grid has channels)
};

// the encoded view direction, then zeros
__device__ __forceinline__ void set_direction_inputs(const MlpDev& m, RayGeom& q)
{
    const float d[3] = {q.dx, q.dy, q.dz};
#pragma unroll
    for (int e = 0; e < 16; ++e) q.extra[e] = e < m.n_enc ? dir_encoding(d, e) : 0.0f;
}

__device__ __forceinline__ RayGeom load_ray_geom(const RaysDev& rays, long long ray)
{
    RayGeom q;
    q.ox = rays.origins[3 * ray + 0]; q.oy = rays.origins[3 * ray + 1]; q.oz = rays.origins[3 * ray + 2];
    q.dx = rays.dirs[3 * ray + 0]; q.dy = rays.dirs[3 * ray + 1]; q.dz = rays.dirs[3 * ray + 2];
    q.near = rays.near[ray];
    q.delta64 = ((double)rays.far[ray] - (double)q.near) / (double)rays.S;
    q.delta = (float)q.delta64;
    q.scene = rays.scene ? rays.scene[ray] : 0;
    q.time = rays.time ? rays.time[ray] : -INFINITY;
    return q;
}

// Cell of sample j (0-based): t_j = near + (j + 1/2) Delta, x = o + t d, in fp64 from the fp32 inputs.
template <bool CC>
__device__ __forceinline__ Cell3 sample_cell(const GridDev& g, const RayGeom& q, int j)
{
    const double t = (double)q.near + ((double)j + 0.5) * q.delta64;
    return locate3<CC>(g, (double)q.ox + t * (double)q.dx, (double)q.oy + t * (double)q.dy,
                   (double)q.oz + t * (double)q.dz);
}

// Same, with the contraction chosen at run time (a uniform branch): for kernels that are bound by
// their scatter, where a second set of instantiations would only cost build time.
__device__ __forceinline__ Cell3 sample_cell_any(const GridDev& g, const RayGeom& q, int j)
{
    return g.contract > 0.0 ? sample_cell<true>(g, q, j) : sample_cell<false>(g, q, j);
}

// Storage type "decided at run time": kernels instantiated with it read g.dtype in a uniform branch
// around their gathers (the decoder kernels, which would otherwise triple their instantiations).
constexpr int kAnyDtype = 3;

// The kernels for grids stored in reduced precision take the contraction at run time as well (no
// second set of instantiations); those for fp32 grids have it compiled in.
template <bool CC, int GT>
__device__ __forceinline__ Cell3 sample_cell_for(const GridDev& g, const RayGeom& q, int j)
{
    if constexpr (GT != LP_F32) return sample_cell_any(g, q, j);
    else return sample_cell<CC>(g, q, j);
}

// Sample (within a 32-sample step) that MFMA column `slot` stands for when the step is
// permuted so that each lane group's D registers of a [sample x channel] block hold 16
// CONSECUTIVE samples: slot 8q + 4g + p  <->  sample 16g + 4q + p.
__host__ __device__ constexpr int slot_to_sample(int slot)
{
    return 16 * ((slot >> 2) & 1) + 4 * (slot >> 3) + (slot & 3);
}
__host__ __device__ constexpr int sample_to_slot(int smp)
{
    return 8 * ((smp >> 2) & 3) + 4 * (smp >> 4) + (smp & 3);
}

// Input features of one sample column as operand fragments: lane (col, grp) holds inputs
// [grp C/2, (grp+1) C/2).  CG == C: all inputs are grid channels.  CG == C/2: lane group 0 holds
// the CG grid channels, lane group 1 the per-ray direction inputs q.extra.
template <int KIND, int C, int CG, int GT = LP_F32>
__device__ __forceinline__ void sample_features_typed(const GridDev& g, const RayGeom& q, const Cell3& c, int grp,
                                                      Frag (&fh)[C / 16], Frag (&fl)[C / 16])
{
    float feat[C / 2];
    if constexpr (CG == C && KIND == LP_GRID_HEXPLANE) {
        gather_half_hexplane<C, C / 2, GT>(g, q.scene, c, q.time, grp * (C / 2), feat);
    } else if constexpr (CG == C) {
        gather_half<KIND, C, C / 2, GT>(g, q.scene, c, grp * (C / 2), feat);
    } else {
        static_assert(2 * CG == C && CG == 16, "direction inputs take the second half of 32 inputs");
        if (grp == 0) {
            if constexpr (KIND == LP_GRID_HEXPLANE) gather_half_hexplane<CG, CG, GT>(g, q.scene, c, q.time, 0, feat);
            else gather_half<KIND, CG, CG, GT>(g, q.scene, c, 0, feat);
        } else {
#pragma unroll
            for (int e = 0; e < CG; ++e) feat[e] = q.extra[e];
        }
    }
#pragma unroll
    for (int s = 0; s < C / 16; ++s) split8(feat + 8 * s, fh[s], fl[s]);
}

// GT = kAnyDtype: the grid's storage type is taken at run time (a uniform branch around the gather).
template <int KIND, int C, int CG, int GT = LP_F32>
__device__ __forceinline__ void sample_features(const GridDev& g, const RayGeom& q, const Cell3& c, int grp,
                                                Frag (&fh)[C / 16], Frag (&fl)[C / 16])
{
    if constexpr (GT == kAnyDtype) {
        if (g.dtype == LP_F32) sample_features_typed<KIND, C, CG, LP_F32>(g, q, c, grp, fh, fl);
        else if (g.dtype == LP_BF16) sample_features_typed<KIND, C, CG, LP_BF16>(g, q, c, grp, fh, fl);
        else sample_features_typed<KIND, C, CG, LP_F16>(g, q, c, grp, fh, fl);
    } else {
        sample_features_typed<KIND, C, CG, GT>(g, q, c, grp, fh, fl);
    }
}

// MLP forward of one step from the input features a.fh / a.fl: fills the hidden activations and
// the decoder outputs a.z.  bias1, if given, replaces the first layer's bias (one that holds a
// ray's constant inputs already contracted).
template <int C, int H, int NH, bool BWD, int NB>
__device__ __forceinline__ void mlp_forward(const uint4* lds, int lane, StepActs<C, H, NH, NB>& a,
                                            const float* bias1 = nullptr)
{
    using L = MlpLds<C, H, NH, BWD, NB>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    const int grp = lane >> 5;
    const float* sbias = reinterpret_cast<const float*>(lds + L::BIAS);

    f32x16 acc[MB][NB];
    init_bias<MB, NB>(acc, bias1 ? bias1 : sbias, grp);
    layer_mfma<MB, KS1, NB>(acc, lds + L::A1, lane, a.fh, a.fl);
    to_operands<MB, true, NB>(acc, a.h1h, a.h1l);
    if constexpr (NH == 2) {
        init_bias<MB, NB>(acc, sbias + H, grp);
        layer_mfma<MB, KSH, NB>(acc, lds + L::A2, lane, a.h1h, a.h1l);
        to_operands<MB, true, NB>(acc, a.h2h, a.h2l);
    }
    const Frag (&lh)[NB][KSH] = NH == 2 ? a.h2h : a.h1h;
    const Frag (&ll)[NB][KSH] = NH == 2 ? a.h2l : a.h1l;

    // output layer: its 4 rows are replicated in rows 0..3 and 4..7, so both lane groups of a
    // sample column hold them.  NB = 2: lanes 0..31 take N block 0, lanes 32..63 N block 1, so
    // that lane l owns sample j0 + l.  NB = 1: both lane groups own sample j0 + col.
    f32x16 o[NB];
    const f32x4 b = *reinterpret_cast<const f32x4*>(sbias + 2 * H);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[nb][r] = r < 4 ? b[r] : 0.0f;
#pragma unroll
    for (int s = 0; s < KSH; ++s) {
        Frag ah, al;
        load_operand(lds + L::A3 + s * 128, lane, ah, al);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) o[nb] = mfma3(ah, al, lh[nb][s], ll[nb][s], o[nb]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) a.z[k] = (NB == 2 && grp) ? o[NB - 1][k] : o[0][k];
}

// Sampling + MLP forward of one step: lane (col, grp) samples its half of the channels of
// sample col of every N block (PERM: of the permuted step, see slot_to_sample).
template <int KIND, int C, int H, int NH, bool BWD, int NB, bool PERM = false, bool CC = false, int CG = C, int GT = LP_F32>
__device__ __forceinline__ void forward_step(const GridDev& g, const uint4* lds, const RayGeom& q, int j0, int S,
                                             int lane, StepActs<C, H, NH, NB>& a)
{
    const int col = lane & 31, grp = lane >> 5;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int j = min(j0 + 32 * nb + (PERM ? slot_to_sample(col) : col), S - 1);
        const Cell3 c = sample_cell_for<CC, GT>(g, q, j);
        a.cell[nb] = c;
        sample_features<KIND, C, CG, GT>(g, q, c, grp, a.fh[nb], a.fl[nb]);
    }
    mlp_forward<C, H, NH, BWD, NB>(lds, lane, a);
}

// MLP of one 64-sample step from the input fragments of its two N blocks, keeping nothing but
// the decoder outputs: the first layer runs on both N blocks at once (sharing the weight
// operands), the remaining layers one N block after the other, so that at most one block's
// accumulators and activations are alive at a time (registers for a second wave per SIMD).
// `lds` points at the MLP's weights (layout MlpLds), `bias1` at the first layer's bias (the
// layout's own, or one that holds a ray's constant inputs already contracted).  z = outputs of
// sample j0 + lane.
template <int C, int H, int NH>
__device__ __forceinline__ void mlp_outputs(const uint4* lds, const float* bias1, int lane,
                                            const Frag (&fh)[2][C / 16], const Frag (&fl)[2][C / 16], float (&z)[4])
{
    using L = MlpLds<C, H, NH, false, 2>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    const int grp = lane >> 5;
    const float* sbias = reinterpret_cast<const float*>(lds + L::BIAS);
    Frag h1h[2][KSH], h1l[2][KSH];
    {
        f32x16 acc[MB][2];
        init_bias<MB, 2>(acc, bias1, grp);
        layer_mfma<MB, KS1, 2>(acc, lds + L::A1, lane, fh, fl);
        to_operands<MB, true, 2>(acc, h1h, h1l);
    }
    const f32x4 bo = *reinterpret_cast<const f32x4*>(sbias + 2 * H);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        Frag lh[1][KSH], ll[1][KSH];
        if constexpr (NH == 2) {
            Frag inh[1][KSH], inl[1][KSH];
#pragma unroll
            for (int s = 0; s < KSH; ++s) { inh[0][s] = h1h[nb][s]; inl[0][s] = h1l[nb][s]; }
            f32x16 acc[MB][1];
            init_bias<MB, 1>(acc, sbias + H, grp);
            layer_mfma<MB, KSH, 1>(acc, lds + L::A2, lane, inh, inl);
            to_operands<MB, true, 1>(acc, lh, ll);
        } else {
#pragma unroll
            for (int s = 0; s < KSH; ++s) { lh[0][s] = h1h[nb][s]; ll[0][s] = h1l[nb][s]; }
        }
        f32x16 o;
#pragma unroll
        for (int r = 0; r < 16; ++r) o[r] = r < 4 ? bo[r] : 0.0f;
#pragma unroll
        for (int s = 0; s < KSH; ++s) {
            Frag ah, al;
            load_operand(lds + L::A3 + s * 128, lane, ah, al);
            o = mfma3(ah, al, lh[0][s], ll[0][s], o);
        }
        // lanes 0..31 own the samples of N block 0, lanes 32..63 those of N block 1
#pragma unroll
        for (int k = 0; k < 4; ++k) z[k] = (nb == 0 || grp) ? o[k] : z[k];
        // keep the two N blocks apart: interleaving them would double the live registers
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Sampling + MLP of one 64-sample step for the forward kernel.  z = outputs of sample j0 + lane.
template <int KIND, int C, int H, int NH, bool CC, int CG = C, int GT = LP_F32>
__device__ __forceinline__ void forward_outputs(const GridDev& g, const uint4* lds, const RayGeom& q, int j0,
                                                int S, int lane, float (&z)[4])
{
    using L = MlpLds<C, H, NH, false, 2>;
    constexpr int KS1 = L::KS1;
    const int col = lane & 31, grp = lane >> 5;
    Frag fh[2][KS1], fl[2][KS1];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int j = min(j0 + 32 * nb + col, S - 1);
        const Cell3 c = sample_cell_for<CC, GT>(g, q, j);
        sample_features<KIND, C, CG, GT>(g, q, c, grp, fh[nb], fl[nb]);
    }
    mlp_outputs<C, H, NH>(lds, reinterpret_cast<const float*>(lds + L::BIAS), lane, fh, fl, z);
}

}  // namespace lp
