// Splatter backward with an MLP on the matrix cores (Section 3.3 "Splatter" and Section 3.4:
// nothing of the forward is stored, every point's MLP forward is recomputed), wavefront per ray.
//
// The gradient that reaches a point's pushed vector is the normalised output gradient read at
// the point: sum over the cell's corners of weight * d_theta / theta_w.  From there the step is
// the Renderer's backward with a wide last layer: input gradients with the transposed weights,
// weight gradients contracted over the 32 points of the step (operands transposed on the matrix
// cores with 0/1 selection matrices), accumulators parked in the accumulation registers for the
// whole kernel and written as one record of partial sums per wave.  The gradient of the MLP's
// inputs is taken with the operands swapped (lane = input, register = point): the prior's
// channels go through the run-merging scatter into the prior's gradient.
//
// The pixel feature and the direction encoding are the same for every point of a ray, so their
// part of the first layer is taken once per ray: W1[:, per-ray inputs] x joins the bias before
// the ray's steps, and after them the sum s of dZ1 over the ray's points gives both the weight
// gradient s x^T (one rank-one matrix-core update per block) and the input gradient W1^T s.
//
// This header holds the kernel and its launcher templates; two translation units instantiate
// them (the instantiations for 32-channel triplanes are built without the build flag that keeps
// matrix-core results in ordinary vector registers: with it the compiler fails on them).
#pragma once
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"
#include "lp_splat_common.h"

namespace lp {

namespace {

constexpr int kWaves = 4;
constexpr int kHidden = 64;

// LDS layout in 16-byte units.  Kernel order of the MLP's inputs: KSP K-steps of prior channels,
// then KSE K-steps of per-ray inputs (pixel feature, direction encoding, zeros); element e of
// lane group g in K-step s is input 16 s + 8 g + e.
// start of a region of `size` units after `at`: moved up to the 64 KiB line (unit 4096) if it
// would straddle it, so that every region is reached from one address register
constexpr int lds_place(int at, int size) { return (at < 4096 && at + size > 4096) ? 4096 : at; }

template <int KSP, int KSE, int NH>
struct SplatBwdLds {
    static constexpr int MB = kHidden / 32, KSH = kHidden / 16;
    static constexpr int NBE = (KSE + 1) / 2;                           // 32-input blocks of per-ray inputs
    static constexpr int HH = NH == 2 ? MB * KSH * 128 : 0;             // a hidden-to-hidden matrix
    static constexpr int A1P = 0;                                       // W1, prior columns   [MB][KSP]
    static constexpr int A1E = A1P + MB * KSP * 128;                    // W1, per-ray columns [MB][KSE]
    static constexpr int A2 = A1E + MB * KSE * 128;                     // W2      [MB][KSH]  (NH == 2)
    static constexpr int T3 = A2 + HH;                                  // Wout^T  [MB][KSP]
    static constexpr int T2 = T3 + MB * KSP * 128;                      // W2^T    [MB][KSH]  (NH == 2)
    static constexpr int T1P = lds_place(T2 + HH, KSH * 128);           // W1^T, prior rows   [1][KSH]
    static constexpr int T1E = lds_place(T1P + KSH * 128, NBE * KSH * 128);  // W1^T, per-ray rows [NBE][KSH]
    static constexpr int SEL = lds_place(T1E + NBE * KSH * 128, 4 * 64);     // 4 selection operands, 64 lanes each
    static constexpr int BIAS = lds_place(SEL + 4 * 64, 2 * kHidden / 4);    // floats b1[64] b2[64]
    // a wave's area: 32 scatter records of 16 dwords, the ray's first-layer bias, the ray's sum of dZ1
    // and its 48 per-ray inputs
    static constexpr int W_INFO = 0, W_BIAS = 128, W_SUM = W_BIAS + kHidden / 4, W_X = W_SUM + kHidden / 4,
                         W_UNITS = W_X + 48 / 4;
    static constexpr int WAVE = lds_place(BIAS + 2 * kHidden / 4, kWaves * W_UNITS);  // per-wave areas
    static constexpr int UNITS = WAVE + kWaves * W_UNITS;
    static_assert(T2 + HH <= 4096, "the regions up to W2^T lie below the 64 KiB line");
};

// column of the caller's first layer (pixel feature, prior channels, direction encoding) that
// kernel input `kin` stands for; -1: padding
template <int CP>
__device__ __forceinline__ int caller_column(int kin, int n_in, int n_extra)
{
    if (kin < CP) return n_in + kin;
    const int x = kin - CP;
    return x < n_in ? x : x < n_extra ? CP + x : -1;
}

template <int KSP, int KSE, int NH>
__device__ __forceinline__ void stage_splat_bwd(uint4* lds, const MlpDev& m, int n_in)
{
    using L = SplatBwdLds<KSP, KSE, NH>;
    constexpr int MB = L::MB, KSH = L::KSH, CP = 16 * KSP;
    const int n_extra = n_in + m.n_enc;
    auto hidden_col = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto block_row = [](int mb, int i) { return 32 * mb + i; };
    stage_operand(lds + L::A1P, m.W[0], MB, KSP, m.dims[0], block_row,
                  [=](int s, int gg, int e) { return caller_column<CP>(16 * s + 8 * gg + e, n_in, n_extra); });
    stage_operand(lds + L::A1E, m.W[0], MB, KSE, m.dims[0], block_row,
                  [=](int s, int gg, int e) { return caller_column<CP>(CP + 16 * s + 8 * gg + e, n_in, n_extra); });
    if constexpr (NH == 2) {
        stage_operand(lds + L::A2, m.W[1], MB, KSH, kHidden, block_row, hidden_col);
        stage_operand_t(lds + L::T2, m.W[1], MB, KSH, kHidden, block_row, hidden_col);
    }
    // Wout^T: rows = hidden units, K = output channels
    stage_operand_t(lds + L::T3, m.W[NH], MB, KSP, kHidden, block_row,
                    [](int s, int gg, int e) { return 16 * s + 8 * gg + e; });
    // W1^T as the B operand of the swapped product: "row" i = input.  Prior channels (16: a second
    // copy in rows 16..31, both halves of a lane group scatter), then blocks of per-ray inputs.
    stage_operand_t(lds + L::T1P, m.W[0], 1, KSH, m.dims[0], [=](int, int i) { return n_in + (i & (CP - 1)); },
                    hidden_col);
    stage_operand_t(lds + L::T1E, m.W[0], L::NBE, KSH, m.dims[0],
                    [=](int be, int i) { return caller_column<CP>(CP + 32 * be + i, n_in, n_extra); }, hidden_col);
    float* sbias = reinterpret_cast<float*>(lds + L::BIAS);
    for (int i = threadIdx.x; i < kHidden; i += blockDim.x) {
        sbias[i] = m.b[0][i];
        sbias[kHidden + i] = NH == 2 ? m.b[1][i] : 0.0f;
    }
    // selection operands: hidden tensors (k_hidden order, two K-steps per block of 32 features),
    // then inputs and outputs (natural order)
    if (threadIdx.x < 64) {
        const int j = threadIdx.x & 31, gg = threadIdx.x >> 5;
        const Frag f[4] = {selection(j, gg, [](int g2, int e) { return k_hidden(0, g2, e); }),
                           selection(j, gg, [](int g2, int e) { return k_hidden(1, g2, e); }),
                           selection(j, gg, [](int g2, int e) { return 8 * g2 + e; }),
                           selection(j, gg, [](int g2, int e) { return 16 + 8 * g2 + e; })};
#pragma unroll
        for (int k = 0; k < 4; ++k) lds[L::SEL + 64 * k + threadIdx.x] = make_uint4(f[k].d[0], f[k].d[1], f[k].d[2], f[k].d[3]);
    }
}

// The normalised output gradient at a point as operand fragments: lane (col, grp) holds channels
// 16 s + 8 grp .. + 7 of its point; zero for a point past the end of the ray.
template <int KIND, int C>
__device__ __forceinline__ void gather_normalised(const GridDev& tgt, const SplatDev& sp, int scene, const Cell3& c,
                                                  int grp, bool valid, Frag (&gh)[1][C / 16], Frag (&gl)[1][C / 16])
{
    constexpr int NC = KIND == LP_GRID_VOXEL ? 8 : 12;
    // corner weights over the weight sums of the forward (0 where nothing landed); cell offsets in
    // 32 bits relative to the scene
    float wn[NC];
    if constexpr (KIND == LP_GRID_VOXEL) {
        const float* W = sp.theta_w_in[0] + (size_t)scene * tgt.N[0] * tgt.N[1] * tgt.N[2];
        const unsigned sy = (unsigned)tgt.N[2], sx = (unsigned)tgt.N[1] * sy;
        const unsigned base = (unsigned)c.i[0] * sx + (unsigned)c.i[1] * sy + (unsigned)c.i[2];
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) * (dz ? c.f[2] : c.g[2]);
            const float ws = W[base + dx * sx + dy * sy + dz];
            wn[d] = (valid && ws > 0.0f) ? w * __frcp_rn(ws) : 0.0f;
        }
    } else {
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            const float* W = sp.theta_w_in[p] + (size_t)scene * tgt.N[a] * tgt.N[b];
            const unsigned sa = (unsigned)tgt.N[b];
            const unsigned base = (unsigned)c.i[a] * sa + (unsigned)c.i[b];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                const float w = (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]);
                const float ws = W[base + da * sa + db];
                wn[4 * p + d] = (valid && ws > 0.0f) ? w * __frcp_rn(ws) : 0.0f;
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    GridDev dth = tgt;
#pragma unroll
    for (int p = 0; p < 3; ++p) dth.data[p] = sp.d_theta[p];
#pragma unroll
    for (int s = 0; s < C / 16; ++s) {
        GatherRaw<KIND, 8, LP_F32> raw;
        gather_issue<KIND, C, 8, LP_F32>(dth, scene, c, 16 * s + 8 * grp, raw);
        float v[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int d = 0; d < NC; ++d)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                float x[4];
                unpack_values<LP_F32>(raw.v[d][i], x);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[4 * i + e] += wn[d] * x[e];
            }
        split8(v, gh[0][s], gl[0][s]);
        __builtin_amdgcn_sched_barrier(0);  // one K-step's loads at a time
    }
}

template <int KIND, int KSP, int KSE, int NH>
__global__ __launch_bounds__(kWaves * 64) void splat_mfma_bwd_kernel(GridDev tgt, MlpDev m, RaysDev rays,
                                                                     SplatDev sp, BwdIo io, long long group_mul)
{
    using L = SplatBwdLds<KSP, KSE, NH>;
    constexpr int MB = L::MB, KSH = L::KSH, NBE = L::NBE;
    constexpr int CP = 16 * KSP;          // channels of the prior and of the target
    extern __shared__ uint4 lds[];
    stage_splat_bwd<KSP, KSE, NH>(lds, m, sp.n_in);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // LDS instructions reach 64 KiB from their address register; everything beyond is addressed
    // from a second base whose value the compiler does not see (it would otherwise keep one
    // register per 1 KiB block for the whole kernel)
    int upper_units = 4096;
    asm volatile("" : "+v"(upper_units));
    const uint4* lds_upper = lds + upper_units;
    auto block = [&](int unit) { return unit < 4096 ? lds + unit : lds_upper + (unit - 4096); };
    uint4* wave_area = const_cast<uint4*>(block(L::WAVE)) + wave * L::W_UNITS;
    float* info = reinterpret_cast<float*>(wave_area + L::W_INFO);
    float* ray_bias = reinterpret_cast<float*>(wave_area + L::W_BIAS);
    float* ray_sum = reinterpret_cast<float*>(wave_area + L::W_SUM);
    float* ray_x = reinterpret_cast<float*>(wave_area + L::W_X);
    const float* sbias = reinterpret_cast<const float*>(block(L::BIAS));
    const int n_in = sp.n_in, n_extra = sp.n_in + m.n_enc;

    auto sel = [&](int k) {
        const uint4 v = block(L::SEL + 64 * k)[lane];
        Frag f;
        f.d[0] = v.x; f.d[1] = v.y; f.d[2] = v.z; f.d[3] = v.w;
        return f;
    };
    // transposes block nb2 (features 32 nb2 .. +31) of a hidden tensor held as operand fragments
    auto transpose_hidden = [&](const Frag (&xh)[kBwdNB][KSH], const Frag (&xl)[kBwdNB][KSH], int nb2,
                                Frag (&th)[kBwdKS], Frag (&tl)[kBwdKS]) {
        const Frag s0 = sel(0), s1 = sel(1);
        f32x16 dh = mfma1(xh[0][2 * nb2], s0, zero16());
        dh = mfma1(xh[0][2 * nb2 + 1], s1, dh);
        f32x16 dl = mfma1(xl[0][2 * nb2], s0, zero16());
        dl = mfma1(xl[0][2 * nb2 + 1], s1, dl);
        pack_exact(dh, th);
        pack_exact(dl, tl);
    };
    // same for a tensor of KSP K-steps (16 or 32 channels) in natural order
    auto transpose_channels = [&](const Frag (&xh)[1][KSP], const Frag (&xl)[1][KSP], Frag (&th)[kBwdKS],
                                  Frag (&tl)[kBwdKS]) {
        const Frag s0 = sel(2);
        f32x16 dh = mfma1(xh[0][0], s0, zero16());
        f32x16 dl = mfma1(xl[0][0], s0, zero16());
        if constexpr (KSP == 2) {
            const Frag s1 = sel(3);
            dh = mfma1(xh[0][1], s1, dh);
            dl = mfma1(xl[0][1], s1, dl);
        }
        pack_exact(dh, th);
        pack_exact(dl, tl);
    };
    // gradient accumulators, alive for the whole kernel
    f32x16 dW1p[MB];          // [64 x prior channels]
    f32x16 dW1e[MB][NBE];     // [64 x per-ray inputs], input block be
    f32x16 dW2[MB][MB];       // [64 x 64]      (NH == 2)
    f32x16 dWo[MB];           // [channels x 64], column block nb
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        dWo[mb] = zero16();  park(dWo[mb]);
        dW1p[mb] = zero16(); park(dW1p[mb]);
#pragma unroll
        for (int be = 0; be < NBE; ++be) { dW1e[mb][be] = zero16(); park(dW1e[mb][be]); }
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) { dW2[mb][nb] = zero16(); park(dW2[mb][nb]); }
    }
    float db1[MB], db2[MB], dbo = 0.0f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) db1[mb] = db2[mb] = 0.0f;

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
            layer_mfma<MB, KSE, 1>(acc, block(L::A1E), lane, eh, el);
            wave_lds_fence();
            if (col == 0) {  // every column holds the same values
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) ray_bias[32 * mb + d_row(r, grp)] = acc[mb][0][r];
            }
            wave_lds_fence();
        }
        float dbr[MB];   // dZ1 summed over this lane group's points of the ray, hidden unit 32 mb + col
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) dbr[mb] = 0.0f;
        __builtin_amdgcn_sched_barrier(0);

        for (int j0 = 0; j0 < S; j0 += kBwdStep) {
            const int j = j0 + slot_to_sample(col);
            const bool valid = j < S;
            const int jj = min(j, S - 1);
            Frag fh[1][KSP], fl[1][KSP];
            const Cell3 cp = sample_cell_any(sp.prior, q, jj);
#pragma unroll
            for (int s = 0; s < KSP; ++s) {
                float feat[8];
                gather_half<KIND, CP, 8, LP_F32>(sp.prior, q.scene, cp, 16 * s + 8 * grp, feat);
                split8(feat, fh[0][s], fl[0][s]);
                // one K-step's loads at a time: issued together they would need a register each
                __builtin_amdgcn_sched_barrier(0);
            }
            Frag gv_h[1][KSP], gv_l[1][KSP];
            gather_normalised<KIND, CP>(tgt, sp, q.scene, sample_cell_any(tgt, q, jj), grp, valid, gv_h, gv_l);
            // scatter record of this lane's point in the prior, read at the end of the step
            wave_lds_fence();
            if (grp == 0) write_scatter_record<KIND, CP>(info + col * 16, sp.prior, cp);

            // ---- forward of the hidden layers ----
            Frag h1h[1][KSH], h1l[1][KSH], h2h[1][KSH], h2l[1][KSH];
            f32x16 acc[MB][1];
            init_bias<MB, 1>(acc, ray_bias, grp);
            layer_mfma<MB, KSP, 1>(acc, block(L::A1P), lane, fh, fl);
            to_operands<MB, true, 1>(acc, h1h, h1l);
            if constexpr (NH == 2) {
                init_bias<MB, 1>(acc, sbias + kHidden, grp);
                layer_mfma<MB, KSH, 1>(acc, block(L::A2), lane, h1h, h1l);
                to_operands<MB, true, 1>(acc, h2h, h2l);
            }
            __builtin_amdgcn_sched_barrier(0);
            const Frag (&lh)[1][KSH] = NH == 2 ? h2h : h1h;
            const Frag (&ll)[1][KSH] = NH == 2 ? h2l : h1l;

            // ---- last layer: dWo += dV Hlast^T ; dbo += sum dV ; dZ = relu'(.) * (Wout^T dV) ----
            layer_mfma<MB, KSP, 1, true>(acc, block(L::T3), lane, gv_h, gv_l);
            {
                Frag ah[kBwdKS], al[kBwdKS];
                transpose_channels(gv_h, gv_l, ah, al);
#pragma unroll
                for (int ks = 0; ks < kBwdKS; ++ks) dbo = frag_sum(al[ks], frag_sum(ah[ks], dbo));
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) {
                    Frag bh[kBwdKS], bl[kBwdKS];
                    transpose_hidden(lh, ll, nb2, bh, bl);
                    mfma6_parked(dWo[nb2], ah, al, bh, bl);
                    __builtin_amdgcn_sched_barrier(0);  // one accumulator block out of its parking place at a time
                }
            }
            relu_mask<MB>(acc, lh);
            Frag gz_h[1][KSH], gz_l[1][KSH];
            to_operands<MB, false, 1>(acc, gz_h, gz_l);
            __builtin_amdgcn_sched_barrier(0);

            if constexpr (NH == 2) {
                // ---- dW2 += dZ2 H1^T ; db2 += sum dZ2 ; dZ1 = relu'(.) * (W2^T dZ2) ----
                Frag ah[MB][kBwdKS], al[MB][kBwdKS];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    transpose_hidden(gz_h, gz_l, mb, ah[mb], al[mb]);
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) db2[mb] = frag_sum(al[mb][ks], frag_sum(ah[mb][ks], db2[mb]));
                }
                layer_mfma<MB, KSH, 1, true>(acc, block(L::T2), lane, gz_h, gz_l);
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) {
                    Frag bh[kBwdKS], bl[kBwdKS];
                    transpose_hidden(h1h, h1l, nb2, bh, bl);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        mfma6_parked(dW2[mb][nb2], ah[mb], al[mb], bh, bl);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                relu_mask<MB>(acc, h1h);
                to_operands<MB, false, 1>(acc, gz_h, gz_l);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- first layer, prior columns: dW1 += dZ1 F^T ; the ray's sum of dZ1 ----
            {
                Frag bh[kBwdKS], bl[kBwdKS];
                transpose_channels(fh, fl, bh, bl);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    Frag ah[kBwdKS], al[kBwdKS];
                    transpose_hidden(gz_h, gz_l, mb, ah, al);
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) dbr[mb] = frag_sum(al[ks], frag_sum(ah[ks], dbr[mb]));
                    mfma6_parked(dW1p[mb], ah, al, bh, bl);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // ---- gradient of the prior's channels, transposed: dF^T[point][channel] = dZ1^T W1 ----
            f32x16 dXp;
#pragma unroll
            for (int s = 0; s < KSH; ++s) {
                Frag th, tl;
                load_operand(block(L::T1P + s * 128), lane, th, tl);
                dXp = s == 0 ? mfma3_first(gz_h[0][s], gz_l[0][s], th, tl) : mfma3(gz_h[0][s], gz_l[0][s], th, tl, dXp);
            }
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_fence();
            scatter_channels<KIND, CP>(sp.prior, io.d_grid, q.scene, info, dXp, col, grp);
        }

        // ---- per-ray inputs: with s = sum of dZ1 over the ray, dW1 += s x^T and dx = W1^T s ----
        float sz[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            db1[mb] += dbr[mb];
            sz[mb] = dbr[mb] + __shfl_xor(dbr[mb], 32, 64);
        }
        wave_lds_fence();
        if (grp == 0) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) ray_sum[32 * mb + col] = sz[mb];
        }
        // rank-one updates: the only non-zero K index is 0 (element 0 of lane group 0)
#pragma unroll
        for (int be = 0; be < NBE; ++be) {
            Frag bh, bl;
            {
                uint32_t h, l;
                split2(32 * be + col < 48 ? ray_x[32 * be + col] : 0.0f, 0.0f, h, l);
                bh.d[0] = grp == 0 ? h : 0u; bl.d[0] = grp == 0 ? l : 0u;
#pragma unroll
                for (int w = 1; w < 4; ++w) bh.d[w] = bl.d[w] = 0u;
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                Frag ah, al;
                uint32_t h, l;
                split2(sz[mb], 0.0f, h, l);
                ah.d[0] = grp == 0 ? h : 0u; al.d[0] = grp == 0 ? l : 0u;
#pragma unroll
                for (int w = 1; w < 4; ++w) ah.d[w] = al.d[w] = 0u;
                dW1e[mb][be] = mfma3(ah, al, bh, bl, dW1e[mb][be]);
                park(dW1e[mb][be]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        wave_lds_fence();
        {
            // s as an operand over the hidden units, the same in every row
            Frag zh[KSH], zl[KSH];
#pragma unroll
            for (int s = 0; s < KSH; ++s) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = ray_sum[k_hidden(s, grp, e)];
                split8(v, zh[s], zl[s]);
            }
#pragma unroll
            for (int be = 0; be < NBE; ++be) {
                f32x16 dx;
#pragma unroll
                for (int s = 0; s < KSH; ++s) {
                    Frag th, tl;
                    load_operand(block(L::T1E + (be * KSH + s) * 128), lane, th, tl);
                    dx = s == 0 ? mfma3_first(zh[s], zl[s], th, tl) : mfma3(zh[s], zl[s], th, tl, dx);
                }
                const int k = 32 * be + col;
                if (grp == 0 && k < n_in) sp.d_feats[(size_t)ray * n_in + k] = dx[0];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- this wave's record of partial sums ----
    float* rec = io.ws + (size_t)(blockIdx.x * kWaves + wave) * io.ws_stride;
    const int ld0 = m.dims[0];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int out = 32 * mb + d_row(r, grp);
            if (col < CP) rec[m.w_off[0] + out * ld0 + n_in + col] = dW1p[mb][r];
#pragma unroll
            for (int be = 0; be < NBE; ++be) {
                const int cc = caller_column<CP>(CP + 32 * be + col, n_in, n_extra);
                if (cc >= 0) rec[m.w_off[0] + out * ld0 + cc] = dW1e[mb][be][r];
            }
            if constexpr (NH == 2) {
#pragma unroll
                for (int nb = 0; nb < MB; ++nb) rec[m.w_off[1] + out * kHidden + 32 * nb + col] = dW2[mb][nb][r];
            }
        }
#pragma unroll
    for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ch = d_row(r, grp);
            if (ch < CP) rec[m.w_off[NH] + ch * kHidden + 32 * nb + col] = dWo[nb][r];
        }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float s1 = db1[mb] + __shfl_xor(db1[mb], 32, 64);
        if (grp == 0) rec[m.b_off[0] + 32 * mb + col] = s1;
        if constexpr (NH == 2) {
            const float s2 = db2[mb] + __shfl_xor(db2[mb], 32, 64);
            if (grp == 0) rec[m.b_off[1] + 32 * mb + col] = s2;
        }
    }
    {
        const float s = dbo + __shfl_xor(dbo, 32, 64);
        if (grp == 0 && col < CP) rec[m.b_off[NH] + col] = s;
    }
}

template <int KIND, int KSP, int KSE, int NH>
hipError_t launch(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, const BwdIo& io,
                  int n_cu, hipStream_t stream)
{
    constexpr int kLdsBytes = SplatBwdLds<KSP, KSE, NH>::UNITS * 16;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    auto kernel = splat_mfma_bwd_kernel<KIND, KSP, KSE, NH>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int blocks = mfma_bwd_records(n_cu) / kWaves;  // every wave writes a record, busy or not
    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, tgt, m, rays, sp, io,
                       splat_group_multiplier(n_groups));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((m.param_total + 63) / 64), dim3(kReduceThreads), 0, stream,
                       m, io, blocks * kWaves);
    return hipGetLastError();
}

template <int KIND, int KSP, int KSE>
hipError_t by_layers(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, const BwdIo& io,
                     int n_cu, hipStream_t stream)
{
    return m.n_layers == 2 ? launch<KIND, KSP, KSE, 1>(tgt, m, rays, sp, io, n_cu, stream)
                           : launch<KIND, KSP, KSE, 2>(tgt, m, rays, sp, io, n_cu, stream);
}

template <int KIND, int KSP>
hipError_t by_extras(const GridDev& tgt, const MlpDev& m, const RaysDev& rays, const SplatDev& sp, const BwdIo& io,
                     int n_cu, hipStream_t stream)
{
    const int n_extra = sp.n_in + m.n_enc;
    if (n_extra <= 16) return by_layers<KIND, KSP, 1>(tgt, m, rays, sp, io, n_cu, stream);
    if (n_extra <= 32) return by_layers<KIND, KSP, 2>(tgt, m, rays, sp, io, n_cu, stream);
    return by_layers<KIND, KSP, 3>(tgt, m, rays, sp, io, n_cu, stream);
}

}  // namespace

}  // namespace lp
