// Matrix-core backward kernel of the Renderer (Eq. (2), Section 3.4 of the paper).
//
// Same mapping as the forward: a wavefront marches one ray, but from the LAST step to the first
// and in steps of 32 samples (one N block; the per-step state of the backward is twice the
// forward's, and the weight-gradient accumulators stay in registers for the whole kernel).
// Per step it
//   1. recomputes sampling + MLP forward (nothing was stored but one scalar per ray),
//   2. rebuilds the transmittance from the cached optical depth (tau_{q-1} = tau_q - sigma_q Delta,
//      T = exp(-tau): the paper's T_{q-1} = T_q exp(Delta sigma_q) in the log domain) and evaluates
//      Eq. (2) with a suffix scan of w_j a_j over the step plus the carry of later steps,
//   3. back-propagates through the MLP on the matrix cores: input gradients with the transposed
//      weights (dX = W^T dZ, chained in registers like the forward), weight gradients as
//      dW = dZ X^T contracted over the samples.  The contraction needs dZ and X with
//      lane = feature and register = sample; that transposition also runs on the matrix cores:
//      multiplying an operand fragment by a 0/1 selection matrix yields the transposed tensor
//      exactly (every output is one bf16 value times 1), hi and lo parts separately,
//   4. scatters the feature gradient into the grid gradient.  The last contraction is evaluated
//      with its operands swapped, which leaves the feature gradient with lane = channel and
//      register = sample; a lane then walks its samples in ray order, sums the contributions
//      of consecutive samples that fall into the same cell, and the lanes of one corner issue
//      one atomic add per channel on consecutive addresses (whole 64-byte lines).
// The weight-gradient accumulators live in the accumulation registers and are updated there
// (mfma6_parked); every other matrix-core result lands in ordinary vector registers (build flag
// of this file), where the vector ALU post-processes it.  Each wave writes one record of partial
// sums at the end and a second kernel adds the records in a fixed order.
//
// This header holds the kernel and its launcher template.  lp_mfma_bwd.hip instantiates the
// shapes it dispatches to; the instantiations with the highest register pressure (direction
// inputs together with contract coordinates, and the widest decoder variant on a triplane)
// crash the compiler's AGPR-copy rewrite pass under that build flag, so lp_mfma_bwd_b.hip builds
// them without it.
#pragma once
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"

namespace lp {

namespace {

constexpr int kWaves = 4;

template <int KIND, int C, int H, int NH, bool CC, int CG, int GT>
__global__ __launch_bounds__(kWaves * 64) void bwd_mfma_kernel(GridDev g, MlpDev m, RaysDev rays, BwdIo io,
                                                               long long group_mul, long long group_step)
{
    using L = MlpLds<C, H, NH, true, kBwdNB>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    extern __shared__ uint4 lds[];
    stage_mlp<C, H, NH, true, kBwdNB, CG>(lds, m);
    __syncthreads();

    const bool identity = m.feat_act != 0;   // rendered features without the sigmoid (two-MLP decoder only)
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* info = reinterpret_cast<float*>(lds + L::END + wave * L::INFO_UNITS * (kRecordDwords<KIND> / 16));

    // selection operands: hidden tensors (two K-steps per 32-feature block), output gradients,
    // input features
    const Frag sel_h0 = selection(col, grp, [](int gg, int e) { return k_hidden(0, gg, e); });
    const Frag sel_h1 = selection(col, grp, [](int gg, int e) { return k_hidden(1, gg, e); });
    const Frag sel_o = selection(col, grp, [](int gg, int e) { return (gg == 0 && e < 4) ? e : -1; });
    Frag sel_f[KS1];
#pragma unroll
    for (int s = 0; s < KS1; ++s)
        sel_f[s] = selection(col, grp, [s](int gg, int e) { return k_input<C>(s, gg, e); });

    // transposes block nb2 (features 32 nb2 .. +31) of a hidden tensor held as operand fragments
    auto transpose_hidden = [&](const Frag (&xh)[kBwdNB][KSH], const Frag (&xl)[kBwdNB][KSH], int nb2,
                                Frag (&th)[kBwdKS], Frag (&tl)[kBwdKS]) {
        f32x16 dh = mfma1(xh[0][2 * nb2], sel_h0, zero16());
        dh = mfma1(xh[0][2 * nb2 + 1], sel_h1, dh);
        f32x16 dl = mfma1(xl[0][2 * nb2], sel_h0, zero16());
        dl = mfma1(xl[0][2 * nb2 + 1], sel_h1, dl);
        pack_exact(dh, th);
        pack_exact(dl, tl);
    };
    // gradient accumulators, alive for the whole kernel
    f32x16 dW1[MB];           // [H x C]   block mb, columns = input channels
    f32x16 dW2[MB][MB];       // [H x H]   (NH == 2)
    f32x16 dWo[MB];           // [4 (of 32) x H], column block nb
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        dW1[mb] = zero16();
        dWo[mb] = zero16();
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) dW2[mb][nb] = zero16();
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        park(dW1[mb]);
        park(dWo[mb]);
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) park(dW2[mb][nb]);
    }
    float db1[MB], db2[MB];
    float dbo[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) db1[mb] = db2[mb] = 0.0f;

    // Rays are taken in groups of kWaves neighbours (one per wave of a workgroup), and the groups
    // in a scrambled order: neighbouring rays add into the same lines of the grid gradient, and
    // atomic adds of many waves to one line queue up behind each other at its L2 channel.
    // Workgroup (xcd, b) visits the group sequence numbers xcd_begin + b, + blocks_per_xcd, ...;
    // sequence number s stands for group (s * mul) mod n_groups, advanced incrementally
    // (group_step = blocks_per_xcd * mul mod n_groups) so that the loop needs no division.
    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    const int S = rays.S;
    const int j_last = ((S - 1) / kBwdStep) * kBwdStep;
    const int blocks_per_xcd = gridDim.x / 8;
    const long long per_xcd = (n_groups + 7) / 8;
    const long long seq_begin = per_xcd * (blockIdx.x % 8) + blockIdx.x / 8;
    const long long seq_last = min(per_xcd * (blockIdx.x % 8 + 1), n_groups);   // end of this XCD's range
    struct Cursor { long long seq, group; };
    auto ray_of = [&](const Cursor& c) { return c.group * kWaves + wave; };
    // next position of this wave that stands for a ray (the last group may be padded)
    auto advance = [&](Cursor c) {
        do {
            c.seq += blocks_per_xcd;
            c.group += group_step;
            if (c.group >= n_groups) c.group -= n_groups;
        } while (c.seq < seq_last && ray_of(c) >= rays.M);
        return c;
    };
    Cursor cur = {seq_begin, seq_begin < seq_last ? (seq_begin * group_mul) % n_groups : 0};
    if (cur.seq < seq_last && ray_of(cur) >= rays.M) cur = advance(cur);

    // Cell and input features of the step about to be processed.  Those of the following step
    // (of this ray, or the last step of the wave's next ray) are sampled while the current
    // step's last contractions run and BEFORE its scatter: the wait for these loads must not
    // come after the scatter's atomic adds (memory operations complete in order, and an atomic
    // add takes much longer than a cached load).
    // Measured: a gain with 16 grid channels (2 to 8 %), a loss with 32 (7 % on eight 256^2
    // triplanes, a factor 2.5 on a 160^3 voxel grid with contract coordinates, where the scatter
    // has 16 lines per sample in flight); with 32 channels a step samples its own features at
    // its start.
    constexpr bool kPrefetch = CG == 16;
    RayGeom q_next;
    Cell3 cell;
    Frag fh[KS1], fl[KS1];
    if (cur.seq < seq_last) {  // a wave without rays only writes its (zero) record
        q_next = load_ray_geom(rays, ray_of(cur));
        if constexpr (CG != C) set_direction_inputs(m, q_next);
        if constexpr (kPrefetch) {
            cell = sample_cell_for<CC, GT>(g, q_next, min(j_last + slot_to_sample(col), S - 1));
            sample_features<KIND, C, CG, GT>(g, q_next, cell, grp, fh, fl);
        }
    }

    while (cur.seq < seq_last) {
        const long long ray = ray_of(cur);
        const RayGeom q = q_next;
        cur = advance(cur);
        if (cur.seq < seq_last) {  // else: a harmless re-sample of this ray
            q_next = load_ray_geom(rays, ray_of(cur));
            if constexpr (CG != C) set_direction_inputs(m, q_next);
        }
        const float p0 = io.d_rgb[3 * ray + 0], p1 = io.d_rgb[3 * ray + 1], p2 = io.d_rgb[3 * ray + 2];
        const float p_alpha = io.d_alpha ? io.d_alpha[ray] : 0.0f;
        const float p_depth = io.d_depth ? io.d_depth[ray] : 0.0f;
        const float tau_S = io.cache[ray];
        // d(loss)/dT_S through alpha = 1 - T_S and rgb += T_S bg, times T_S
        const float kS = __expf(-tau_S) * (p_alpha - (p0 * io.bg[0] + p1 * io.bg[1] + p2 * io.bg[2]));
        float tau_end = tau_S;  // optical depth up to the end of the current step
        float carry = 0.0f;     // sum of w_j a_j over all later steps

        for (int j0 = j_last; j0 >= 0; j0 -= kBwdStep) {
            if constexpr (!kPrefetch) {
                cell = sample_cell_for<CC, GT>(g, q, min(j0 + slot_to_sample(col), S - 1));
                sample_features<KIND, C, CG, GT>(g, q, cell, grp, fh, fl);
            }
            StepActs<C, H, NH, kBwdNB> a;
            a.cell[0] = cell;
#pragma unroll
            for (int s = 0; s < KS1; ++s) { a.fh[0][s] = fh[s]; a.fl[0][s] = fl[s]; }
            mlp_forward<C, H, NH, true, kBwdNB>(lds, lane, a);

            // ---- emission-absorption backward; MFMA column col stands for sample
            //      j0 + slot_to_sample(col) (both lane groups alike), so the scans along the
            //      ray run on values moved into sample order and their results are moved back ----
            const int to_slot = sample_to_slot(col), to_smp = slot_to_sample(col);
            const int j = j0 + to_smp;
            const bool valid = j < S;
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const float sd = valid ? fast_softplus(a.z[0]) * q.delta : 0.0f;
            const float incl_ord = group_scan_incl<kBwdStep>(__shfl(sd, to_slot, kBwdStep), col);
            const float incl = __shfl(incl_ord, to_smp, kBwdStep);
            const float tau_start = tau_end - __shfl(incl_ord, kBwdStep - 1, kBwdStep);
            const float Tprev = __expf(-(tau_start + (incl - sd)));
            const float w = Tprev * one_minus_exp_neg(sd);
            const float Tq = Tprev - w;
            const float c1 = feature_head(a.z[1], identity), c2 = feature_head(a.z[2], identity), c3 = feature_head(a.z[3], identity);
            const float aa = p0 * c1 + p1 * c2 + p2 * c3 + p_depth * t;
            const float wa = w * aa;
            const float wa_ord = __shfl(wa, to_slot, kBwdStep);
            const float pre_ord = group_scan_incl<kBwdStep>(wa_ord, col);
            const float wa_total = __shfl(pre_ord, kBwdStep - 1, kBwdStep);
            const float suf = __shfl(wa_total - pre_ord + wa_ord, to_smp, kBwdStep);
            const float dsigma = q.delta * (Tq * aa - (suf - wa + carry) + kS);
            carry += wa_total;
            tau_end = tau_start;
            float dz[4];
            dz[0] = valid ? dsigma * fast_logistic(a.z[0]) : 0.0f;
            dz[1] = valid ? w * p0 * feature_head_slope(c1, identity) : 0.0f;
            dz[2] = valid ? w * p1 * feature_head_slope(c2, identity) : 0.0f;
            dz[3] = valid ? w * p2 * feature_head_slope(c3, identity) : 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) dbo[k] += grp == 0 ? dz[k] : 0.0f;

            uint32_t zh0, zl0, zh1, zl1;
            split2(dz[0], dz[1], zh0, zl0);
            split2(dz[2], dz[3], zh1, zl1);
            Frag gzo_h[kBwdNB][1], gzo_l[kBwdNB][1];
            {
                const bool mine = grp == 0;
                gzo_h[0][0].d[0] = mine ? zh0 : 0u; gzo_h[0][0].d[1] = mine ? zh1 : 0u;
                gzo_h[0][0].d[2] = 0u; gzo_h[0][0].d[3] = 0u;
                gzo_l[0][0].d[0] = mine ? zl0 : 0u; gzo_l[0][0].d[1] = mine ? zl1 : 0u;
                gzo_l[0][0].d[2] = 0u; gzo_l[0][0].d[3] = 0u;
            }
            // scatter record of this lane's sample, read at the end of the step
            wave_lds_fence();
            if (grp == 0) write_scatter_record<KIND, CG>(info + col * kRecordDwords<KIND>, g, a.cell[0], q.time);

            const Frag (&lh)[kBwdNB][KSH] = NH == 2 ? a.h2h : a.h1h;  // last hidden layer's activations
            const Frag (&ll)[kBwdNB][KSH] = NH == 2 ? a.h2l : a.h1l;

            // ---- output layer: dWo += dZo * Hlast^T over the samples of the step ;
            //      last hidden layer: dZ = relu'(.) * (Wout^T dZo) ----
            f32x16 acc[MB][kBwdNB];
            layer_mfma<MB, 1, kBwdNB, true>(acc, lds + L::T3, lane, gzo_h, gzo_l);
            {
                Frag ah[kBwdKS], al[kBwdKS];
                pack_exact(mfma1(gzo_h[0][0], sel_o, zero16()), ah);
                pack_exact(mfma1(gzo_l[0][0], sel_o, zero16()), al);
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) {
                    Frag bh[kBwdKS], bl[kBwdKS];
                    transpose_hidden(lh, ll, nb2, bh, bl);
                    mfma6_parked(dWo[nb2], ah, al, bh, bl);
                }
            }
            relu_mask<MB>(acc, lh);
            Frag gz_h[kBwdNB][KSH], gz_l[kBwdNB][KSH];
            to_operands<MB, false, kBwdNB>(acc, gz_h, gz_l);
            __builtin_amdgcn_sched_barrier(0);

            // the next step's texel loads are issued here, before the contractions of the hidden
            // layers, and interpolated after them, so that their latency passes under that work
            // (measured: 66.1 -> 63.6 ms on the largest config; issued a stage earlier they cost more
            // in displaced registers than they hide).  Voxel grids only: the 12 corners of a triplane
            // sample are half as many registers again, which the compiler does not survive.
            constexpr bool kEarly = kPrefetch && CG == C && KIND == LP_GRID_VOXEL;
            GatherRaw<KIND, C / 2, GT> raw_next;
            Cell3 cell_next;
            if constexpr (kEarly) {
                const bool same = j0 > 0;
                const RayGeom& qn = same ? q : q_next;
                cell_next = sample_cell_for<CC, GT>(g, qn, min((same ? j0 - kBwdStep : j_last) + slot_to_sample(col), S - 1));
                gather_issue<KIND, C, C / 2, GT>(g, qn.scene, cell_next, grp * (C / 2), raw_next);
                __builtin_amdgcn_sched_barrier(0);
            }

            if constexpr (NH == 2) {
                // ---- dW2 += dZ2 * H1^T ; db2 += sum dZ2 ; dZ1 = relu'(.) * (W2^T dZ2) ----
                Frag ah[MB][kBwdKS], al[MB][kBwdKS];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    transpose_hidden(gz_h, gz_l, mb, ah[mb], al[mb]);
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) db2[mb] = frag_sum(al[mb][ks], frag_sum(ah[mb][ks], db2[mb]));
                }
                layer_mfma<MB, KSH, kBwdNB, true>(acc, lds + L::T2, lane, gz_h, gz_l);
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) {
                    Frag bh[kBwdKS], bl[kBwdKS];
                    transpose_hidden(a.h1h, a.h1l, nb2, bh, bl);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        mfma6_parked(dW2[mb][nb2], ah[mb], al[mb], bh, bl);
                    }
                }
                relu_mask<MB>(acc, a.h1h);
                to_operands<MB, false, kBwdNB>(acc, gz_h, gz_l);
                __builtin_amdgcn_sched_barrier(0);
            }

            // ---- first layer: dW1 += dZ1 * F^T ; db1 += sum dZ1 ; feature gradient, transposed:
            //      dF^T[sample][channel] = dZ1^T W1 ; meanwhile the sampling of the next step ----
            {
                Frag bh[kBwdKS], bl[kBwdKS];
                {
                    f32x16 dh = mfma1(a.fh[0][0], sel_f[0], zero16());
                    f32x16 dl = mfma1(a.fl[0][0], sel_f[0], zero16());
#pragma unroll
                    for (int s = 1; s < KS1; ++s) {
                        dh = mfma1(a.fh[0][s], sel_f[s], dh);
                        dl = mfma1(a.fl[0][s], sel_f[s], dl);
                    }
                    pack_exact(dh, bh);
                    pack_exact(dl, bl);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    Frag ah[kBwdKS], al[kBwdKS];
                    transpose_hidden(gz_h, gz_l, mb, ah, al);
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) db1[mb] = frag_sum(al[ks], frag_sum(ah[ks], db1[mb]));
                    mfma6_parked(dW1[mb], ah, al, bh, bl);
                }
            }
            f32x16 dFt;
#pragma unroll
            for (int s = 0; s < KSH; ++s) {
                Frag th, tl;
                load_operand(lds + L::T1 + s * 128, lane, th, tl);
                dFt = s == 0 ? mfma3_first(gz_h[0][s], gz_l[0][s], th, tl) : mfma3(gz_h[0][s], gz_l[0][s], th, tl, dFt);
            }
            if constexpr (kEarly) {
                __builtin_amdgcn_sched_barrier(0);
                float feat[C / 2];
                gather_finish<KIND, C / 2, GT>(cell_next, raw_next, feat);
#pragma unroll
                for (int s = 0; s < KS1; ++s) split8(feat + 8 * s, fh[s], fl[s]);
                cell = cell_next;
                // the sampled features must be complete here (not sunk below the scatter)
#pragma unroll
                for (int s = 0; s < KS1; ++s)
#pragma unroll
                    for (int w = 0; w < 4; ++w) asm volatile("" : "+v"(fh[s].d[w]), "+v"(fl[s].d[w]));
            } else if constexpr (kPrefetch) {
                // cell of the next step of this ray, or of the last step of the next ray
                const bool same = j0 > 0;
                const RayGeom& qn = same ? q : q_next;
                cell = sample_cell_for<CC, GT>(g, qn, min((same ? j0 - kBwdStep : j_last) + slot_to_sample(col), S - 1));
                __builtin_amdgcn_sched_barrier(0);
                sample_features<KIND, C, CG, GT>(g, qn, cell, grp, fh, fl);
                // the sampled features must be complete here (not sunk below the scatter)
#pragma unroll
                for (int s = 0; s < KS1; ++s)
#pragma unroll
                    for (int w = 0; w < 4; ++w) asm volatile("" : "+v"(fh[s].d[w]), "+v"(fl[s].d[w]));
            }
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_fence();
            scatter_channels<KIND, CG>(g, io.d_grid, q.scene, info, dFt, col, grp, io.d_grid_t);
        }
    }

    // ---- this wave's record of partial sums ----
    float* rec = io.ws + (size_t)(blockIdx.x * kWaves + wave) * io.ws_stride;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int out = 32 * mb + d_row(r, grp);
            if (col < C) rec[m.w_off[0] + out * C + col] = dW1[mb][r];
            if constexpr (NH == 2) {
#pragma unroll
                for (int nb = 0; nb < MB; ++nb) rec[m.w_off[1] + out * H + 32 * nb + col] = dW2[mb][nb][r];
            }
        }
#pragma unroll
    for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (grp == 0) rec[m.w_off[NH] + r * H + 32 * nb + col] = dWo[nb][r];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float s1 = db1[mb] + __shfl_xor(db1[mb], 32, 64);
        if (grp == 0) rec[m.b_off[0] + 32 * mb + col] = s1;
        if constexpr (NH == 2) {
            const float s2 = db2[mb] + __shfl_xor(db2[mb], 32, 64);
            if (grp == 0) rec[m.b_off[1] + 32 * mb + col] = s2;
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float s = wave_sum(dbo[k]);
        if (lane == 0) rec[m.b_off[NH] + k] = s;
    }
}

template <int KIND, int C, int H, int NH, bool CC, int CG, int GT = LP_F32>
hipError_t launch_bwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                       hipStream_t stream)
{
    using L = MlpLds<C, H, NH, true, kBwdNB>;
    constexpr int kLdsBytes = L::bytes(kWaves) + kWaves * L::INFO_UNITS * (kRecordDwords<KIND> / 16 - 1) * 16;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    auto kernel = bwd_mfma_kernel<KIND, C, H, NH, CC, CG, GT>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int blocks = mfma_bwd_records(n_cu) / kWaves;  // every wave writes a record, busy or not
    // multiplier of the ray-group scramble: a prime that does not divide the number of groups,
    // so that group -> group * mul mod n_groups is a bijection
    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    long long group_mul = 1;
    for (long long p : {7919LL, 7907LL, 7901LL, 7883LL})
        if (n_groups > p && n_groups % p != 0) { group_mul = p; break; }
    const long long group_step = ((long long)(blocks / 8) * group_mul) % n_groups;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, m, rays, io,
                       group_mul, group_step);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((m.param_total + 63) / 64), dim3(kReduceThreads), 0, stream,
                       m, io, blocks * kWaves);
    return hipGetLastError();
}

}  // namespace

}  // namespace lp
