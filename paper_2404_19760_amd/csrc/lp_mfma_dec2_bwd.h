// Backward of the Renderer with the paper's two-MLP decoder at its experimental size (see
// lp_mfma_dec2.h), in two passes over the rays.
//
// The weight-gradient accumulators of ONE 3-layer MLP of width 64 fill half of a wavefront's
// registers (the single-MLP backward kernel keeps them there for the whole kernel); those of two
// do not fit beside the working set of a step.  So the backward runs twice, recomputing the
// forward each time as Section 3.4 prescribes anyway:
//   pass 0 accumulates the opacity MLP's gradients and scatters the feature gradient of BOTH
//          chains into the grid gradient (the feature chain's input-gradient chain runs without
//          its weight-gradient contractions);
//   pass 1 accumulates the feature MLP's gradients and scatters nothing.  The direction inputs
//          are constant along a ray: with s = the ray's sum of dZ1, their weight gradient is
//          s enc(d)^T, one rank-one matrix-core update per ray.
// A step runs both chains forward, evaluates the emission-absorption backward (Eq. (2)), then
// the backward of the chain whose weight gradients the pass accumulates, on that chain's live
// activations.  In pass 0 the feature chain also has to pass its input gradient on; for that its
// backward needs only the ReLU masks of its hidden layers, i.e. the high halves of their
// activation fragments (32 registers), which are kept across the opacity chain's work.
// Each pass writes one record of partial sums per wave and is followed by the reduction kernel.
#pragma once
#include "lp_mfma_bwd_common.h"
#include "lp_mfma_dec2.h"

namespace lp {

namespace {

using dec2::kH;
using dec2::kWaves;

// gradient accumulators of one chain, alive for a whole pass
template <int C>
struct ChainGrads {
    f32x16 dW1[2];      // [64 x C]   row block mb, columns = grid channels
    f32x16 dW2[2][2];   // [64 x 64]
    f32x16 dWo[2];      // [4 (of 32) x 64], column block nb
    float db1[2], db2[2], dbo[4];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            dW1[mb] = zero16(); park(dW1[mb]);
            dWo[mb] = zero16(); park(dWo[mb]);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) { dW2[mb][nb] = zero16(); park(dW2[mb][nb]); }
            db1[mb] = db2[mb] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) dbo[k] = 0.0f;
    }
};

struct SelFrags {
    Frag h0, h1, o, f[2];
};

// transposes block nb2 (features 32 nb2 .. +31) of a hidden tensor held as operand fragments
__device__ __forceinline__ void transpose_hidden(const SelFrags& sel, const Frag (&xh)[1][4], const Frag (&xl)[1][4],
                                                 int nb2, Frag (&th)[kBwdKS], Frag (&tl)[kBwdKS])
{
    f32x16 dh = mfma1(xh[0][2 * nb2], sel.h0, zero16());
    dh = mfma1(xh[0][2 * nb2 + 1], sel.h1, dh);
    f32x16 dl = mfma1(xl[0][2 * nb2], sel.h0, zero16());
    dl = mfma1(xl[0][2 * nb2 + 1], sel.h1, dl);
    pack_exact(dh, th);
    pack_exact(dl, tl);
}

// Backward of one chain for one step.  `cl` = the chain's weights in LDS, `a` = its forward of
// this step, gzo = the output gradients (all four rows; the chain's transposed last layer picks
// its own).  ACC: contract the weight gradients into G (else only the input-gradient chain
// runs).  WANT_DF: add the chain's feature gradient (lane = channel, register = sample) to dFt
// (started when first_df).  ray_db1, if not NULL: also add this step's sum of dZ1 there.
template <int C, bool ACC, bool WANT_DF>
__device__ __forceinline__ void chain_backward(const uint4* cl, int lane, const SelFrags& sel,
                                               const StepActs<C, kH, 2, 1>& a, const Frag (&gzo_h)[1][1],
                                               const Frag (&gzo_l)[1][1], ChainGrads<C>& G, f32x16& dFt, bool first_df,
                                               float* ray_db1)
{
    using L = MlpLds<C, kH, 2, true, 1>;
    constexpr int MB = 2, KS1 = C / 16, KSH = 4;
    // ---- output layer ----
    f32x16 acc[MB][1];
    layer_mfma<MB, 1, 1, true>(acc, cl + L::T3, lane, gzo_h, gzo_l);
    if constexpr (ACC) {
        Frag ah[kBwdKS], al[kBwdKS];
        pack_exact(mfma1(gzo_h[0][0], sel.o, zero16()), ah);
        pack_exact(mfma1(gzo_l[0][0], sel.o, zero16()), al);
#pragma unroll
        for (int nb2 = 0; nb2 < MB; ++nb2) {
            Frag bh[kBwdKS], bl[kBwdKS];
            transpose_hidden(sel, a.h2h, a.h2l, nb2, bh, bl);
            mfma6_parked(G.dWo[nb2], ah, al, bh, bl);
        }
    }
    relu_mask<MB>(acc, a.h2h);
    Frag gz_h[1][KSH], gz_l[1][KSH];
    to_operands<MB, false, 1>(acc, gz_h, gz_l);
    __builtin_amdgcn_sched_barrier(0);

    // ---- second hidden layer ----
    if constexpr (ACC) {
        Frag ah[MB][kBwdKS], al[MB][kBwdKS];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            transpose_hidden(sel, gz_h, gz_l, mb, ah[mb], al[mb]);
#pragma unroll
            for (int ks = 0; ks < kBwdKS; ++ks) G.db2[mb] = frag_sum(al[mb][ks], frag_sum(ah[mb][ks], G.db2[mb]));
        }
        layer_mfma<MB, KSH, 1, true>(acc, cl + L::T2, lane, gz_h, gz_l);
#pragma unroll
        for (int nb2 = 0; nb2 < MB; ++nb2) {
            Frag bh[kBwdKS], bl[kBwdKS];
            transpose_hidden(sel, a.h1h, a.h1l, nb2, bh, bl);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                mfma6_parked(G.dW2[mb][nb2], ah[mb], al[mb], bh, bl);
            }
        }
    } else {
        layer_mfma<MB, KSH, 1, true>(acc, cl + L::T2, lane, gz_h, gz_l);
    }
    relu_mask<MB>(acc, a.h1h);
    to_operands<MB, false, 1>(acc, gz_h, gz_l);
    __builtin_amdgcn_sched_barrier(0);

    // ---- first layer ----
    if constexpr (ACC) {
        Frag bh[kBwdKS], bl[kBwdKS];
        {
            f32x16 dh = mfma1(a.fh[0][0], sel.f[0], zero16());
            f32x16 dl = mfma1(a.fl[0][0], sel.f[0], zero16());
#pragma unroll
            for (int s = 1; s < KS1; ++s) {
                dh = mfma1(a.fh[0][s], sel.f[s], dh);
                dl = mfma1(a.fl[0][s], sel.f[s], dl);
            }
            pack_exact(dh, bh);
            pack_exact(dl, bl);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            Frag ah[kBwdKS], al[kBwdKS];
            transpose_hidden(sel, gz_h, gz_l, mb, ah, al);
            float sum = 0.0f;
#pragma unroll
            for (int ks = 0; ks < kBwdKS; ++ks) sum = frag_sum(al[ks], frag_sum(ah[ks], sum));
            G.db1[mb] += sum;
            if (ray_db1) ray_db1[mb] += sum;
            mfma6_parked(G.dW1[mb], ah, al, bh, bl);
        }
    }
    if constexpr (WANT_DF) {
#pragma unroll
        for (int s = 0; s < KSH; ++s) {
            Frag th, tl;
            load_operand(cl + L::T1 + s * 128, lane, th, tl);
            dFt = (first_df && s == 0) ? mfma3_first(gz_h[0][s], gz_l[0][s], th, tl)
                                       : mfma3(gz_h[0][s], gz_l[0][s], th, tl, dFt);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

// one chain's record of partial sums: W1 [64][ld1] (grid columns 0 .. C-1), W2, Wo rows
// first_row .. first_row + n_out - 1 of the four, the biases
template <int C>
__device__ __forceinline__ void write_chain_record(float* rec, const MlpDev& m, const ChainGrads<C>& G, int lane,
                                                   int n_out, int first_row)
{
    const int col = lane & 31, grp = lane >> 5;
    const int ld1 = m.dims[0];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int out = 32 * mb + d_row(r, grp);
            if (col < C) rec[m.w_off[0] + out * ld1 + col] = G.dW1[mb][r];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) rec[m.w_off[1] + out * kH + 32 * nb + col] = G.dW2[mb][nb][r];
        }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (grp == 0 && r >= first_row && r < first_row + n_out)
                rec[m.w_off[2] + (r - first_row) * kH + 32 * nb + col] = G.dWo[nb][r];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const float s1 = G.db1[mb] + __shfl_xor(G.db1[mb], 32, 64);
        const float s2 = G.db2[mb] + __shfl_xor(G.db2[mb], 32, 64);
        if (grp == 0) {
            rec[m.b_off[0] + 32 * mb + col] = s1;
            rec[m.b_off[1] + 32 * mb + col] = s2;
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float s = wave_sum(G.dbo[k]);
        if (lane == 0 && k >= first_row && k < first_row + n_out) rec[m.b_off[2] + k - first_row] = s;
    }
}

// PASS 0: opacity MLP's gradients + grid gradient; PASS 1: feature MLP's gradients.
// m = the pass's MLP (offsets of its record); io.dW / io.db are not used here.
template <int KIND, int C, bool CC, int PASS>
__global__ __launch_bounds__(kWaves * 64) void dec2_bwd_kernel(GridDev g, Dec2Dev d, MlpDev m, RaysDev rays, BwdIo io,
                                                               long long group_mul)
{
    using L = dec2::Lds<C, true, 1>;
    using CL = typename L::Chain;
    constexpr int KS1 = C / 16;
    extern __shared__ uint4 lds[];
    dec2::stage_decoder<C, true, 1>(lds, d);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint4* lds_s = lds + L::S;
    const uint4* lds_v = lds + L::V;
    uint4* wave_area = lds + L::WAVE + wave * L::W_UNITS;
    const float* bias_v = reinterpret_cast<const float*>(wave_area + L::W_BIAS);
    const float* ray_x = reinterpret_cast<const float*>(wave_area + L::W_X);
    float* info = reinterpret_cast<float*>(lds + L::END + wave * CL::INFO_UNITS);

    SelFrags sel;
    sel.h0 = selection(col, grp, [](int gg, int e) { return k_hidden(0, gg, e); });
    sel.h1 = selection(col, grp, [](int gg, int e) { return k_hidden(1, gg, e); });
    sel.o = selection(col, grp, [](int gg, int e) { return (gg == 0 && e < 4) ? e : -1; });
#pragma unroll
    for (int s = 0; s < KS1; ++s) sel.f[s] = selection(col, grp, [s](int gg, int e) { return k_input<C>(s, gg, e); });

    ChainGrads<C> G;
    G.clear();
    f32x16 dW1e[2];   // PASS 1: [64 x direction inputs]
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) { dW1e[mb] = zero16(); park(dW1e[mb]); }

    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    const RaySchedule sched = ray_schedule(n_groups * kWaves, kWaves);
    const int S = rays.S;
    const int j_last = ((S - 1) / kBwdStep) * kBwdStep;
    for (long long seq = sched.first; seq < sched.end; seq += sched.stride) {
        const long long ray = ((seq / kWaves) * group_mul % n_groups) * kWaves + seq % kWaves;
        if (ray >= rays.M) continue;
        const RayGeom q = load_ray_geom(rays, ray);
        dec2::ray_direction_bias<C, true, 1>(lds, d, q, lane, wave);
        const float p0 = io.d_rgb[3 * ray + 0], p1 = io.d_rgb[3 * ray + 1], p2 = io.d_rgb[3 * ray + 2];
        const float p_alpha = io.d_alpha ? io.d_alpha[ray] : 0.0f;
        const float p_depth = io.d_depth ? io.d_depth[ray] : 0.0f;
        const float tau_S = io.cache[ray];
        // d(loss)/dT_S through alpha = 1 - T_S and rgb += T_S bg, times T_S
        const float kS = __expf(-tau_S) * (p_alpha - (p0 * io.bg[0] + p1 * io.bg[1] + p2 * io.bg[2]));
        float tau_end = tau_S;  // optical depth up to the end of the current step
        float carry = 0.0f;     // sum of w_j a_j over all later steps
        float ray_db1[2] = {0.0f, 0.0f};  // PASS 1: the ray's sum of the feature chain's dZ1
        __builtin_amdgcn_sched_barrier(0);

        for (int j0 = j_last; j0 >= 0; j0 -= kBwdStep) {
            StepActs<C, kH, 2, 1> a;
            const int to_slot = sample_to_slot(col), to_smp = slot_to_sample(col);
            const int j = j0 + to_smp;
            const bool valid = j < S;
            a.cell[0] = sample_cell<CC>(g, q, min(j, S - 1));
            sample_features<KIND, C, C, kAnyDtype>(g, q, a.cell[0], grp, a.fh[0], a.fl[0]);
            if constexpr (PASS == 0) {
                wave_lds_fence();
                if (grp == 0) write_scatter_record<KIND, C>(info + col * 16, g, a.cell[0]);
            }
            // ---- both chains forward for the decoder outputs ----
            // PASS 0: the feature chain first; of its activations only the high halves of the two
            // hidden layers are kept (its backward here needs nothing but their ReLU masks), then the
            // opacity chain, whose activations stay alive for its weight gradients.
            // PASS 1: the opacity chain for its output only, then the feature chain, which stays alive.
            float z[4];
            StepActs<C, kH, 2, 1> masks_v;   // PASS 0: h1h / h2h of the feature chain
            if constexpr (PASS == 0) {
                mlp_forward<C, kH, 2, true, 1>(lds_v, lane, a, bias_v);
                z[1] = a.z[1]; z[2] = a.z[2]; z[3] = a.z[3];
#pragma unroll
                for (int s = 0; s < 4; ++s) { masks_v.h1h[0][s] = a.h1h[0][s]; masks_v.h2h[0][s] = a.h2h[0][s]; }
                __builtin_amdgcn_sched_barrier(0);
                mlp_forward<C, kH, 2, true, 1>(lds_s, lane, a);
                z[0] = a.z[0];
            } else {
                mlp_forward<C, kH, 2, true, 1>(lds_s, lane, a);
                z[0] = a.z[0];
                __builtin_amdgcn_sched_barrier(0);
                mlp_forward<C, kH, 2, true, 1>(lds_v, lane, a, bias_v);
                z[1] = a.z[1]; z[2] = a.z[2]; z[3] = a.z[3];
            }
            __builtin_amdgcn_sched_barrier(0);

            // ---- emission-absorption backward; MFMA column col stands for sample
            //      j0 + slot_to_sample(col) (both lane groups alike) ----
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const float sd = valid ? fast_softplus(z[0]) * q.delta : 0.0f;
            const float incl_ord = group_scan_incl<kBwdStep>(__shfl(sd, to_slot, kBwdStep), col);
            const float incl = __shfl(incl_ord, to_smp, kBwdStep);
            const float tau_start = tau_end - __shfl(incl_ord, kBwdStep - 1, kBwdStep);
            const float Tprev = __expf(-(tau_start + (incl - sd)));
            const float w = Tprev * one_minus_exp_neg(sd);
            const float Tq = Tprev - w;
            const bool identity = d.feat_act != 0;
            const float c1 = feature_head(z[1], identity), c2 = feature_head(z[2], identity), c3 = feature_head(z[3], identity);
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
            dz[0] = valid ? dsigma * fast_logistic(z[0]) : 0.0f;
            dz[1] = valid ? w * p0 * feature_head_slope(c1, identity) : 0.0f;
            dz[2] = valid ? w * p1 * feature_head_slope(c2, identity) : 0.0f;
            dz[3] = valid ? w * p2 * feature_head_slope(c3, identity) : 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) G.dbo[k] += grp == 0 ? dz[k] : 0.0f;
            Frag gzo_h[1][1], gzo_l[1][1];
            {
                uint32_t zh0, zl0, zh1, zl1;
                split2(dz[0], dz[1], zh0, zl0);
                split2(dz[2], dz[3], zh1, zl1);
                const bool mine = grp == 0;
                gzo_h[0][0].d[0] = mine ? zh0 : 0u; gzo_h[0][0].d[1] = mine ? zh1 : 0u;
                gzo_h[0][0].d[2] = 0u; gzo_h[0][0].d[3] = 0u;
                gzo_l[0][0].d[0] = mine ? zl0 : 0u; gzo_l[0][0].d[1] = mine ? zl1 : 0u;
                gzo_l[0][0].d[2] = 0u; gzo_l[0][0].d[3] = 0u;
            }
            __builtin_amdgcn_sched_barrier(0);

            f32x16 dFt;
            if constexpr (PASS == 0) {
                // the opacity chain's activations are the ones alive: its full backward first, then the
                // feature chain's input-gradient chain from the kept masks
                chain_backward<C, true, true>(lds_s, lane, sel, a, gzo_h, gzo_l, G, dFt, true, nullptr);
                chain_backward<C, false, true>(lds_v, lane, sel, masks_v, gzo_h, gzo_l, G, dFt, false, nullptr);
                wave_lds_fence();
                scatter_channels<KIND, C>(g, io.d_grid, q.scene, info, dFt, col, grp);
            } else {
                chain_backward<C, true, false>(lds_v, lane, sel, a, gzo_h, gzo_l, G, dFt, true, ray_db1);
            }
        }
        if constexpr (PASS == 1) {
            // direction columns of the first layer: dW1 += s enc(d)^T with s = the ray's sum of
            // dZ1; the only non-zero K index is 0 (element 0 of lane group 0)
            Frag bh, bl;
            {
                uint32_t h, l;
                split2(ray_x[col], 0.0f, h, l);
                bh.d[0] = grp == 0 ? h : 0u; bl.d[0] = grp == 0 ? l : 0u;
#pragma unroll
                for (int w = 1; w < 4; ++w) bh.d[w] = bl.d[w] = 0u;
            }
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                const float sz = ray_db1[mb] + __shfl_xor(ray_db1[mb], 32, 64);
                Frag ah, al;
                uint32_t h, l;
                split2(sz, 0.0f, h, l);
                ah.d[0] = grp == 0 ? h : 0u; al.d[0] = grp == 0 ? l : 0u;
#pragma unroll
                for (int w = 1; w < 4; ++w) ah.d[w] = al.d[w] = 0u;
                dW1e[mb] = mfma3(ah, al, bh, bl, dW1e[mb]);
                park(dW1e[mb]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- this wave's record of partial sums ----
    float* rec = io.ws + (size_t)(blockIdx.x * kWaves + wave) * io.ws_stride;
    if constexpr (PASS == 0) {
        write_chain_record<C>(rec, m, G, lane, 1, 0);
    } else {
        write_chain_record<C>(rec, m, G, lane, 3, 1);
        const int ld1 = m.dims[0];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (col < d.E) rec[m.w_off[0] + (32 * mb + d_row(r, grp)) * ld1 + C + col] = dW1e[mb][r];
    }
}

template <int KIND, int C, bool CC>
hipError_t launch_dec2_bwd_t(const GridDev& g, const Dec2Dev& d, const MlpDev& ms, const MlpDev& mv,
                             const RaysDev& rays, const BwdIo& io, int n_cu, hipStream_t stream)
{
    using L = dec2::Lds<C, true, 1>;
    constexpr int kLdsBytes = (L::END + kWaves * L::Chain::INFO_UNITS) * 16;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    const int blocks = mfma_bwd_records(n_cu) / kWaves;  // every wave writes a record, busy or not
    const long long n_groups = (rays.M + kWaves - 1) / kWaves;
    long long group_mul = 1;
    for (long long p : {7919LL, 7907LL, 7901LL, 7883LL})
        if (n_groups > p && n_groups % p != 0) { group_mul = p; break; }
    BwdIo io_s = io, io_v = io;
    for (int l = 0; l < 3; ++l) {
        io_s.dW[l] = d.dWs[l]; io_s.db[l] = d.dbs[l];
        io_v.dW[l] = d.dWv[l]; io_v.db[l] = d.dbv[l];
    }
    auto k0 = dec2_bwd_kernel<KIND, C, CC, 0>;
    auto k1 = dec2_bwd_kernel<KIND, C, CC, 1>;
    hipError_t e = hipFuncSetAttribute((const void*)k0, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)k1, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k0, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, d, ms, rays, io_s, group_mul);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((ms.param_total + 63) / 64), dim3(kReduceThreads), 0, stream, ms,
                       io_s, blocks * kWaves);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // the second pass reuses the records (same stream: the reduction above has read them)
    hipLaunchKernelGGL(k1, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, d, mv, rays, io_v, group_mul);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((mv.param_total + 63) / 64), dim3(kReduceThreads), 0, stream, mv,
                       io_v, blocks * kWaves);
    return hipGetLastError();
}

}  // namespace

}  // namespace lp
