// Matrix-core backward kernel of the Renderer (Eq. (2), Section 3.4 of the paper).
//
// Same mapping as the forward: a wavefront marches one ray, but from the LAST step to the first
// and in steps of 32 samples (one N block; the per-step state of the backward is twice the
// forward's, and the weight-gradient accumulators live in registers for the whole kernel).
// Per step it
//   1. recomputes sampling + MLP forward (nothing was stored but one scalar per ray),
//   2. rebuilds the transmittance from the cached optical depth (tau_{q-1} = tau_q - sigma_q Delta,
//      T = exp(-tau): the paper's T_{q-1} = T_q exp(Delta sigma_q) in the log domain) and evaluates
//      Eq. (2) with a suffix scan of w_j a_j over the step plus the carry of later steps,
//   3. back-propagates through the MLP on the matrix cores: input gradients with the transposed
//      weights (dX = W^T dZ, chained in registers like the forward), weight gradients as
//      dW = dZ X^T contracted over the samples, for which dZ and X are transposed through a
//      per-wave LDS tile (bf16 hi/lo planes, 16-bit stores, 128-bit operand loads),
//   4. scatters the feature gradient into the grid gradient.  The last contraction is evaluated
//      with its operands swapped, which leaves the feature gradient with lane = channel and
//      register = sample; a lane then walks its samples in ray order, sums the contributions
//      of consecutive samples that fall into the same cell, and the lanes of one corner issue
//      one atomic add per channel on consecutive addresses (whole 64-byte lines).
// Weight / bias gradients stay in registers for the whole kernel; each wave writes one record
// of partial sums at the end and a second kernel adds the records in a fixed order.
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"

namespace lp {

namespace {

constexpr int kWaves = 4;
constexpr int kNB = 1;            // N blocks (of 32 samples) per step
constexpr int kStep = 32 * kNB;   // samples per step
constexpr int kKS = 2 * kNB;      // K-steps of a contraction over the samples of a step

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wave execute in order; this only pins the compiler's ordering of
    // the tile stores of some lanes against the tile loads of others
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_sched_barrier(0);
}

template <int RS>
struct Tile {
    uint16_t* hi;
    uint16_t* lo;

    // operand fragments [NB][KS] whose element e of lane-group g is row row_of(s, g, e) of sample
    // column (lane & 31) + 32 nb  ->  tile[row][sample]
    template <int KS, class RowFn>
    __device__ __forceinline__ void store(const Frag (&fh)[kNB][KS], const Frag (&fl)[kNB][KS], int lane,
                                          RowFn row_of) const
    {

        const int col = lane & 31, grp = lane >> 5;
#pragma unroll
        for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const int o0 = row_of(s, grp, 2 * d) * RS + col + 32 * nb;
                    const int o1 = row_of(s, grp, 2 * d + 1) * RS + col + 32 * nb;
                    hi[o0] = (uint16_t)fh[nb][s].d[d];
                    hi[o1] = (uint16_t)(fh[nb][s].d[d] >> 16);
                    lo[o0] = (uint16_t)fl[nb][s].d[d];
                    lo[o1] = (uint16_t)(fl[nb][s].d[d] >> 16);
                }
    }

    // MFMA operand with the samples of the step on the K axis: 8 consecutive samples of `row`
    __device__ __forceinline__ void load(int row, int s, int grp, bool live, Frag& fh, Frag& fl) const
    {

        const uint4 h = *reinterpret_cast<const uint4*>(hi + row * RS + 16 * s + 8 * grp);
        const uint4 l = *reinterpret_cast<const uint4*>(lo + row * RS + 16 * s + 8 * grp);
        fh.d[0] = live ? h.x : 0u; fh.d[1] = live ? h.y : 0u; fh.d[2] = live ? h.z : 0u; fh.d[3] = live ? h.w : 0u;
        fl.d[0] = live ? l.x : 0u; fl.d[1] = live ? l.y : 0u; fl.d[2] = live ? l.z : 0u; fl.d[3] = live ? l.w : 0u;
    }
};

// sum of the 8 bf16 values of a fragment, added to acc
__device__ __forceinline__ float frag_sum(const Frag& f, float acc)
{
    bf16x2 one;
    one[0] = (__bf16)1.0f;
    one[1] = (__bf16)1.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, f.d[d]), one, acc, false);
    return acc;
}

// zeroes the entries of a D block whose ReLU output (hi part of the stored activation) is zero
template <int MB>
__device__ __forceinline__ void relu_mask(f32x16 (&acc)[MB][kNB], const Frag (&act_hi)[kNB][2 * MB])
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int s = 2 * mb + r / 8, e = r % 8;
                const uint32_t bits = (act_hi[nb][s].d[e / 2] >> (16 * (e & 1))) & 0xffffu;
                acc[mb][nb][r] = bits ? acc[mb][nb][r] : 0.0f;
            }
}

// ---- scatter records: what the channel lanes need to know about each sample of the step ----
// 16 dwords per sample.  voxel: 8 corner weights (corner 4dx + 2dy + dz), then the element offset of
// corner 0.  triplane: 12 weights (plane p, corner 2da + db at 4p + ..), then 3 plane offsets.
template <int KIND, int C>
__device__ __forceinline__ void write_scatter_record(float* rec, const GridDev& g, const Cell3& c)
{
    if constexpr (KIND == LP_GRID_VOXEL) {
        const float x1 = c.f[0], x0 = 1.0f - x1, y1 = c.f[1], y0 = 1.0f - y1, z1 = c.f[2], z0 = 1.0f - z1;
        const float4 w0 = make_float4(x0 * y0 * z0, x0 * y0 * z1, x0 * y1 * z0, x0 * y1 * z1);
        const float4 w1 = make_float4(x1 * y0 * z0, x1 * y0 * z1, x1 * y1 * z0, x1 * y1 * z1);
        const unsigned sz = C, sy = (unsigned)g.N[2] * C, sx = (unsigned)g.N[1] * sy;
        const unsigned base = (unsigned)c.i[0] * sx + (unsigned)c.i[1] * sy + (unsigned)c.i[2] * sz;
        reinterpret_cast<float4*>(rec)[0] = w0;
        reinterpret_cast<float4*>(rec)[1] = w1;
        reinterpret_cast<unsigned*>(rec)[8] = base;
    } else {
        unsigned base[3];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            const float a1 = c.f[a], a0 = 1.0f - a1, b1 = c.f[b], b0 = 1.0f - b1;
            reinterpret_cast<float4*>(rec)[p] = make_float4(a0 * b0, a0 * b1, a1 * b0, a1 * b1);
            base[p] = ((unsigned)c.i[a] * (unsigned)g.N[b] + (unsigned)c.i[b]) * C;
        }
        reinterpret_cast<uint4*>(rec)[3] = make_uint4(base[0], base[1], base[2], 0u);
    }
}

// Accumulators of the 2^NBITS corners of the current cell while a lane walks its samples in ray
// order.  When the ray steps into the neighbouring cell along ONE axis, the corners on the
// shared face stay (their sums move to the mirrored corner index) and only the corners left
// behind are added to memory; any other move flushes all corners.
template <int NBITS>
struct CornerAcc {
    static constexpr int N = 1 << NBITS;
    float acc[N];

    // BIT = corner-index bit of the axis stepped along; `up` = towards larger index.
    // flush(d, value) adds `value` to corner d of the OLD cell.
    template <int BIT, class Flush>
    __device__ __forceinline__ void step_axis(bool up, Flush flush)
    {
#pragma unroll
        for (int d = 0; d < N; ++d) {
            if (d & BIT) continue;
            const float lo = acc[d], hi = acc[d | BIT];
            flush(up ? d : (d | BIT), up ? lo : hi);   // the face left behind
            acc[d] = up ? hi : 0.0f;                   // the shared face changes side
            acc[d | BIT] = up ? 0.0f : lo;
        }
    }
};

// This lane (channel `ch` of lane group `grp`) holds in dFt[r] the feature gradient of MFMA
// column d_row(r, grp), which (permuted step) is sample 16 grp + r of the step: 16 consecutive
// samples in ray order.  Contributions are summed per corner while the ray stays in a cell
// (and on shared corners across a step into a neighbouring cell) before one atomic add per
// corner; the lanes ch = 0..C-1 of a group address consecutive floats.
template <int KIND, int C>
__device__ __forceinline__ void scatter_channels(const GridDev& g, float* const d_grid[3], int scene,
                                                 const float* info, const f32x16& dFt, int ch, int grp)
{
    const bool live = ch < C;
    if constexpr (KIND == LP_GRID_VOXEL) {
        // uniform base pointer + 32-bit byte offset per lane (a scene's tensor is below 4 GiB)
        char* V = reinterpret_cast<char*>(d_grid[0] + (size_t)scene * g.N[0] * g.N[1] * g.N[2] * C);
        const unsigned sz = C, sy = (unsigned)g.N[2] * C, sx = (unsigned)g.N[1] * sy;
        CornerAcc<3> ca;
        unsigned prev = 0;
        // one uniform pointer per corner, so that a flush needs a single per-lane offset
        char* Vd[8];
#pragma unroll
        for (int d = 0; d < 8; ++d)
            Vd[d] = V + 4u * (size_t)((d >> 2) * sx + ((d >> 1) & 1) * sy + (d & 1) * sz);
        auto add = [&](int d, float v) {
            if (live) atomicAdd(reinterpret_cast<float*>(Vd[d] + 4u * (prev + ch)), v);
        };
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float* rec = info + d_row(r, grp) * 16;
            const float4 w0 = reinterpret_cast<const float4*>(rec)[0];
            const float4 w1 = reinterpret_cast<const float4*>(rec)[1];
            const unsigned base = reinterpret_cast<const unsigned*>(rec)[8];
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            const float v = dFt[r];
            if (r > 0 && base != prev) {
                // Keeping shared corners across a cell change pays when changes are rare; with a
                // few samples per cell (fine voxel grids) the extra selects cost more than the
                // atomic requests they save (measured), so voxel cells are simply flushed.
                constexpr bool kCarryVoxel = false;
                const bool up = base > prev;
                const unsigned dist = up ? base - prev : prev - base;
                if (kCarryVoxel && dist == sz) ca.template step_axis<1>(up, add);
                else if (kCarryVoxel && dist == sy) ca.template step_axis<2>(up, add);
                else if (kCarryVoxel && dist == sx) ca.template step_axis<4>(up, add);
                else {
#pragma unroll
                    for (int d = 0; d < 8; ++d) { add(d, ca.acc[d]); ca.acc[d] = 0.0f; }
                }
            }
            prev = base;
#pragma unroll
            for (int d = 0; d < 8; ++d) ca.acc[d] = r == 0 ? w[d] * v : ca.acc[d] + w[d] * v;
        }
#pragma unroll
        for (int d = 0; d < 8; ++d) add(d, ca.acc[d]);
    } else {
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
            const int a = pl, b = (pl + 1) % 3;
            char* P = reinterpret_cast<char*>(d_grid[pl] + (size_t)scene * g.N[a] * g.N[b] * C);
            const unsigned sb = C, sa = (unsigned)g.N[b] * C;
            CornerAcc<2> ca;
            unsigned prev = 0;
            char* Pd[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) Pd[d] = P + 4u * (size_t)((d >> 1) * sa + (d & 1) * sb);
            auto add = [&](int d, float v) {
                if (live) atomicAdd(reinterpret_cast<float*>(Pd[d] + 4u * (prev + ch)), v);
            };
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float* rec = info + d_row(r, grp) * 16;
                const float4 w4 = reinterpret_cast<const float4*>(rec)[pl];
                const unsigned base = reinterpret_cast<const unsigned*>(rec)[12 + pl];
                const float w[4] = {w4.x, w4.y, w4.z, w4.w};
                const float v = dFt[r];
                if (r > 0 && base != prev) {
                    const bool up = base > prev;
                    const unsigned dist = up ? base - prev : prev - base;
                    if (dist == sb) ca.template step_axis<1>(up, add);
                    else if (dist == sa) ca.template step_axis<2>(up, add);
                    else {
#pragma unroll
                        for (int d = 0; d < 4; ++d) { add(d, ca.acc[d]); ca.acc[d] = 0.0f; }
                    }
                }
                prev = base;
#pragma unroll
                for (int d = 0; d < 4; ++d) ca.acc[d] = r == 0 ? w[d] * v : ca.acc[d] + w[d] * v;
            }
#pragma unroll
            for (int d = 0; d < 4; ++d) add(d, ca.acc[d]);
        }
    }
}

template <int KIND, int C, int H, int NH>
__global__ __launch_bounds__(kWaves * 64) void bwd_mfma_kernel(GridDev g, MlpDev m, RaysDev rays, BwdIo io)
{
    using L = MlpLds<C, H, NH, true, kNB>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH, RS = L::TILE_RS;
    extern __shared__ uint4 lds[];
    stage_mlp<C, H, NH, true, kNB>(lds, m);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Tile<RS> tile;
    tile.hi = reinterpret_cast<uint16_t*>(lds + L::TILE + wave * L::TILE_UNITS);
    tile.lo = tile.hi + L::TILE_ROWS * RS;
    float* info = reinterpret_cast<float*>(lds + L::TILE + wave * L::TILE_UNITS + 2 * L::TILE_PLANE_UNITS);

    auto hidden_row = [](int s, int gg, int e) { return k_hidden(s, gg, e); };
    auto input_row = [](int s, int gg, int e) { return k_input<C>(s, gg, e); };

    // gradient accumulators, alive for the whole kernel
    f32x16 dW1[MB];           // [H x C]   block mb, columns = input channels
    f32x16 dW2[MB][MB];       // [H x H]   (NH == 2)
    f32x16 dWo[MB];           // [4 (of 32) x H], column block nb
    float db1[MB], db2[MB];   // lane = row within the block (partial over this lane group's samples)
    float dbo[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        db1[mb] = db2[mb] = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dW1[mb][r] = 0.0f;
            dWo[mb][r] = 0.0f;
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) dW2[mb][nb][r] = 0.0f;
        }
    }

    const RaySchedule sched = ray_schedule(rays.M, kWaves);
    const int S = rays.S;

    for (long long ray = sched.first; ray < sched.end; ray += sched.stride) {
        const RayGeom q = load_ray_geom(rays, ray);
        const float p0 = io.d_rgb[3 * ray + 0], p1 = io.d_rgb[3 * ray + 1], p2 = io.d_rgb[3 * ray + 2];
        const float p_alpha = io.d_alpha ? io.d_alpha[ray] : 0.0f;
        const float p_depth = io.d_depth ? io.d_depth[ray] : 0.0f;
        const float tau_S = io.cache[ray];
        // d(loss)/dT_S through alpha = 1 - T_S and rgb += T_S bg, times T_S
        const float kS = __expf(-tau_S) * (p_alpha - (p0 * io.bg[0] + p1 * io.bg[1] + p2 * io.bg[2]));
        float tau_end = tau_S;  // optical depth up to the end of the current step
        float carry = 0.0f;     // sum of w_j a_j over all later steps

        for (int j0 = ((S - 1) / kStep) * kStep; j0 >= 0; j0 -= kStep) {
            StepActs<C, H, NH, kNB> a;
            forward_step<KIND, C, H, NH, true, kNB, true>(g, lds, q, j0, S, lane, a);

            // ---- emission-absorption backward; MFMA column col stands for sample
            //      j0 + slot_to_sample(col) (both lane groups alike), so the scans along the
            //      ray run on values moved into sample order and their results are moved back ----
            const int to_slot = sample_to_slot(col), to_smp = slot_to_sample(col);
            const int j = j0 + to_smp;
            const bool valid = j < S;
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const float sd = valid ? fast_softplus(a.z[0]) * q.delta : 0.0f;
            const float incl_ord = group_scan_incl<kStep>(__shfl(sd, to_slot, kStep), col);
            const float incl = __shfl(incl_ord, to_smp, kStep);
            const float tau_start = tau_end - __shfl(incl_ord, kStep - 1, kStep);
            const float Tprev = __expf(-(tau_start + (incl - sd)));
            const float w = Tprev * one_minus_exp_neg(sd);
            const float Tq = Tprev - w;
            const float c1 = fast_logistic(a.z[1]), c2 = fast_logistic(a.z[2]), c3 = fast_logistic(a.z[3]);
            const float aa = p0 * c1 + p1 * c2 + p2 * c3 + p_depth * t;
            const float wa = w * aa;
            // inclusive suffix sum = total - inclusive prefix + own value
            const float wa_ord = __shfl(wa, to_slot, kStep);
            const float pre_ord = group_scan_incl<kStep>(wa_ord, col);
            const float wa_total = __shfl(pre_ord, kStep - 1, kStep);
            const float suf = __shfl(wa_total - pre_ord + wa_ord, to_smp, kStep);
            const float dsigma = q.delta * (Tq * aa - (suf - wa + carry) + kS);
            carry += wa_total;
            tau_end = tau_start;
            float dz[4];
            dz[0] = valid ? dsigma * fast_logistic(a.z[0]) : 0.0f;
            dz[1] = valid ? w * p0 * c1 * (1.0f - c1) : 0.0f;
            dz[2] = valid ? w * p1 * c2 * (1.0f - c2) : 0.0f;
            dz[3] = valid ? w * p2 * c3 * (1.0f - c3) : 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) dbo[k] += grp == 0 ? dz[k] : 0.0f;

            // output gradients as a B operand (K = 16, the 4 rows at k = 0..3 of lane group 0)
            uint32_t zh0, zl0, zh1, zl1;
            split2(dz[0], dz[1], zh0, zl0);
            split2(dz[2], dz[3], zh1, zl1);
            Frag gzo_h[kNB][1], gzo_l[kNB][1];
            {
                const bool mine = grp == 0;
                gzo_h[0][0].d[0] = mine ? zh0 : 0u; gzo_h[0][0].d[1] = mine ? zh1 : 0u;
                gzo_h[0][0].d[2] = 0u; gzo_h[0][0].d[3] = 0u;
                gzo_l[0][0].d[0] = mine ? zl0 : 0u; gzo_l[0][0].d[1] = mine ? zl1 : 0u;
                gzo_l[0][0].d[2] = 0u; gzo_l[0][0].d[3] = 0u;
            }

            const Frag (&lh)[kNB][KSH] = NH == 2 ? a.h2h : a.h1h;  // last hidden layer's activations
            const Frag (&ll)[kNB][KSH] = NH == 2 ? a.h2l : a.h1l;

            // The phases below alternate "store a tensor into the tile" / "work that does not touch
            // the tile" / "load the transposed operands", so that the LDS round trip of every
            // transposition is covered by matrix-core or vector work.

            // ---- output layer ----
            wave_lds_fence();
            tile.template store<KSH>(lh, ll, lane, hidden_row);          // Hlast^T
            if (grp == 0) {
                tile.hi[(H + 0) * RS + col] = (uint16_t)zh0; tile.hi[(H + 1) * RS + col] = (uint16_t)(zh0 >> 16);
                tile.hi[(H + 2) * RS + col] = (uint16_t)zh1; tile.hi[(H + 3) * RS + col] = (uint16_t)(zh1 >> 16);
                tile.lo[(H + 0) * RS + col] = (uint16_t)zl0; tile.lo[(H + 1) * RS + col] = (uint16_t)(zl0 >> 16);
                tile.lo[(H + 2) * RS + col] = (uint16_t)zl1; tile.lo[(H + 3) * RS + col] = (uint16_t)(zl1 >> 16);
                // scatter record of this lane's sample, read at the end of the step
                write_scatter_record<KIND, C>(info + col * 16, g, a.cell[0]);
            }
            // meanwhile: dZ of the last hidden layer = relu'(.) * (Wout^T dZo)
            f32x16 acc[MB][kNB];
            layer_mfma<MB, 1, kNB, true>(acc, lds + L::T3, lane, gzo_h, gzo_l);
            relu_mask<MB>(acc, lh);
            Frag gz_h[kNB][KSH], gz_l[kNB][KSH];
            to_operands<MB, false, kNB>(acc, gz_h, gz_l);
            wave_lds_fence();
            {
                // dWo += dZo * Hlast^T over the samples of the step
                Frag ah[kKS], al[kKS];
#pragma unroll
                for (int s = 0; s < kKS; ++s) tile.load(H + (col & 3), s, grp, col < 4, ah[s], al[s]);
#pragma unroll
                for (int nb = 0; nb < MB; ++nb)
#pragma unroll
                    for (int s = 0; s < kKS; ++s) {
                        Frag bh, bl;
                        tile.load(32 * nb + col, s, grp, true, bh, bl);
                        dWo[nb] = mfma3(ah[s], al[s], bh, bl, dWo[nb]);
                    }
            }
            wave_lds_fence();

            if constexpr (NH == 2) {
                // ---- second hidden layer: dW2 += dZ2 * H1^T ; db2 += sum dZ2 ; dZ1 = relu'(.) * (W2^T dZ2) ----
                tile.template store<KSH>(gz_h, gz_l, lane, hidden_row);  // dZ2^T
                layer_mfma<MB, KSH, kNB, true>(acc, lds + L::T2, lane, gz_h, gz_l);   // meanwhile: W2^T dZ2
                wave_lds_fence();
                Frag ah[MB][kKS], al[MB][kKS];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int s = 0; s < kKS; ++s) {
                        tile.load(32 * mb + col, s, grp, true, ah[mb][s], al[mb][s]);
                        db2[mb] = frag_sum(al[mb][s], frag_sum(ah[mb][s], db2[mb]));
                    }
                wave_lds_fence();
                tile.template store<KSH>(a.h1h, a.h1l, lane, hidden_row);  // H1^T
                relu_mask<MB>(acc, a.h1h);                                 // meanwhile: dZ1
                to_operands<MB, false, kNB>(acc, gz_h, gz_l);
                wave_lds_fence();
#pragma unroll
                for (int nb = 0; nb < MB; ++nb)
#pragma unroll
                    for (int s = 0; s < kKS; ++s) {
                        Frag bh, bl;
                        tile.load(32 * nb + col, s, grp, true, bh, bl);
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) dW2[mb][nb] = mfma3(ah[mb][s], al[mb][s], bh, bl, dW2[mb][nb]);
                    }
                wave_lds_fence();
            }

            // ---- first layer: dW1 += dZ1 * F^T ; db1 += sum dZ1 ; feature gradient, transposed:
            //      dF^T[sample][channel] = dZ1^T W1 ----
            tile.template store<KSH>(gz_h, gz_l, lane, hidden_row);      // dZ1^T
            f32x16 dFt;
#pragma unroll
            for (int s = 0; s < KSH; ++s) {                              // meanwhile: dF^T
                Frag th, tl;
                load_operand(lds + L::T1 + s * 128, lane, th, tl);
                dFt = s == 0 ? mfma3_first(gz_h[0][s], gz_l[0][s], th, tl) : mfma3(gz_h[0][s], gz_l[0][s], th, tl, dFt);
            }
            wave_lds_fence();
            {
                Frag ah[MB][kKS], al[MB][kKS];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int s = 0; s < kKS; ++s) {
                        tile.load(32 * mb + col, s, grp, true, ah[mb][s], al[mb][s]);
                        db1[mb] = frag_sum(al[mb][s], frag_sum(ah[mb][s], db1[mb]));
                    }
                wave_lds_fence();
                tile.template store<KS1>(a.fh, a.fl, lane, input_row);   // F^T
                wave_lds_fence();
#pragma unroll
                for (int s = 0; s < kKS; ++s) {
                    Frag bh, bl;
                    tile.load(col & (C - 1), s, grp, col < C, bh, bl);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) dW1[mb] = mfma3(ah[mb][s], al[mb][s], bh, bl, dW1[mb]);
                }
            }
            scatter_channels<KIND, C>(g, io.d_grid, q.scene, info, dFt, col, grp);
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

template <int KIND, int C, int H, int NH>
hipError_t launch_bwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                      hipStream_t stream)
{
    constexpr int kLdsBytes = MlpLds<C, H, NH, true, kNB>::bytes(kWaves);
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    auto kernel = bwd_mfma_kernel<KIND, C, H, NH>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int blocks = mfma_bwd_records(n_cu) / kWaves;  // every wave writes a record, busy or not
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kWaves * 64), kLdsBytes, stream, g, m, rays, io);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int threads = 256;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((m.param_total + threads - 1) / threads), dim3(threads), 0, stream,
                       m, io, blocks * kWaves);
    return hipGetLastError();
}

template <int KIND>
hipError_t dispatch_bwd(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                        hipStream_t stream)
{
    const int C = g.C, H = m.dims[1], NH = m.n_layers - 1;
#define LP_CASE(c, h, nh) \
    if (C == c && H == h && NH == nh) return launch_bwd<KIND, c, h, nh>(g, m, rays, io, n_cu, stream);
    LP_CASE(16, 32, 1) LP_CASE(16, 64, 1) LP_CASE(32, 32, 1) LP_CASE(32, 64, 1)
    LP_CASE(16, 32, 2) LP_CASE(16, 64, 2) LP_CASE(32, 32, 2) LP_CASE(32, 64, 2)
#undef LP_CASE
    return hipErrorInvalidValue;
}

}  // namespace

// one workgroup of 4 waves per compute unit, rounded up to a multiple of the 8 XCDs
int mfma_bwd_records(int n_cu) { return ((n_cu + 7) / 8 * 8) * kWaves; }

hipError_t launch_bwd_mfma(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                           hipStream_t stream)
{
    return g.kind == LP_GRID_VOXEL ? dispatch_bwd<LP_GRID_VOXEL>(g, m, rays, io, n_cu, stream)
                                   : dispatch_bwd<LP_GRID_TRIPLANE>(g, m, rays, io, n_cu, stream);
}

}  // namespace lp
