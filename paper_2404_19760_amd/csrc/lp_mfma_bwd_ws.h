// Matrix-core backward kernel of the Renderer (Eq. (2), Section 3.4 of the paper) with the work of
// a ray split between TWO waves that share a SIMD.
//
// Why: a wave cannot overlap its own vector instructions with its own matrix instructions (measured
// on this chip: a loop of one 32x32x16 product and K independent multiply-adds takes 32 + 4 K
// cycles, the sum), only different waves of a SIMD overlap.  The weight-gradient accumulators of a
// 16-64-64-4 MLP are 128 registers per lane, so two waves that each do the whole backward of a
// ray do not fit the 512 registers of a SIMD lane.  Two waves of different ROLES do:
//
//   chain wave    samples the hash structure (Section 3.2; the texel loads of the next step are issued
//                 at the start of a step and interpolated at its end), recomputes the MLP forward of
//                 a 32-sample step, evaluates Eq. (2), and runs the input-gradient chain dX = W^T dZ
//                 down to the first layer's pre-activation gradient dZ1: the dependent sequence
//                 layer -> split into bf16 operands -> layer.  It holds no accumulators and issues no
//                 atomic adds, so its loads never queue behind them.
//   weights wave  transposes the activations and pre-activation gradients the chain wave hands over
//                 (0/1 selection products), accumulates dW += dZ X^T and
//                 db, takes the chain's last link (feature gradient dF = W1^T dZ1: matrix
//                 instructions only, and this wave's matrix work is hidden under the chain wave's
//                 vector work) and scatters it into the grid gradient (run-merged atomic adds).
//                 Apart from those atomic adds it touches no global memory inside a step.
//
// Waves w and w + 4 of a workgroup of eight land on the same SIMD (measured: two matrix-bound waves
// w, w + 4 take twice the time of one; w, w + 1 do not), so pair p = (wave p: chain, wave p + 4:
// weights) marches the rays the one-wave kernel gives to wave p.  Steps are marched in sample order
// (MFMA column c = sample j0 + c): the scans of Eq. (2) then run in lane order, and the order the walk
// wants (16 consecutive samples per lane group) is produced by the way the weights wave reads the
// feature gradient back from LDS.
//
// Hand-over through LDS, per pair: two 8 KiB slots for the hidden tensors as operand fragments (h1
// then dZ1 in one, h2 then dZ2 in the other), the input features, the output gradients, two buffers
// of scatter records (and the weights wave's own area for re-ordering the feature gradient); nothing
// per sample goes to global memory.  Each wave
// publishes ONE counter in LDS that says how far it has got (see HandOver); LDS operations of a wave
// execute in order, so data written before a counter value is visible to whoever reads that value.
// Waits poll with s_sleep and give up after kSpinLimit polls: the wave then stops waiting for good
// and the weight-gradient record is poisoned with NaN, so a broken hand-over ends as a wrong (loudly
// wrong) result, never as a hang.
//
// Tried and dropped (largest configuration, same box; this layout: 60 ms, one wave per ray: 63.6 ms):
// sampling in the weights wave (its loads queue behind its own atomic adds: 83 ms); the walk of a step
// deferred behind the next step's transposes (more live registers than the 256 of a wave: spills that
// also queue behind the atomic adds, 62.6 - 80 ms); the second half of the input-gradient chain in
// the weights wave (64 ms: that wave becomes the longer one).  With the weights wave idle the chain
// wave alone takes 53 ms, so the split as such cannot go below that.
#pragma once
#include "lp_kernels.h"
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"
#include "lp_mfma_bwd_common.h"

namespace lp {

namespace {

constexpr int kPairs = 4;             // (chain, weights) wave pairs per workgroup

// Measurement build (-DLP_WS_PHASES): both roles add up the cycles they spend between the marks
// LP_PHASE(k) of a step (s_memtime; each mark is also a scheduling barrier, so such a build is a
// few per cent slower), lp_diag_ws_phases() reads the sums.  Off by default: the marks are empty.
#ifdef LP_WS_PHASES
__device__ unsigned long long g_ws_phase_cycles[2][16];
#define LP_PHASE_STATE long long ph[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; long long ph_prev = clock64();
#define LP_PHASE(k)                                             \
    do {                                                        \
        __builtin_amdgcn_sched_barrier(0);                      \
        const long long ph_now = clock64();                     \
        ph[k] += ph_now - ph_prev;                              \
        ph_prev = ph_now;                                       \
        __builtin_amdgcn_sched_barrier(0);                      \
    } while (0)
#define LP_PHASE_FLUSH(role)                                                                            \
    do {                                                                                                \
        if (lane == 0)                                                                                  \
            for (int k = 0; k < 16; ++k) atomicAdd(&g_ws_phase_cycles[role][k], (unsigned long long)ph[k]); \
    } while (0)
#else
#define LP_PHASE_STATE
#define LP_PHASE(k)
#define LP_PHASE_FLUSH(role)
#endif
constexpr int kSpinLimit = 1 << 20;   // polls of one wait before the wave gives up (normal: a handful)

// LDS area of one pair in 16-byte units.
template <int C, int H>
struct PairLds {
    static constexpr int KS1 = C / 16, KSH = H / 16;
    static constexpr int SLOT = KSH * 128;                 // a hidden tensor: KSH fragments, hi and lo
    static constexpr int SLOT0 = 0;                        // h1, then dZ1
    static constexpr int SLOT1 = SLOT0 + SLOT;             // h2, then dZ2
    static constexpr int F = SLOT1 + SLOT;                 // input features: KS1 fragments, hi and lo
    static constexpr int ZO = F + KS1 * 128;               // output gradients of sample column c: (hi01, hi23, lo01, lo23)
    static constexpr int DFT = ZO + 32;                    // (weights wave only) feature gradient: [8 quads of samples][C channels] x 4 samples
    static constexpr int REC = DFT + 4 * 2 * C;            // two buffers of 32 scatter records (16 dwords each)
    static constexpr int FLAGS = REC + 2 * 128;            // the two progress counters, 32 bytes apart
    static constexpr int UNITS = FLAGS + 4;
};

// Hand-over protocol.  Each wave of a pair publishes ONE counter, 8 n + stage: "in step n, I am done
// with everything up to `stage`".  For the chain wave the stages are the buffers it has WRITTEN, in its
// program order; for the weights wave the buffers it has finished READING (plus the end of its walk).
// A wave that needs the partner to have passed (n, stage) compares with the last value it has seen and
// reads the counter again only if that is not enough, so most checks cost nothing.
enum ChainStage { C_H1, C_H2, C_ZO, C_Z2, C_F, C_Z1 };
enum WeightsStage { W_H2, W_ZO, W_H1, W_Z2, W_F, W_Z1, W_WALK };
__host__ __device__ constexpr int progress(int n, int stage) { return 8 * n + stage; }

typedef __attribute__((address_space(3))) int LdsInt;   // the counters are addressed as LDS, never through flat instructions
                                                        // (a flat access waits for the wave's global memory operations too)

struct HandOver {
    LdsInt* own;           // counter this wave publishes
    const LdsInt* other;   // the partner's counter
    int seen;              // last value read from the partner's counter
    bool dead;             // a wait ran into the spin limit: never wait again

    // everything this wave wrote to LDS before is visible to whoever reads the new value
    __device__ __forceinline__ void post(int value)
    {
        wave_lds_fence();
        *const_cast<volatile LdsInt*>(own) = value;
    }
    __device__ __forceinline__ void await(int need)
    {
        if (seen < need && !dead) {
            int spins = 0;
            while ((seen = __builtin_amdgcn_readfirstlane(*const_cast<const volatile LdsInt*>(other))) < need) {
                __builtin_amdgcn_s_sleep(10);   // 640 cycles: polling faster than this only takes issue slots from the partner wave
                if (++spins > kSpinLimit) { dead = true; break; }
            }
        }
        wave_lds_fence();
    }
};

template <int KS>
__device__ __forceinline__ void store_frags(uint4* slot, int lane, const Frag (&h)[1][KS], const Frag (&l)[1][KS])
{
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        slot[s * 128 + lane] = make_uint4(h[0][s].d[0], h[0][s].d[1], h[0][s].d[2], h[0][s].d[3]);
        slot[s * 128 + 64 + lane] = make_uint4(l[0][s].d[0], l[0][s].d[1], l[0][s].d[2], l[0][s].d[3]);
    }
}

template <int KS>
__device__ __forceinline__ void load_frags(const uint4* slot, int lane, Frag (&h)[1][KS], Frag (&l)[1][KS])
{
#pragma unroll
    for (int s = 0; s < KS; ++s) load_operand(slot + s * 128, lane, h[0][s], l[0][s]);
}

// The rays of one pair, in the order of the one-wave kernel: groups of kPairs neighbouring rays (one
// per pair), the groups of an XCD's contiguous range in a scrambled order (neighbouring rays add
// into the same lines of the grid gradient; spread over time they do not queue up at one L2 channel).
struct RayCursor {
    long long seq, group, seq_last, n_groups, group_step, M;
    int blocks_per_xcd, pair;
    __device__ __forceinline__ bool live() const { return seq < seq_last; }
    __device__ __forceinline__ long long ray() const { return group * kPairs + pair; }
    __device__ __forceinline__ void advance()
    {
        do {
            seq += blocks_per_xcd;
            group += group_step;
            if (group >= n_groups) group -= n_groups;
        } while (seq < seq_last && ray() >= M);
    }
    __device__ __forceinline__ void init(long long M_, int pair_, long long group_mul, long long group_step_)
    {
        M = M_; pair = pair_; group_step = group_step_;
        n_groups = (M + kPairs - 1) / kPairs;
        blocks_per_xcd = gridDim.x / 8;
        const long long per_xcd = (n_groups + 7) / 8;
        seq = per_xcd * (blockIdx.x % 8) + blockIdx.x / 8;
        seq_last = min(per_xcd * (blockIdx.x % 8 + 1), n_groups);
        group = seq < seq_last ? (seq * group_mul) % n_groups : 0;
        if (seq < seq_last && ray() >= M) advance();
    }
};

template <int KIND, int C, int H, bool CC, int GT>
__global__ __launch_bounds__(2 * kPairs * 64) void bwd_ws_kernel(GridDev g, MlpDev m, RaysDev rays, BwdIo io,
                                                                 long long group_mul, long long group_step)
{
    constexpr int NH = 2;
    using L = MlpLds<C, H, NH, true, kBwdNB>;
    using P = PairLds<C, H>;
    constexpr int MB = L::MB, KS1 = L::KS1, KSH = L::KSH;
    extern __shared__ uint4 lds[];
    stage_mlp<C, H, NH, true, kBwdNB, C>(lds, m);
    // the 0/1 selection operands of the transposes, one 16-byte entry per lane each: hidden tensors
    // (two K-steps per 32-feature block), output gradients, input features
    constexpr int kSel = L::END + kPairs * P::UNITS, kSelH0 = 0, kSelH1 = 1, kSelO = 2, kSelF = 3;
    if (threadIdx.x < 64) {
        const int c = threadIdx.x & 31, gq = threadIdx.x >> 5;
        auto put = [&](int k, const Frag& f) { lds[kSel + k * 64 + threadIdx.x] = make_uint4(f.d[0], f.d[1], f.d[2], f.d[3]); };
        put(kSelH0, selection(c, gq, [](int gg, int e) { return k_hidden(0, gg, e); }));
        put(kSelH1, selection(c, gq, [](int gg, int e) { return k_hidden(1, gg, e); }));
        put(kSelO, selection(c, gq, [](int gg, int e) { return (gg == 0 && e < 4) ? e : -1; }));
#pragma unroll
        for (int s = 0; s < KS1; ++s) put(kSelF + s, selection(c, gq, [s](int gg, int e) { return k_input<C>(s, gg, e); }));
    }
    if (threadIdx.x < kPairs * 16) {
        const int p = threadIdx.x / 16, i = threadIdx.x % 16;
        reinterpret_cast<int*>(lds + L::END + p * P::UNITS + P::FLAGS)[i] = i == 8 ? progress(0, W_WALK) : 0;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int col = lane & 31, grp = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pair = wave & (kPairs - 1);
    const bool chain = wave < kPairs;
    uint4* mine = lds + L::END + pair * P::UNITS;
    // the two counters sit in different 32-byte halves of the flag area
    LdsInt* flags = (LdsInt*)reinterpret_cast<int*>(mine + P::FLAGS);
    HandOver ho;
    ho.own = flags + (chain ? 0 : 8);
    ho.other = flags + (chain ? 8 : 0);
    ho.seen = chain ? progress(0, W_WALK) : 0;
    ho.dead = false;
    float* rec = io.ws + (size_t)(blockIdx.x * kPairs + pair) * io.ws_stride;

    const int S = rays.S;
    const int j_last = ((S - 1) / kBwdStep) * kBwdStep;
    RayCursor cur;
    cur.init(rays.M, pair, group_mul, group_step);
    int n = 0;  // number of the current step of this pair

    LP_PHASE_STATE
    if (chain) {
        // ================= chain wave =================
        float dbo[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        // Cell and input features of the step about to be processed.  The texel loads of the following
        // step (of this ray, or the last step of the pair's next ray) are issued at the start of a step
        // and interpolated at its end, so that their latency passes under the step's work.
        RayGeom q_next;
        Cell3 cell;
        Frag fh[KS1], fl[KS1];
        if (cur.live()) {
            q_next = load_ray_geom(rays, cur.ray());
            cell = sample_cell_for<CC, GT>(g, q_next, min(j_last + col, S - 1));
            sample_features<KIND, C, C, GT>(g, q_next, cell, grp, fh, fl);
        }
        while (cur.live()) {
            const long long ray = cur.ray();
            const RayGeom q = q_next;
            cur.advance();
            if (cur.live()) q_next = load_ray_geom(rays, cur.ray());
            const float near = q.near, delta = q.delta;
            const float p0 = io.d_rgb[3 * ray + 0], p1 = io.d_rgb[3 * ray + 1], p2 = io.d_rgb[3 * ray + 2];
            const float p_alpha = io.d_alpha ? io.d_alpha[ray] : 0.0f;
            const float p_depth = io.d_depth ? io.d_depth[ray] : 0.0f;
            const float tau_S = io.cache[ray];
            // d(loss)/dT_S through alpha = 1 - T_S and rgb += T_S bg, times T_S
            const float kS = __expf(-tau_S) * (p_alpha - (p0 * io.bg[0] + p1 * io.bg[1] + p2 * io.bg[2]));
            float tau_end = tau_S;  // optical depth up to the end of the current step
            float carry = 0.0f;     // sum of w_j a_j over all later steps

            for (int j0 = j_last; j0 >= 0; j0 -= kBwdStep) {
                ++n;
                LP_PHASE(0);
                // the next step's cell and texel loads
                const bool same = j0 > 0;
                const bool more = same || cur.live();
                const RayGeom& qn = same ? q : q_next;
                GatherRaw<KIND, C / 2, GT> raw_next;
                Cell3 cell_next = cell;
                if (more) {
                    cell_next = sample_cell_for<CC, GT>(g, qn, min((same ? j0 - kBwdStep : j_last) + col, S - 1));
                    gather_issue<KIND, C, C / 2, GT>(g, qn.scene, cell_next, grp * (C / 2), raw_next);
                }
                __builtin_amdgcn_sched_barrier(0);
                // scatter records of this step's samples, for the walk of the weights wave
                ho.await(progress(n - 2, W_WALK));   // (implied by the slots' waits today; kept so that the record buffers do not rest on that)
                if (grp == 0)
                    write_scatter_record<KIND, C>(reinterpret_cast<float*>(mine + P::REC + (n & 1) * 128) + col * 16, g, cell);

                LP_PHASE(1);
                StepActs<C, H, NH, kBwdNB> a;
#pragma unroll
                for (int s = 0; s < KS1; ++s) { a.fh[0][s] = fh[s]; a.fl[0][s] = fl[s]; }
                mlp_forward<C, H, NH, true, kBwdNB>(lds, lane, a);
                LP_PHASE(2);
                ho.await(progress(n - 1, W_Z1));
                store_frags<KSH>(mine + P::SLOT0, lane, a.h1h, a.h1l);
                ho.post(progress(n, C_H1));
                ho.await(progress(n - 1, W_Z2));
                store_frags<KSH>(mine + P::SLOT1, lane, a.h2h, a.h2l);
                ho.post(progress(n, C_H2));

                LP_PHASE(3);
                // ---- emission-absorption backward; MFMA column col stands for sample j0 + col (both lane
                //      groups alike): the scans along the ray run over the 32 lanes of a group ----
                const int j = j0 + col;
                const bool valid = j < S;
                const float t = near + ((float)j + 0.5f) * delta;
                const float sd = valid ? fast_softplus(a.z[0]) * delta : 0.0f;
                const float incl = group_scan_incl<kBwdStep>(sd, col);
                const float tau_start = tau_end - __int_as_float(__builtin_amdgcn_readlane(__float_as_int(incl), kBwdStep - 1));
                const float Tprev = __expf(-(tau_start + (incl - sd)));
                const float w = Tprev * one_minus_exp_neg(sd);
                const float Tq = Tprev - w;
                const float c1 = fast_logistic(a.z[1]), c2 = fast_logistic(a.z[2]), c3 = fast_logistic(a.z[3]);
                const float aa = p0 * c1 + p1 * c2 + p2 * c3 + p_depth * t;
                const float wa = w * aa;
                const float pre = group_scan_incl<kBwdStep>(wa, col);
                const float wa_total = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pre), kBwdStep - 1));
                const float suf = wa_total - pre + wa;
                const float dsigma = delta * (Tq * aa - (suf - wa + carry) + kS);
                carry += wa_total;
                tau_end = tau_start;
                float dz[4];
                dz[0] = valid ? dsigma * fast_logistic(a.z[0]) : 0.0f;
                dz[1] = valid ? w * p0 * c1 * (1.0f - c1) : 0.0f;
                dz[2] = valid ? w * p1 * c2 * (1.0f - c2) : 0.0f;
                dz[3] = valid ? w * p2 * c3 * (1.0f - c3) : 0.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k) dbo[k] += grp == 0 ? dz[k] : 0.0f;

                LP_PHASE(4);
                uint32_t zh0, zl0, zh1, zl1;
                split2(dz[0], dz[1], zh0, zl0);
                split2(dz[2], dz[3], zh1, zl1);
                ho.await(progress(n - 1, W_ZO));
                if (grp == 0) mine[P::ZO + col] = make_uint4(zh0, zh1, zl0, zl1);
                ho.post(progress(n, C_ZO));
                Frag gzo_h[kBwdNB][1], gzo_l[kBwdNB][1];
                {
                    const bool own = grp == 0;
                    gzo_h[0][0].d[0] = own ? zh0 : 0u; gzo_h[0][0].d[1] = own ? zh1 : 0u;
                    gzo_h[0][0].d[2] = 0u; gzo_h[0][0].d[3] = 0u;
                    gzo_l[0][0].d[0] = own ? zl0 : 0u; gzo_l[0][0].d[1] = own ? zl1 : 0u;
                    gzo_l[0][0].d[2] = 0u; gzo_l[0][0].d[3] = 0u;
                }

                LP_PHASE(5);
                // ---- input-gradient chain: dZ2 = relu'(.) * (Wout^T dZo), dZ1 = relu'(.) * (W2^T dZ2); the
                //      last link (the feature gradient) is left to the weights wave, which holds dZ1 anyway ----
                f32x16 acc[MB][kBwdNB];
                Frag gz_h[kBwdNB][KSH], gz_l[kBwdNB][KSH];
                layer_mfma<MB, 1, kBwdNB, true>(acc, lds + L::T3, lane, gzo_h, gzo_l);
                relu_mask<MB>(acc, a.h2h);
                to_operands<MB, false, kBwdNB>(acc, gz_h, gz_l);
                LP_PHASE(6);
                ho.await(progress(n, W_H2));
                store_frags<KSH>(mine + P::SLOT1, lane, gz_h, gz_l);
                ho.post(progress(n, C_Z2));
                LP_PHASE(7);
                layer_mfma<MB, KSH, kBwdNB, true>(acc, lds + L::T2, lane, gz_h, gz_l);
                relu_mask<MB>(acc, a.h1h);
                to_operands<MB, false, kBwdNB>(acc, gz_h, gz_l);
                LP_PHASE(8);
                ho.await(progress(n - 1, W_F));
                store_frags<KS1>(mine + P::F, lane, a.fh, a.fl);
                ho.post(progress(n, C_F));
                ho.await(progress(n, W_H1));
                store_frags<KSH>(mine + P::SLOT0, lane, gz_h, gz_l);
                ho.post(progress(n, C_Z1));
                LP_PHASE(9);
                if (more) {
                    float feat[C / 2];
                    gather_finish<KIND, C / 2, GT>(cell_next, raw_next, feat);
#pragma unroll
                    for (int s = 0; s < KS1; ++s) split8(feat + 8 * s, fh[s], fl[s]);
                    cell = cell_next;
                }
                LP_PHASE(10);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float s = wave_sum(dbo[k]);
            if (lane == 0) rec[m.b_off[NH] + k] = s;
        }
        LP_PHASE_FLUSH(0);
        return;
    }

    // ================= weights wave =================
    // (read from LDS where they are used: sixteen registers less that live through the whole loop)
    auto sel = [&](int k) {
        const uint4 v = lds[kSel + k * 64 + lane];
        Frag f;
        f.d[0] = v.x; f.d[1] = v.y; f.d[2] = v.z; f.d[3] = v.w;
        return f;
    };
    // block nb2 (features 32 nb2 .. +31) of the hidden tensor in `slot`, transposed; the hi and the lo
    // parts one after the other (issuing the four products back to back measured no faster)
    auto transpose_block = [&](const uint4* slot, int nb2, Frag (&th)[kBwdKS], Frag (&tl)[kBwdKS]) {
        Frag x0h, x0l, x1h, x1l;
        load_operand(slot + (2 * nb2) * 128, lane, x0h, x0l);
        load_operand(slot + (2 * nb2 + 1) * 128, lane, x1h, x1l);
        {
            f32x16 d = mfma1(x0h, sel(kSelH0), zero16());
            d = mfma1(x1h, sel(kSelH1), d);
            pack_exact(d, th);
        }
        __builtin_amdgcn_sched_barrier(0);
        {
            f32x16 d = mfma1(x0l, sel(kSelH0), zero16());
            d = mfma1(x1l, sel(kSelH1), d);
            pack_exact(d, tl);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto transpose_features = [&](const Frag (&xh)[KS1], const Frag (&xl)[KS1], Frag (&th)[kBwdKS], Frag (&tl)[kBwdKS]) {
        {
            f32x16 d = mfma1(xh[0], sel(kSelF), zero16());
#pragma unroll
            for (int s = 1; s < KS1; ++s) d = mfma1(xh[s], sel(kSelF + s), d);
            pack_exact(d, th);
        }
        __builtin_amdgcn_sched_barrier(0);
        {
            f32x16 d = mfma1(xl[0], sel(kSelF), zero16());
#pragma unroll
            for (int s = 1; s < KS1; ++s) d = mfma1(xl[s], sel(kSelF + s), d);
            pack_exact(d, tl);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // acc += A B over the two K-steps of a step, small terms first
    auto accumulate = [](f32x16& acc, const Frag (&ah)[kBwdKS], const Frag (&al)[kBwdKS], const Frag (&bh)[kBwdKS],
                         const Frag (&bl)[kBwdKS]) {
#pragma unroll
        for (int ks = 0; ks < kBwdKS; ++ks) acc = mfma3(ah[ks], al[ks], bh[ks], bl[ks], acc);
    };

    f32x16 dW1[MB], dW2[MB][MB], dWo[MB];
    float db1[MB], db2[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        dW1[mb] = zero16();
        dWo[mb] = zero16();
        db1[mb] = db2[mb] = 0.0f;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) dW2[mb][nb] = zero16();
    }

    while (cur.live()) {
        const int scene = rays.scene ? rays.scene[cur.ray()] : 0;
        cur.advance();
        for (int j0 = j_last; j0 >= 0; j0 -= kBwdStep) {
            ++n;
            LP_PHASE(0);
            // ---- dWo += dZo H2^T ----
            {
                Frag t2h[MB][kBwdKS], t2l[MB][kBwdKS];
                ho.await(progress(n, C_H2));
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) transpose_block(mine + P::SLOT1, nb2, t2h[nb2], t2l[nb2]);
            LP_PHASE(1);
                ho.post(progress(n, W_H2));
                ho.await(progress(n, C_ZO));
            LP_PHASE(2);
                const uint4 zo = mine[P::ZO + col];
                ho.post(progress(n, W_ZO));
                Frag gh, gl;
                gh.d[0] = grp == 0 ? zo.x : 0u; gh.d[1] = grp == 0 ? zo.y : 0u; gh.d[2] = 0u; gh.d[3] = 0u;
                gl.d[0] = grp == 0 ? zo.z : 0u; gl.d[1] = grp == 0 ? zo.w : 0u; gl.d[2] = 0u; gl.d[3] = 0u;
                Frag ah[kBwdKS], al[kBwdKS];
                pack_exact(mfma1(gh, sel(kSelO), zero16()), ah);
                __builtin_amdgcn_sched_barrier(0);
                pack_exact(mfma1(gl, sel(kSelO), zero16()), al);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) accumulate(dWo[nb2], ah, al, t2h[nb2], t2l[nb2]);
            }
            __builtin_amdgcn_sched_barrier(0);

            LP_PHASE(3);
            // ---- dW2 += dZ2 H1^T ; db2 += sum dZ2 ----
            {
                Frag t1h[MB][kBwdKS], t1l[MB][kBwdKS];
                ho.await(progress(n, C_H1));
#pragma unroll
                for (int nb2 = 0; nb2 < MB; ++nb2) transpose_block(mine + P::SLOT0, nb2, t1h[nb2], t1l[nb2]);
            LP_PHASE(4);
                ho.post(progress(n, W_H1));
                ho.await(progress(n, C_Z2));
            LP_PHASE(5);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    Frag ah[kBwdKS], al[kBwdKS];
                    transpose_block(mine + P::SLOT1, mb, ah, al);
                    if (mb == MB - 1) ho.post(progress(n, W_Z2));
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) db2[mb] = frag_sum(al[ks], frag_sum(ah[ks], db2[mb]));
#pragma unroll
                    for (int nb2 = 0; nb2 < MB; ++nb2) accumulate(dW2[mb][nb2], ah, al, t1h[nb2], t1l[nb2]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);

            LP_PHASE(6);
            // ---- dW1 += dZ1 F^T ; db1 += sum dZ1 ; feature gradient ----
            {
                Frag bf_h[kBwdKS], bf_l[kBwdKS];
                {
                    Frag f_h[1][KS1], f_l[1][KS1];
                    ho.await(progress(n, C_F));
                    load_frags<KS1>(mine + P::F, lane, f_h, f_l);
                    ho.post(progress(n, W_F));
                    transpose_features(f_h[0], f_l[0], bf_h, bf_l);
                }
            LP_PHASE(7);
                ho.await(progress(n, C_Z1));
            LP_PHASE(8);
                // feature gradient, transposed: dF^T[sample][channel] = dZ1^T W1 (operands swapped: lane =
                // channel, registers = samples 8q + 4 grp ..), K-steps in order; parked in this wave's LDS
                // area at once, from where the walk reads it in its own order
                {
                    f32x16 dFt;
#pragma unroll
                    for (int s = 0; s < KSH; ++s) {
                        Frag xh, xl, th, tl;
                        load_operand(mine + P::SLOT0 + s * 128, lane, xh, xl);
                        load_operand(lds + L::T1 + s * 128, lane, th, tl);
                        dFt = s == 0 ? mfma3_first(xh, xl, th, tl) : mfma3(xh, xl, th, tl, dFt);
                    }
                    if (col < C) {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            mine[P::DFT + (q * 2 + grp) * C + col] =
                                make_uint4(__float_as_uint(dFt[4 * q]), __float_as_uint(dFt[4 * q + 1]),
                                           __float_as_uint(dFt[4 * q + 2]), __float_as_uint(dFt[4 * q + 3]));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    Frag ah[kBwdKS], al[kBwdKS];
                    transpose_block(mine + P::SLOT0, mb, ah, al);
                    if (mb == MB - 1) ho.post(progress(n, W_Z1));
#pragma unroll
                    for (int ks = 0; ks < kBwdKS; ++ks) db1[mb] = frag_sum(al[ks], frag_sum(ah[ks], db1[mb]));
                    accumulate(dW1[mb], ah, al, bf_h, bf_l);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);

            LP_PHASE(9);
            // ---- scatter of the feature gradient (lane = channel, register = 16 consecutive samples) ----
            wave_lds_fence();
            f32x16 dFt;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const uint4 v = mine[P::DFT + (4 * grp + qd) * C + (col & (C - 1))];   // samples 16 grp + 4 qd ..
                dFt[4 * qd] = __uint_as_float(v.x); dFt[4 * qd + 1] = __uint_as_float(v.y);
                dFt[4 * qd + 2] = __uint_as_float(v.z); dFt[4 * qd + 3] = __uint_as_float(v.w);
            }
            scatter_channels<KIND, C, true>(g, io.d_grid, scene, reinterpret_cast<const float*>(mine + P::REC + (n & 1) * 128),
                                      dFt, col, grp);
            ho.post(progress(n, W_WALK));
            LP_PHASE(10);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    LP_PHASE_FLUSH(1);
    // ---- this pair's record of partial sums (the chain wave adds the output layer's bias gradient) ----
    const float poison = ho.dead ? __builtin_nanf("") : 0.0f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int out = 32 * mb + d_row(r, grp);
            if (col < C) rec[m.w_off[0] + out * C + col] = dW1[mb][r] + poison;
#pragma unroll
            for (int nb = 0; nb < MB; ++nb) rec[m.w_off[1] + out * H + 32 * nb + col] = dW2[mb][nb][r] + poison;
        }
#pragma unroll
    for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (grp == 0) rec[m.w_off[NH] + r * H + 32 * nb + col] = dWo[nb][r] + poison;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const float s1 = db1[mb] + __shfl_xor(db1[mb], 32, 64);
        if (grp == 0) rec[m.b_off[0] + 32 * mb + col] = s1;
        const float s2 = db2[mb] + __shfl_xor(db2[mb], 32, 64);
        if (grp == 0) rec[m.b_off[1] + 32 * mb + col] = s2;
    }
}

template <int KIND, int C, int H, bool CC, int GT = LP_F32>
hipError_t launch_bwd_ws(const GridDev& g, const MlpDev& m, const RaysDev& rays, const BwdIo& io, int n_cu,
                         hipStream_t stream)
{
    constexpr int kLdsBytes = (MlpLds<C, H, 2, true, kBwdNB>::END + kPairs * PairLds<C, H>::UNITS + (3 + C / 16) * 64) * 16;
    static_assert(kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    auto kernel = bwd_ws_kernel<KIND, C, H, CC, GT>;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    const int blocks = mfma_bwd_records(n_cu) / kPairs;  // every pair writes a record, busy or not
    // multiplier of the ray-group scramble: a prime that does not divide the number of groups,
    // so that group -> group * mul mod n_groups is a bijection
    const long long n_groups = (rays.M + kPairs - 1) / kPairs;
    long long group_mul = 1;
    for (long long p : {7919LL, 7907LL, 7901LL, 7883LL})
        if (n_groups > p && n_groups % p != 0) { group_mul = p; break; }
    const long long group_step = ((long long)(blocks / 8) * group_mul) % n_groups;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(2 * kPairs * 64), kLdsBytes, stream, g, m, rays, io,
                       group_mul, group_step);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reduce_params_kernel, dim3((m.param_total + 63) / 64), dim3(kReduceThreads), 0, stream,
                       m, io, blocks * kPairs);
    return hipGetLastError();
}

}  // namespace

}  // namespace lp
