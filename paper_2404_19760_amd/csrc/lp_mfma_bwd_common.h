// Pieces shared by the matrix-core backward kernels: wave-level LDS fence, ReLU-derivative
// masking, bias-gradient sums, and the scatter of the feature gradient into the grid gradient.
#pragma once
#include "lp_mfma.h"
#include "lp_mfma_mlp.h"

namespace lp {

constexpr int kBwdNB = 1;               // N blocks (of 32 samples) per backward step
constexpr int kBwdStep = 32 * kBwdNB;   // samples per step
constexpr int kBwdKS = 2 * kBwdNB;      // K-steps of a contraction over the samples of a step

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wave execute in order; this only pins the compiler's ordering of
    // the tile stores of some lanes against the tile loads of others
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_sched_barrier(0);
}

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
__device__ __forceinline__ void relu_mask(f32x16 (&acc)[MB][kBwdNB], const Frag (&act_hi)[kBwdNB][2 * MB])
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < kBwdNB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int s = 2 * mb + r / 8, e = r % 8;
                const uint32_t bits = (act_hi[nb][s].d[e / 2] >> (16 * (e & 1))) & 0xffffu;
                acc[mb][nb][r] = bits ? acc[mb][nb][r] : 0.0f;
            }
}

// ---- matrix-core helpers of the backward kernels ----
__device__ __forceinline__ f32x16 mfma1(const Frag& a, const Frag& b, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), acc, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16()
{
    const f32x16 z = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    return z;
}

// Keeps a long-lived accumulator in the accumulation register file between its updates, so
// that the vector registers stay free for the working set of a step.
__device__ __forceinline__ void park(f32x16& acc)
{
    asm volatile("" : "+a"(acc));
}

// acc += A B over the two K-steps of a 32-sample step, each product as (a_hi + a_lo)(b_hi + b_lo)
// without lo*lo, for an accumulator that LIVES in the accumulation registers: the six
// instructions read and write it there, with no copies through vector registers (left to itself
// the compiler keeps some of the long-lived accumulators in vector-register form and copies them
// in and out of the accumulation registers at every step: 64 copies per step for two blocks).
// The compiler does not look inside the block, so the block keeps the rules that apply itself:
//   - a matrix instruction may read a vector register two wait states after a vector instruction
//     wrote it at the earliest: the leading s_nop;
//   - it may take the previous matrix instruction's result as its addend without wait states only
//     when it follows it immediately: six in a row, nothing in between;
//   - whatever touches the accumulator next (a copy the register allocator decides to make, the
//     record at the end of the kernel) must find the last result landed: an 8-pass instruction's
//     result may be read 18 wait states after its issue, the trailing s_nops.
__device__ __forceinline__ void mfma6_parked(f32x16& acc, const Frag (&ah)[kBwdKS], const Frag (&al)[kBwdKS],
                                             const Frag (&bh)[kBwdKS], const Frag (&bl)[kBwdKS])
{
    static_assert(kBwdKS == 2, "two K-steps per backward step");
    asm volatile("s_nop 1\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %3, %4, %0\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %3, %2, %0\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %5, %6, %0\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %7, %8, %0\n\t"
                 "v_mfma_f32_32x32x16_bf16 %0, %7, %6, %0\n\t"
                 "s_nop 15\n\t"
                 "s_nop 1"
                 : "+a"(acc)
                 : "v"(as_bf16x8(al[0])), "v"(as_bf16x8(bh[0])), "v"(as_bf16x8(ah[0])), "v"(as_bf16x8(bl[0])),
                   "v"(as_bf16x8(al[1])), "v"(as_bf16x8(bh[1])), "v"(as_bf16x8(ah[1])), "v"(as_bf16x8(bl[1])));
}

// Registers of a transposed block D[sample][feature] (values exactly representable in bf16)
// -> operand fragments over the samples: K-step ks takes registers 8 ks .. 8 ks + 7.
__device__ __forceinline__ void pack_exact(const f32x16& d, Frag (&f)[kBwdKS])
{
#pragma unroll
    for (int ks = 0; ks < kBwdKS; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w)
            f[ks].d[w] = __builtin_amdgcn_perm(__float_as_uint(d[8 * ks + 2 * w + 1]), __float_as_uint(d[8 * ks + 2 * w]),
                                               0x07060302u);
}

// 0/1 selection operand: element e of lane (j, grp) is 1.0 iff index_of(grp, e) == j.
template <class IndexFn>
__device__ __forceinline__ Frag selection(int j, int grp, IndexFn index_of)
{
    Frag f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t lo = index_of(grp, 2 * w) == j ? 0x3f80u : 0u;
        const uint32_t hi = index_of(grp, 2 * w + 1) == j ? 0x3f80u : 0u;
        f.d[w] = lo | (hi << 16);
    }
    return f;
}

// ---- scatter records: what the channel lanes need to know about each sample of the step ----
// 16 dwords per sample.  voxel: 8 corner weights, then the element offset of corner 0; the
// weights are in corner order 4dx + 2dy + dz for 32 channels and in order 4dz + 2dx + dy for 16
// channels (where the two halves of a lane group take the corners of one dz each).
// triplane: 12 weights (plane p, corner 2da + db at 4p + ..), then 3 plane offsets.
// hash table: the 8 corner weights in the voxel's order for this channel count, then the element
// offsets (entry x channels) of the 8 corners in the same order.
// HexPlane: 32 dwords per sample: 12 weights of the spatial planes as for a triplane, 12 weights of the
// space-time planes (pair p, corner 2dc + dt at 12 + 4p + ..), then the 3 + 3 plane offsets.
// EXACT: the complements 1 - f come from the fp64 index (the Splatter, whose result divides by sums
// of these weights); otherwise from the rounded f (the Renderer's gradient scatter).
template <int KIND>
constexpr int kRecordDwords = KIND == LP_GRID_HEXPLANE ? 32 : 16;

template <int KIND, int C, bool EXACT = false>
__device__ __forceinline__ void write_scatter_record(float* rec, const GridDev& g, const Cell3& c, float time = 0.0f)
{
    if constexpr (KIND == LP_GRID_HEXPLANE) {
        int it;
        float ft;
        time_cell(g, time, it, ft);
        unsigned offs[6];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
            const float a1 = c.f[a], a0 = 1.0f - a1, b1 = c.f[b], b0 = 1.0f - b1;
            const float c1 = c.f[cc], c0 = 1.0f - c1, t1 = ft, t0 = 1.0f - ft;
            reinterpret_cast<float4*>(rec)[p] = make_float4(a0 * b0, a0 * b1, a1 * b0, a1 * b1);
            reinterpret_cast<float4*>(rec)[3 + p] = make_float4(c0 * t0, c0 * t1, c1 * t0, c1 * t1);
            offs[p] = ((unsigned)c.i[a] * (unsigned)g.N[b] + (unsigned)c.i[b]) * C;
            offs[3 + p] = ((unsigned)c.i[cc] * (unsigned)g.NT + (unsigned)it) * C;
        }
        reinterpret_cast<uint4*>(rec)[6] = make_uint4(offs[0], offs[1], offs[2], offs[3]);
        reinterpret_cast<uint4*>(rec)[7] = make_uint4(offs[4], offs[5], 0u, 0u);
        return;
    }
    if constexpr (KIND == LP_GRID_VOXEL) {
        const float x1 = c.f[0], x0 = EXACT ? c.g[0] : 1.0f - x1, y1 = c.f[1], y0 = EXACT ? c.g[1] : 1.0f - y1,
                    z1 = c.f[2], z0 = EXACT ? c.g[2] : 1.0f - z1;
        const float4 w0 = C == 16 ? make_float4(x0 * y0 * z0, x0 * y1 * z0, x1 * y0 * z0, x1 * y1 * z0)
                                  : make_float4(x0 * y0 * z0, x0 * y0 * z1, x0 * y1 * z0, x0 * y1 * z1);
        const float4 w1 = C == 16 ? make_float4(x0 * y0 * z1, x0 * y1 * z1, x1 * y0 * z1, x1 * y1 * z1)
                                  : make_float4(x1 * y0 * z0, x1 * y0 * z1, x1 * y1 * z0, x1 * y1 * z1);
        const unsigned sz = C, sy = (unsigned)g.N[2] * C, sx = (unsigned)g.N[1] * sy;
        const unsigned base = (unsigned)c.i[0] * sx + (unsigned)c.i[1] * sy + (unsigned)c.i[2] * sz;
        reinterpret_cast<float4*>(rec)[0] = w0;
        reinterpret_cast<float4*>(rec)[1] = w1;
        reinterpret_cast<unsigned*>(rec)[8] = base;
    } else if constexpr (KIND == LP_GRID_HASH) {
        const float x1 = c.f[0], x0 = EXACT ? c.g[0] : 1.0f - x1, y1 = c.f[1], y0 = EXACT ? c.g[1] : 1.0f - y1,
                    z1 = c.f[2], z0 = EXACT ? c.g[2] : 1.0f - z1;
        unsigned s[8];   // corner 4dx + 2dy + dz
        hash_corner_slots(c, g.hash_size, s);
        if constexpr (C == 16) {   // order 4dz + 2dx + dy: the two halves of a lane group take one dz each
            reinterpret_cast<float4*>(rec)[0] = make_float4(x0 * y0 * z0, x0 * y1 * z0, x1 * y0 * z0, x1 * y1 * z0);
            reinterpret_cast<float4*>(rec)[1] = make_float4(x0 * y0 * z1, x0 * y1 * z1, x1 * y0 * z1, x1 * y1 * z1);
            reinterpret_cast<uint4*>(rec)[2] = make_uint4(s[0] * C, s[2] * C, s[4] * C, s[6] * C);
            reinterpret_cast<uint4*>(rec)[3] = make_uint4(s[1] * C, s[3] * C, s[5] * C, s[7] * C);
        } else {                   // order 4dx + 2dy + dz
            reinterpret_cast<float4*>(rec)[0] = make_float4(x0 * y0 * z0, x0 * y0 * z1, x0 * y1 * z0, x0 * y1 * z1);
            reinterpret_cast<float4*>(rec)[1] = make_float4(x1 * y0 * z0, x1 * y0 * z1, x1 * y1 * z0, x1 * y1 * z1);
            reinterpret_cast<uint4*>(rec)[2] = make_uint4(s[0] * C, s[1] * C, s[2] * C, s[3] * C);
            reinterpret_cast<uint4*>(rec)[3] = make_uint4(s[4] * C, s[5] * C, s[6] * C, s[7] * C);
        }
    } else {
        unsigned base[3];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            const float a1 = c.f[a], a0 = EXACT ? c.g[a] : 1.0f - a1, b1 = c.f[b], b0 = EXACT ? c.g[b] : 1.0f - b1;
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
// IN_ORDER: record s belongs to sample s of the step and dFt[r] to sample 16 grp + r (a kernel that
// passes the feature gradient through LDS reads it back in this order without permuting the step).
constexpr int kWalkAhead = 2;   // samples whose scatter records are read ahead in the 32-channel and triplane walks

template <int KIND, int C, bool IN_ORDER = false>
__device__ __forceinline__ void scatter_channels(const GridDev& g, float* const d_grid[3], int scene,
                                                 const float* info, const f32x16& dFt, int ch, int grp,
                                                 float* const d_grid_t[3] = nullptr)
{
    const bool live = ch < C;
    auto record_of = [grp](int r) { return IN_ORDER ? 16 * grp + r : d_row(r, grp); };
    if constexpr (KIND == LP_GRID_HEXPLANE) {
        // HexPlane: by the product rule each plane of a pair receives the feature gradient times the
        // OTHER plane's read, which this channel's lane forms again from four loads.  With 32 channels a
        // lane serves both planes of every pair; with 16 channels the first half of a lane group serves
        // the spatial planes and the second half the space-time planes.  Per plane, the contributions of
        // consecutive samples that fall into the same texel cell are summed before one atomic add per
        // corner (the time of a ray is fixed, so a space-time plane changes cell only along one axis).
        const int c16 = ch & (C - 1);
        const bool do_s = C == 32 || ch < 16, do_u = C == 32 || ch >= 16;
        float acc_s[3][4], acc_u[3][4];
        unsigned prev_s[3] = {0u, 0u, 0u}, prev_u[3] = {0u, 0u, 0u};
        size_t Sb[3], Ub[3];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
            Sb[p] = (size_t)scene * g.N[a] * g.N[b] * C + c16;
            Ub[p] = (size_t)scene * g.N[cc] * g.NT * C + c16;
        }
        // the other plane's reads of sample r + 1 are loaded before the adds of sample r are issued, so
        // that their latency passes behind those adds
        auto other_reads = [&](int r, float (&u)[3], float (&sv)[3]) {
            const float* rec = info + record_of(r) * 32;
            const uint4 o0 = reinterpret_cast<const uint4*>(rec)[6], o1 = reinterpret_cast<const uint4*>(rec)[7];
            const unsigned off[6] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y};
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                const int b = (p + 1) % 3;
                const unsigned sa = (unsigned)g.N[b] * C, ua = (unsigned)g.NT * C;
                u[p] = sv[p] = 0.0f;
                if (do_s) {
                    const float4 w4 = reinterpret_cast<const float4*>(rec)[3 + p];
                    const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        u[p] += w[d] * grid_load(g, g.data_t[p], Ub[p] + off[3 + p] + (d >> 1) * ua + (d & 1) * C);
                }
                if (do_u) {
                    const float4 w4 = reinterpret_cast<const float4*>(rec)[p];
                    const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        sv[p] += w[d] * grid_load(g, g.data[p], Sb[p] + off[p] + (d >> 1) * sa + (d & 1) * C);
                }
            }
        };
        float cur_u[3], cur_s[3];
        other_reads(0, cur_u, cur_s);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float* rec = info + record_of(r) * 32;
            const float v = dFt[r];
            const uint4 o0 = reinterpret_cast<const uint4*>(rec)[6], o1 = reinterpret_cast<const uint4*>(rec)[7];
            const unsigned off[6] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y};
            float nxt_u[3] = {0.0f, 0.0f, 0.0f}, nxt_s[3] = {0.0f, 0.0f, 0.0f};
            if (r + 1 < 16) other_reads(r + 1, nxt_u, nxt_s);
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                const int b = (p + 1) % 3;
                const float4 ws4 = reinterpret_cast<const float4*>(rec)[p], wu4 = reinterpret_cast<const float4*>(rec)[3 + p];
                const float ws[4] = {ws4.x, ws4.y, ws4.z, ws4.w}, wu[4] = {wu4.x, wu4.y, wu4.z, wu4.w};
                const unsigned sa = (unsigned)g.N[b] * C, ua = (unsigned)g.NT * C;   // step to the next row of either plane
                if (do_s) {   // spatial plane += weights * (gradient * read of the space-time plane)
                    const float vu = v * cur_u[p];
                    const bool moved = off[p] != prev_s[p];
                    if (r > 0 && moved) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) atomicAdd(d_grid[p] + Sb[p] + prev_s[p] + (d >> 1) * sa + (d & 1) * C, acc_s[p][d]);
                    }
#pragma unroll
                    for (int d = 0; d < 4; ++d) acc_s[p][d] = (r == 0 || moved) ? ws[d] * vu : acc_s[p][d] + ws[d] * vu;
                    prev_s[p] = off[p];
                }
                if (do_u) {   // space-time plane += weights * (gradient * read of the spatial plane)
                    const float vs = v * cur_s[p];
                    const bool moved = off[3 + p] != prev_u[p];
                    if (r > 0 && moved) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) atomicAdd(d_grid_t[p] + Ub[p] + prev_u[p] + (d >> 1) * ua + (d & 1) * C, acc_u[p][d]);
                    }
#pragma unroll
                    for (int d = 0; d < 4; ++d) acc_u[p][d] = (r == 0 || moved) ? wu[d] * vs : acc_u[p][d] + wu[d] * vs;
                    prev_u[p] = off[3 + p];
                }
            }
#pragma unroll
            for (int p = 0; p < 3; ++p) { cur_u[p] = nxt_u[p]; cur_s[p] = nxt_s[p]; }
        }
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const int b = (p + 1) % 3;
            const unsigned sa = (unsigned)g.N[b] * C, ua = (unsigned)g.NT * C;
            if (do_s) {
#pragma unroll
                for (int d = 0; d < 4; ++d) atomicAdd(d_grid[p] + Sb[p] + prev_s[p] + (d >> 1) * sa + (d & 1) * C, acc_s[p][d]);
            }
            if (do_u) {
#pragma unroll
                for (int d = 0; d < 4; ++d) atomicAdd(d_grid_t[p] + Ub[p] + prev_u[p] + (d >> 1) * ua + (d & 1) * C, acc_u[p][d]);
            }
        }
        return;
    }
    if constexpr (KIND == LP_GRID_HASH) {
        // Hash table: a lane (channel; with 16 channels the two halves of a lane group take the four
        // corners of one dz each, as for voxels) sums the contributions of consecutive samples whose
        // corners are the SAME table entries and adds them when any entry changes; equal entries are
        // the merge criterion, so colliding corners of different cells merge as well.
        constexpr int N = C == 16 ? 4 : 8;          // corners per lane
        const int c16 = ch & (C - 1), half = C == 16 ? ch >> 4 : 0;
        float* V = d_grid[0] + (size_t)scene * g.hash_size * C;
        float acc[N];
        unsigned prev[N] = {};
        auto flush = [&]() {
            if (live || C == 16) {
#pragma unroll
                for (int k = 0; k < N; ++k) atomicAdd(V + prev[k] + c16, acc[k]);
            }
        };
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float* rec = info + record_of(r) * 16;
            float w[N];
            unsigned o[N];
            if constexpr (C == 16) {
                const float4 w4 = reinterpret_cast<const float4*>(rec)[half];
                const uint4 o4 = reinterpret_cast<const uint4*>(rec)[2 + half];
                w[0] = w4.x; w[1] = w4.y; w[2] = w4.z; w[3] = w4.w;
                o[0] = o4.x; o[1] = o4.y; o[2] = o4.z; o[3] = o4.w;
            } else {
                const float4 wa = reinterpret_cast<const float4*>(rec)[0], wb = reinterpret_cast<const float4*>(rec)[1];
                const uint4 oa = reinterpret_cast<const uint4*>(rec)[2], ob = reinterpret_cast<const uint4*>(rec)[3];
                w[0] = wa.x; w[1] = wa.y; w[2] = wa.z; w[3] = wa.w; w[4] = wb.x; w[5] = wb.y; w[6] = wb.z; w[7] = wb.w;
                o[0] = oa.x; o[1] = oa.y; o[2] = oa.z; o[3] = oa.w; o[4] = ob.x; o[5] = ob.y; o[6] = ob.z; o[7] = ob.w;
            }
            const float v = dFt[r];
            bool moved = false;
#pragma unroll
            for (int k = 0; k < N; ++k) moved = moved || (o[k] != prev[k]);
            if (r > 0 && moved) flush();
#pragma unroll
            for (int k = 0; k < N; ++k) {
                acc[k] = (r == 0 || moved) ? w[k] * v : acc[k] + w[k] * v;
                prev[k] = o[k];
            }
        }
        flush();
    } else if constexpr (KIND == LP_GRID_VOXEL && C == 16) {
        // 16 channels fill half a lane group: lanes 16..31 hold the same feature gradients as lanes
        // 0..15 (the transposed first-layer weights are staged twice), and each half takes the four
        // corners of one dz, so that a flush is four instructions on two full 64-byte lines each
        const int c16 = ch & 15, dz = ch >> 4;
        const unsigned sz = C, sy = (unsigned)g.N[2] * C, sx = (unsigned)g.N[1] * sy;
        char* V = reinterpret_cast<char*>(d_grid[0] + (size_t)scene * g.N[0] * g.N[1] * g.N[2] * C);
        char* Vd[4];  // uniform pointer per (dx, dy)
#pragma unroll
        for (int k = 0; k < 4; ++k) Vd[k] = V + 4u * (size_t)((k >> 1) * sx + (k & 1) * sy);
        const unsigned lane_off = dz * sz + c16;
        float acc[4];
        unsigned prev = 0;
        auto flush = [&]() {
#pragma unroll
            for (int k = 0; k < 4; ++k) atomicAdd(reinterpret_cast<float*>(Vd[k] + 4u * (prev + lane_off)), acc[k]);
        };
        // the records are read two samples ahead of their use, so that the LDS latency is covered by
        // the work on the samples in between
        constexpr int kAhead = IN_ORDER ? 6 : 2;   // (the two-wave kernel's weights wave has registers to spare here)
        float4 wq[kAhead];
        unsigned bq[kAhead];
#pragma unroll
        for (int r = 0; r < kAhead; ++r) {
            const float* rec = info + record_of(r) * 16;
            wq[r] = reinterpret_cast<const float4*>(rec)[dz];
            bq[r] = reinterpret_cast<const unsigned*>(rec)[8];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float4 w4 = wq[r % kAhead];
            const unsigned base = bq[r % kAhead];
            if (r + kAhead < 16) {
                const float* rec = info + record_of(r + kAhead) * 16;
                wq[r % kAhead] = reinterpret_cast<const float4*>(rec)[dz];
                bq[r % kAhead] = reinterpret_cast<const unsigned*>(rec)[8];
            }
            const float w[4] = {w4.x, w4.y, w4.z, w4.w};
            const float v = dFt[r];
            if (r > 0 && base != prev) {
                flush();
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[k] = 0.0f;
            }
            prev = base;
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] = r == 0 ? w[k] * v : acc[k] + w[k] * v;
        }
        flush();
    } else if constexpr (KIND == LP_GRID_VOXEL) {
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
        // the records are read kWalkAhead samples ahead of their use (the adds to global memory in between
        // keep the compiler from moving the LDS reads up by itself)
        float4 w0q[kWalkAhead], w1q[kWalkAhead];
        unsigned bq[kWalkAhead];
#pragma unroll
        for (int r = 0; r < kWalkAhead; ++r) {
            const float* rec = info + record_of(r) * 16;
            w0q[r] = reinterpret_cast<const float4*>(rec)[0];
            w1q[r] = reinterpret_cast<const float4*>(rec)[1];
            bq[r] = reinterpret_cast<const unsigned*>(rec)[8];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float4 w0 = w0q[r % kWalkAhead], w1 = w1q[r % kWalkAhead];
            const unsigned base = bq[r % kWalkAhead];
            if (r + kWalkAhead < 16) {
                const float* rec = info + record_of(r + kWalkAhead) * 16;
                w0q[r % kWalkAhead] = reinterpret_cast<const float4*>(rec)[0];
                w1q[r % kWalkAhead] = reinterpret_cast<const float4*>(rec)[1];
                bq[r % kWalkAhead] = reinterpret_cast<const unsigned*>(rec)[8];
            }
            const float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            const float v = dFt[r];
            if (r > 0 && base != prev) {
                // Keeping shared corners across a cell change costs selects and saves atomic
                // requests.  Measured: it pays where a corner spans two 64-byte lines (32 channels,
                // the kernel then runs at the atomic units' request rate) and loses where a corner
                // is one line and the kernel is bound by its own instruction stream (16 channels).
                constexpr bool kCarryVoxel = C >= 32;
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
            float4 wq[kWalkAhead];
            unsigned bq[kWalkAhead];
#pragma unroll
            for (int r = 0; r < kWalkAhead; ++r) {
                const float* rec = info + record_of(r) * 16;
                wq[r] = reinterpret_cast<const float4*>(rec)[pl];
                bq[r] = reinterpret_cast<const unsigned*>(rec)[12 + pl];
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float4 w4 = wq[r % kWalkAhead];
                const unsigned base = bq[r % kWalkAhead];
                if (r + kWalkAhead < 16) {
                    const float* rec = info + record_of(r + kWalkAhead) * 16;
                    wq[r % kWalkAhead] = reinterpret_cast<const float4*>(rec)[pl];
                    bq[r % kWalkAhead] = reinterpret_cast<const unsigned*>(rec)[12 + pl];
                }
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

}  // namespace lp
