// Building blocks of the matrix-core (MFMA) kernels for gfx950.
//
// One wavefront marches one ray in chunks of 64 consecutive samples.  The decoder MLP of a
// chunk is a dense contraction [out x in] x [in x 64 samples], evaluated transposed
// (D = W * X, samples along the N axis) with v_mfma_f32_32x32x16_bf16 so that a layer's
// output registers are, without any data movement, the next layer's B operand:
//
//   operand layout of the instruction (A is M x K, B is K x N, D is M x N, M = N = 32, K = 16):
//     lane l = 32 g + i holds A[i][8g .. 8g+7], B[8g .. 8g+7][i], and D[8q + 4g + p][i] in
//     register r = 4q + p (q, p = 0..3).
//
//   Registers 8h .. 8h+7 (h = 0, 1) of a D block, taken as the 8 B-operand elements of one
//   K-step, therefore stand for the rows  8 (e / 4) + 16 h + 4 g + (e % 4),  e = 0..7, of that
//   block.  The A operands (weights) are staged in LDS with their K index permuted the same
//   way, so the contraction is unchanged.
//
// fp32 operands are split into bf16 hi + lo (x = hi + lo + O(2^-18 |x|)); each product is
// evaluated as lo*hi + hi*lo + hi*hi with fp32 accumulation inside the matrix core.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lp_device.h"

namespace lp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

struct Frag {  // one MFMA A or B operand: 8 bf16 = 4 dwords
    uint32_t d[4];
};

__device__ __forceinline__ bf16x8 as_bf16x8(const Frag& f)
{
    return __builtin_bit_cast(bf16x8, f);
}

// hi = bf16(x) (round to nearest even), lo = bf16(x - hi); two values per dword.  The
// residuals x - hi are exact in fp32; each is one dot-product instruction on the packed hi
// pair: x0 + (hi0, hi1).(-1, 0) and x1 + (hi0, hi1).(0, -1).
__device__ __forceinline__ void split2(float x0, float x1, uint32_t& hi, uint32_t& lo)
{
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    // one packed conversion per pair (a vector conversion keeps the two halves together)
    const f32x2 x = {x0, x1};
    const bf16x2 h = __builtin_convertvector(x, bf16x2);
    // (-1, -0): the natural (-1, +0) = 0x0000bf80 is turned into the inline constant "-1.0",
    // which this instruction does not read as a packed bf16 pair
    const bf16x2 sel0 = __builtin_bit_cast(bf16x2, 0x8000bf80u);
    const bf16x2 sel1 = __builtin_bit_cast(bf16x2, 0xbf800000u);  // (0, -1)
    const float r0 = __builtin_amdgcn_fdot2_f32_bf16(h, sel0, x0, false);
    const float r1 = __builtin_amdgcn_fdot2_f32_bf16(h, sel1, x1, false);
    const f32x2 r = {r0, r1};
    const bf16x2 l = __builtin_convertvector(r, bf16x2);
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, l);
}

// max(x, 0) as one integer instruction: a float with its sign bit set is a negative integer
// (-0.0 included), any other float is unchanged.
__device__ __forceinline__ float relu_f(float x)
{
    return __int_as_float(max(__float_as_int(x), 0));
}

__device__ __forceinline__ void split8(const float* x, Frag& hi, Frag& lo)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) split2(x[2 * i], x[2 * i + 1], hi.d[i], lo.d[i]);
}

// acc += (a_hi + a_lo) * (b_hi + b_lo) without the lo*lo term; small terms first.
__device__ __forceinline__ f32x16 mfma3(const Frag& ah, const Frag& al, const Frag& bh, const Frag& bl,
                                        f32x16 acc)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(al), as_bf16x8(bh), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(bl), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(bh), acc, 0, 0, 0);
    return acc;
}

// Same, starting a new accumulation: the first product takes the constant 0 as its C operand
// (an inline constant of the instruction), so no register has to be cleared beforehand.
__device__ __forceinline__ f32x16 mfma3_first(const Frag& ah, const Frag& al, const Frag& bh, const Frag& bl)
{
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(al), as_bf16x8(bh), zero, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(bl), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ah), as_bf16x8(bh), acc, 0, 0, 0);
    return acc;
}

// Row of a 32-row D block that register r of lane-group g holds.
__host__ __device__ constexpr int d_row(int r, int g) { return 8 * (r / 4) + 4 * g + (r % 4); }

// Input feature that element e of lane-group g stands for in K-step s, when the B operand is
// taken from the D registers of the previous layer (blocks of 32 rows, two K-steps per block).
__host__ __device__ constexpr int k_hidden(int s, int g, int e)
{
    return 32 * (s / 2) + 16 * (s % 2) + 8 * (e / 4) + 4 * g + (e % 4);
}

// Input channel for the first layer: lane-group g holds the contiguous half [g C/2, (g+1) C/2).
template <int C>
__host__ __device__ constexpr int k_input(int s, int g, int e)
{
    return g * (C / 2) + 8 * s + e;
}

// Stages one weight matrix as MFMA A operands: for block (mb, s) 64 lanes x 8 bf16 of the hi
// parts (1 KiB) followed by the lo parts.  row_of(mb, i) gives the source row of the weight
// matrix for output row i of block mb (negative: zero row); col_of(s, g, e) the source column
// (negative: zero).
template <class RowFn, class ColFn>
__device__ __forceinline__ void stage_operand(uint4* dst, const float* __restrict__ W, int n_mb, int n_ks,
                                              int ld, RowFn row_of, ColFn col_of)
{
    __bf16* out = reinterpret_cast<__bf16*>(dst);
    const int total = n_mb * n_ks * 512;
#pragma unroll 1
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int e = idx & 7, lane = (idx >> 3) & 63, blk = idx >> 9;
        const int s = blk % n_ks, mb = blk / n_ks;
        const int r = row_of(mb, lane & 31);
        const int c = col_of(s, lane >> 5, e);
        const float v = (r >= 0 && c >= 0) ? W[(size_t)r * ld + c] : 0.0f;
        const __bf16 h = (__bf16)v;
        const __bf16 l = (__bf16)(v - (float)h);
        out[(size_t)blk * 1024 + lane * 8 + e] = h;
        out[(size_t)blk * 1024 + 512 + lane * 8 + e] = l;
    }
}

// Same for the TRANSPOSED matrix: A[m][k] = W[k][m].  row_of(mb, i) gives the source COLUMN of W
// for output row i of block mb, col_of(s, g, e) the source ROW; a negative index gives zero.
template <class RowFn, class ColFn>
__device__ __forceinline__ void stage_operand_t(uint4* dst, const float* __restrict__ W, int n_mb, int n_ks,
                                                int ld, RowFn row_of, ColFn col_of)
{
    __bf16* out = reinterpret_cast<__bf16*>(dst);
    const int total = n_mb * n_ks * 512;
#pragma unroll 1
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int e = idx & 7, lane = (idx >> 3) & 63, blk = idx >> 9;
        const int s = blk % n_ks, mb = blk / n_ks;
        const int c = row_of(mb, lane & 31);
        const int r = col_of(s, lane >> 5, e);
        const float v = (r >= 0 && c >= 0) ? W[(size_t)r * ld + c] : 0.0f;
        const __bf16 h = (__bf16)v;
        const __bf16 l = (__bf16)(v - (float)h);
        out[(size_t)blk * 1024 + lane * 8 + e] = h;
        out[(size_t)blk * 1024 + 512 + lane * 8 + e] = l;
    }
}

__device__ __forceinline__ void load_operand(const uint4* blk, int lane, Frag& hi, Frag& lo)
{
    const uint4 h = blk[lane];
    const uint4 l = blk[64 + lane];
    hi.d[0] = h.x; hi.d[1] = h.y; hi.d[2] = h.z; hi.d[3] = h.w;
    lo.d[0] = l.x; lo.d[1] = l.y; lo.d[2] = l.z; lo.d[3] = l.w;
}

// v shifted by data-parallel-primitive control `CTRL` (lanes without a source get 0).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

// Inclusive prefix sum over groups of W consecutive lanes (W = 64: the whole wave; W = 32: each
// half on its own), on the DPP network: shifts by 1, 2, 4, 8 inside rows of 16 lanes, then
// the last lane of a row is broadcast into the next row (and of lane 31 into the upper half).
template <int W>
__device__ __forceinline__ float group_scan_incl(float v, int /*pos*/)
{
    v += dpp_or_zero<0x111, 0xf>(v);  // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);  // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);  // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);  // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    if constexpr (W == 64) v += dpp_or_zero<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ float wave_scan_incl(float v, int lane) { return group_scan_incl<64>(v, lane); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// 1 - exp(-x) for x >= 0 without cancellation for small x.
__device__ __forceinline__ float one_minus_exp_neg(float x)
{
    const float series = x * (1.0f - 0.5f * x * (1.0f - (1.0f / 3.0f) * x * (1.0f - 0.25f * x)));
    const float direct = 1.0f - __expf(-x);
    return x < 0.03f ? series : direct;
}

__device__ __forceinline__ float fast_softplus(float z)
{
    return fmaxf(z, 0.0f) + __logf(1.0f + __expf(-fabsf(z)));
}

__device__ __forceinline__ float fast_logistic(float z)
{
    return __frcp_rn(1.0f + __expf(-z));
}

// Rendered feature from its decoder output: logistic sigmoid, or the output itself (`identity`, a
// uniform run-time flag), and the derivative of that head given its value.
__device__ __forceinline__ float feature_head(float z, bool identity) { return identity ? z : fast_logistic(z); }
__device__ __forceinline__ float feature_head_slope(float c, bool identity) { return identity ? 1.0f : c * (1.0f - c); }

// ---- sampling of the hash structure (Section 3.2) for one lane's half of the channels ----

struct Cell3 {
    int i[3];
    float f[3];
    float g[3];  // 1 - f from the fp64 index (only the Splatter reads it; unused copies cost nothing)
};

template <bool CC>
__device__ __forceinline__ Cell3 locate3(const GridDev& g, double x, double y, double z)
{
    Cell3 c;
    axis_cell<CC>(x, g.amin[0], g.scale[0], g.N[0], g.contract, c.i[0], c.f[0], c.g[0]);
    axis_cell<CC>(y, g.amin[1], g.scale[1], g.N[1], g.contract, c.i[1], c.f[1], c.g[1]);
    axis_cell<CC>(z, g.amin[2], g.scale[2], g.N[2], g.contract, c.i[2], c.f[2], c.g[2]);
    return c;
}

// Table entries of the 8 lattice corners of cell c in a hash table whose size is a power of two (the
// matrix-core kernels take only those): corner 4dx + 2dy + dz.  The spatial hash of Teschner et al.
// 2003 with Instant-NGP's primes, in 32-bit unsigned arithmetic; `mod size` is a mask here.
__device__ __forceinline__ void hash_corner_slots(const Cell3& c, unsigned hash_size, unsigned (&slot)[8])
{
    const unsigned mask = hash_size - 1u;
    const unsigned hx = (unsigned)c.i[0], hy = (unsigned)c.i[1] * 2654435761u, hz = (unsigned)c.i[2] * 805459861u;
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        const unsigned x = hx + (unsigned)(d >> 2);
        const unsigned y = hy + (((d >> 1) & 1) ? 2654435761u : 0u);
        const unsigned z = hz + ((d & 1) ? 805459861u : 0u);
        slot[d] = (x ^ y ^ z) & mask;
    }
}

// The texels one lane reads for a sample: NCH consecutive channels of every corner (voxel: corner
// 4dx + 2dy + dz; triplane: plane p, corner 2da + db at 4p + ..), as 16-byte loads of the grid's
// storage type GT (lp_dtype: 4 fp32 or 8 bf16 / fp16 values each).  Loading and interpolating
// are separate steps so that a kernel can issue the loads early and do other work meanwhile.
template <int KIND, int NCH, int GT>
struct GatherRaw {
    static constexpr int kCorners = KIND == LP_GRID_TRIPLANE ? 12 : 8;
    static constexpr int kPerVec = GT == LP_F32 ? 4 : 8;
    static constexpr int kVecs = NCH / kPerVec;
    uint4 v[kCorners][kVecs];
};

template <int KIND, int C, int NCH, int GT>
__device__ __forceinline__ void gather_issue(const GridDev& g, int scene, const Cell3& c, int ch0,
                                             GatherRaw<KIND, NCH, GT>& raw)
{
    constexpr int kVecs = GatherRaw<KIND, NCH, GT>::kVecs;
    constexpr unsigned kElem = GT == LP_F32 ? 4u : 2u;  // bytes per stored value
    if constexpr (KIND == LP_GRID_VOXEL) {
        const char* V = reinterpret_cast<const char*>(g.data[0]) + (size_t)scene * g.N[0] * g.N[1] * g.N[2] * C * kElem;
        const unsigned sz = C, sy = (unsigned)g.N[2] * C, sx = (unsigned)g.N[1] * sy;
        const unsigned base = (unsigned)c.i[0] * sx + (unsigned)c.i[1] * sy + (unsigned)c.i[2] * sz + ch0;
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const uint4* p = reinterpret_cast<const uint4*>(V + (size_t)(base + dx * sx + dy * sy + dz * sz) * kElem);
#pragma unroll
            for (int i = 0; i < kVecs; ++i) raw.v[d][i] = p[i];
        }
    } else if constexpr (KIND == LP_GRID_HASH) {
        const char* V = reinterpret_cast<const char*>(g.data[0]) + (size_t)scene * g.hash_size * C * kElem;
        unsigned slot[8];
        hash_corner_slots(c, g.hash_size, slot);
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const uint4* p = reinterpret_cast<const uint4*>(V + ((size_t)slot[d] * C + ch0) * kElem);
#pragma unroll
            for (int i = 0; i < kVecs; ++i) raw.v[d][i] = p[i];
        }
    } else {
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
            const int a = pl, b = (pl + 1) % 3;
            const char* P = reinterpret_cast<const char*>(g.data[pl]) + (size_t)scene * g.N[a] * g.N[b] * C * kElem;
            const unsigned sb = C, sa = (unsigned)g.N[b] * C;
            const unsigned base = (unsigned)c.i[a] * sa + (unsigned)c.i[b] * sb + ch0;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                const uint4* p = reinterpret_cast<const uint4*>(P + (size_t)(base + da * sa + db * sb) * kElem);
#pragma unroll
                for (int i = 0; i < kVecs; ++i) raw.v[4 * pl + d][i] = p[i];
            }
        }
    }
}

// the stored values of one 16-byte load as fp32
template <int GT>
__device__ __forceinline__ void unpack_values(const uint4& u, float* out)
{
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
    if constexpr (GT == LP_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = __uint_as_float(w[i]);
    } else if constexpr (GT == LP_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __half2float(__ushort_as_half((unsigned short)(w[i] & 0xffffu)));
            out[2 * i + 1] = __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
        }
    }
}

// feat[0..NCH) = the interpolated channels (Section 3.2: trilinear / sum of three bilinear)
template <int KIND, int NCH, int GT>
__device__ __forceinline__ void gather_finish(const Cell3& c, const GatherRaw<KIND, NCH, GT>& raw, float* feat)
{
    using R = GatherRaw<KIND, NCH, GT>;
#pragma unroll
    for (int k = 0; k < NCH; ++k) feat[k] = 0.0f;
#pragma unroll
    for (int d = 0; d < R::kCorners; ++d) {
        float w;
        if constexpr (KIND != LP_GRID_TRIPLANE) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            w = (dx ? c.f[0] : 1.0f - c.f[0]) * (dy ? c.f[1] : 1.0f - c.f[1]) * (dz ? c.f[2] : 1.0f - c.f[2]);
        } else {
            const int a = d >> 2, b = (a + 1) % 3, da = (d >> 1) & 1, db = d & 1;
            w = (da ? c.f[a] : 1.0f - c.f[a]) * (db ? c.f[b] : 1.0f - c.f[b]);
        }
#pragma unroll
        for (int i = 0; i < R::kVecs; ++i) {
            float v[R::kPerVec];
            unpack_values<GT>(raw.v[d][i], v);
#pragma unroll
            for (int e = 0; e < R::kPerVec; ++e) feat[R::kPerVec * i + e] += w * v[e];
        }
    }
}

// feat[0..NCH) = channels [ch0, ch0 + NCH) of h(x) in scene `scene`.
template <int KIND, int C, int NCH, int GT = LP_F32>
__device__ __forceinline__ void gather_half(const GridDev& g, int scene, const Cell3& c, int ch0, float* feat)
{
    GatherRaw<KIND, NCH, GT> raw;
    gather_issue<KIND, C, NCH, GT>(g, scene, c, ch0, raw);
    gather_finish<KIND, NCH, GT>(c, raw, feat);
}

// HexPlane (Section 3.2 names it among the structures; Cao & Johnson 2023): the cell of the ray's time on
// the time axis (not contracted, clamped at both ends).
__device__ __forceinline__ void time_cell(const GridDev& g, float time, int& it, float& ft)
{
    float gt;
    axis_cell<false>((double)time, g.tmin, g.tscale, g.NT, 0.0, it, ft, gt);
}

// feat[0..NCH) = channels [ch0, ch0 + NCH) of a HexPlane at cell c and time `time`: for each of the three
// pairs, the bilinear read of the spatial plane over axes (a, b) = (0,1), (1,2), (2,0) times the bilinear
// read of the space-time plane over (c, t), c the third axis; the three products added.
template <int C, int NCH, int GT>
__device__ __forceinline__ void gather_half_hexplane(const GridDev& g, int scene, const Cell3& c, float time,
                                                     int ch0, float* feat)
{
    constexpr int kPerVec = GT == LP_F32 ? 4 : 8, kVecs = NCH / kPerVec;
    constexpr unsigned kElem = GT == LP_F32 ? 4u : 2u;
    int it;
    float ft;
    time_cell(g, time, it, ft);
#pragma unroll
    for (int k = 0; k < NCH; ++k) feat[k] = 0.0f;
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
        const char* P = reinterpret_cast<const char*>(g.data[p]) + (size_t)scene * g.N[a] * g.N[b] * C * kElem;
        const char* Q = reinterpret_cast<const char*>(g.data_t[p]) + (size_t)scene * g.N[cc] * g.NT * C * kElem;
        const unsigned bs = ((unsigned)c.i[a] * (unsigned)g.N[b] + (unsigned)c.i[b]) * C + ch0;
        const unsigned bu = ((unsigned)c.i[cc] * (unsigned)g.NT + (unsigned)it) * C + ch0;
        uint4 rs[4][kVecs], ru[4][kVecs];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int da = d >> 1, db = d & 1;
            const uint4* ps = reinterpret_cast<const uint4*>(P + (size_t)(bs + (da * (unsigned)g.N[b] + db) * C) * kElem);
            const uint4* pu = reinterpret_cast<const uint4*>(Q + (size_t)(bu + (da * (unsigned)g.NT + db) * C) * kElem);
#pragma unroll
            for (int i = 0; i < kVecs; ++i) { rs[d][i] = ps[i]; ru[d][i] = pu[i]; }
        }
        float s[NCH], u[NCH];
#pragma unroll
        for (int k = 0; k < NCH; ++k) s[k] = u[k] = 0.0f;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int da = d >> 1, db = d & 1;
            const float ws = (da ? c.f[a] : 1.0f - c.f[a]) * (db ? c.f[b] : 1.0f - c.f[b]);
            const float wu = (da ? c.f[cc] : 1.0f - c.f[cc]) * (db ? ft : 1.0f - ft);
#pragma unroll
            for (int i = 0; i < kVecs; ++i) {
                float vs[kPerVec], vu[kPerVec];
                unpack_values<GT>(rs[d][i], vs);
                unpack_values<GT>(ru[d][i], vu);
#pragma unroll
                for (int e = 0; e < kPerVec; ++e) {
                    s[kPerVec * i + e] += ws * vs[e];
                    u[kPerVec * i + e] += wu * vu[e];
                }
            }
        }
#pragma unroll
        for (int k = 0; k < NCH; ++k) feat[k] += s[k] * u[k];
    }
}

// Ranges of rays per XCD: workgroup b runs on XCD b % 8, so giving XCD x the contiguous ray
// range x keeps neighbouring rays (which read neighbouring texels) behind one L2.
struct RaySchedule {
    long long first;   // first ray of this wave
    long long end;     // end of this XCD's range
    long long stride;  // rays between consecutive iterations of this wave
};

__device__ __forceinline__ RaySchedule ray_schedule(long long M, int waves_per_block)
{
    constexpr int kXcd = 8;
    const int xcd = blockIdx.x % kXcd;
    const int local_block = blockIdx.x / kXcd;
    const int blocks_per_xcd = gridDim.x / kXcd;  // gridDim.x is a multiple of 8
    const long long per_xcd = (M + kXcd - 1) / kXcd;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    RaySchedule s;
    const long long begin = per_xcd * xcd;
    s.end = begin + per_xcd < M ? begin + per_xcd : M;
    s.first = begin + (long long)local_block * waves_per_block + wave;
    s.stride = (long long)blocks_per_xcd * waves_per_block;
    return s;
}

}  // namespace lp
