// Device-side views of the C-ABI arguments and the few formulas every kernel shares:
// sample placement, world -> grid addressing (Section 3.2 of the paper) and the
// density / colour heads.  HIP for gfx950 only.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lightplane.h"

namespace lp {

struct GridDev {
    const void* data[3];  // elements of type dtype
    int kind, B, C;
    int dtype;            // lp_dtype
    int N[3];
    double amin[3];
    double scale[3];  // (N-1)/(max-min): world -> continuous index
    double contract;  // foreground scale a of the contract coordinates, 0 = off
    unsigned hash_size;  // LP_GRID_HASH: entries of one scene's table
    // LP_GRID_HEXPLANE: the space-time planes (pair p: plane data[p] with data_t[p] over (axis p + 2, time))
    const void* data_t[3];
    int NT;
    double tmin, tscale;  // (NT-1)/(t_max-t_min)
};

struct MlpDev {
    int n_layers;
    int dims[LP_MAX_LAYERS + 1];
    const float* W[LP_MAX_LAYERS];
    const float* b[LP_MAX_LAYERS];
    int w_off[LP_MAX_LAYERS];  // offsets of W[l] / b[l] in one packed float array
    int b_off[LP_MAX_LAYERS];
    int param_total;           // floats of all weights and biases
    int max_width;             // widest layer input or output
    int act_total;             // dims[0] + ... + dims[n_layers]
    // decoder shape: dims[0] = grid channels + n_enc direction inputs (+ zero padding);
    // the last layer has 1 + n_feat outputs (density, then the rendered features)
    int n_freq;                // octaves of the direction encoding (unused when n_enc == 0)
    int n_enc;                 // 0: no direction input, else 3 + 6 n_freq
    int n_feat;                // rendered feature channels (3 for the single-MLP decoder)
    int feat_act;              // 0 logistic sigmoid, 1 identity
};

struct RaysDev {
    long long M;
    int S;
    const float* origins;
    const float* dirs;
    const float* near;
    const float* far;
    const int* scene;
    const float* time;  // per ray, or null (LP_GRID_HEXPLANE)
};

struct FwdOut {
    float* rgb;   // [M][n_feat]
    float* alpha;
    float* depth;
    float* cache;
    float bg[LP_MAX_FEATURES];
};

struct BwdIo {
    const float* d_rgb;
    const float* d_alpha;
    const float* d_depth;
    const float* cache;
    float* d_grid[3];
    float* d_grid_t[3];  // LP_GRID_HEXPLANE: gradients of the space-time planes
    float* dW[LP_MAX_LAYERS];
    float* db[LP_MAX_LAYERS];
    float bg[LP_MAX_FEATURES];
    float* ws;         // per-wave (or per-block) partial sums of the MLP gradients
    int ws_stride;     // floats between consecutive partial-sum records
    int acc_in_record; // generic kernels: accumulate MLP gradients in the record itself, not in LDS
};

// element `idx` of a grid tensor as fp32
__device__ __forceinline__ float grid_load(const GridDev& g, const void* base, size_t idx)
{
    if (g.dtype == LP_F32) return reinterpret_cast<const float*>(base)[idx];
    const unsigned short h = reinterpret_cast<const unsigned short*>(base)[idx];
    if (g.dtype == LP_BF16) return __uint_as_float((unsigned)h << 16);
    return __half2float(__ushort_as_half(h));
}

// Table entry of lattice corner (ix, iy, iz) in a hash-table structure: the spatial hash of Teschner et
// al. 2003 (the one Instant-NGP uses), in 32-bit unsigned arithmetic.
__device__ __forceinline__ unsigned hash_slot(int ix, int iy, int iz, unsigned hash_size)
{
    return (((unsigned)ix * 1u) ^ ((unsigned)iy * 2654435761u) ^ ((unsigned)iz * 805459861u)) % hash_size;
}

// Splatter arguments (Section 3.3 "Splatter"): pixel features, optional prior structure, the
// accumulators of the forward, the inputs and outputs of the backward.
struct SplatDev {
    int n_in;               // channels of the pixel features
    int has_prior;
    const float* feats;     // [M][n_in]
    GridDev prior;          // valid when has_prior
    float* theta[3];        // forward: target accumulators, then the normalised result
    float* theta_w[3];      // forward: weight sums
    const float* d_theta[3];     // backward: gradient of the normalised result
    const float* theta_w_in[3];  // backward: weight sums of the forward
    float* d_feats;         // backward: [M][n_in], written
};

// Continuous index along one axis, clamped to the box; cell index in [0, N-2] and the
// fraction inside the cell in [0, 1].  The index is formed in fp64 (full rate on this chip):
// in fp32 an index of a few hundred has a spacing of 1e-5 and more, which would put a relative
// error of up to 1e-4 on every interpolated feature of a fine grid.
// CC = true: the coordinate first goes through the contraction of the paper's appendix with
// foreground scale a = `contract` (0.5 a x inside the unit interval,
// 0.5 ((2 - a)(1 - 1/|x|) + a) sign(x) beyond), each axis on its own.  1/|x| from the fp32
// reciprocal plus one Newton step in fp64 (relative error ~1e-14).
// g = 1 - f, rounded from the fp64 index as well: formed from the rounded f it would carry an
// absolute error of 6e-8 however small it is, which the Splatter's division by a cell's weight
// sum turns into an unbounded relative error for cells that only receive tiny weights.
template <bool CC = false>
__device__ __forceinline__ void axis_cell(double x, double lo, double scale, int N, double contract, int& i,
                                          float& f, float& g)
{
    if constexpr (CC) {
        const double m = fmax(fabs(x), 1.0);
        double r = (double)__frcp_rn((float)m);
        r = r * (2.0 - m * r);
        const double far = copysign(0.5 * ((2.0 - contract) * (1.0 - r) + contract), x);
        x = fabs(x) <= 1.0 ? 0.5 * contract * x : far;
    }
    double u = (x - lo) * scale;
    u = fmin(fmax(u, 0.0), (double)(N - 1));
    int c = (int)u;  // u >= 0: truncation is floor
    c = min(c, N - 2);
    i = c;
    const double fr = u - (double)c;
    f = (float)fr;
    g = (float)(1.0 - fr);
}

template <bool CC = false>
__device__ __forceinline__ void axis_cell(double x, double lo, double scale, int N, double contract, int& i,
                                          float& f)
{
    float g;
    axis_cell<CC>(x, lo, scale, N, contract, i, f, g);
}

// Entry e of the view-direction encoding (Section 3.3: the feature MLP also receives the view
// direction; the form of the encoding is this library's reading): the direction itself, then per
// octave k the sines and the cosines of 2^k pi d, component by component.
__device__ __forceinline__ float dir_encoding(const float d[3], int e)
{
    if (e < 3) return d[e];
    const int k = (e - 3) / 6, r = (e - 3) % 6;
    const float x = (float)(1 << k) * d[r % 3];
    return r < 3 ? sinpif(x) : cospif(x);
}

// softplus(z) = max(z,0) + log1p(exp(-|z|)); its derivative is the logistic function.
__device__ __forceinline__ float softplus_f(float z)
{
    return fmaxf(z, 0.0f) + log1pf(__expf(-fabsf(z)));
}

__device__ __forceinline__ float logistic_f(float z)
{
    return 1.0f / (1.0f + __expf(-z));
}

}  // namespace lp
