/*
 * lightplane.h — C ABI of the MI355X (gfx950) Lightplane Renderer library.
 *
 * The library computes the Renderer of "Lightplane" (arXiv 2404.19760): fused,
 * differentiable emission-absorption ray marching over a hybrid 3D representation
 * f = g o h (Section 3.2), where h is bi/tri-linear sampling of a triplane or voxel
 * feature grid and g a tiny MLP, with a backward pass that stores one scalar per ray
 * and recomputes everything else (Section 3.4).
 *
 * General rules
 *   - Every pointer named "device" is a pointer to GPU memory owned by the caller
 *     (for example a torch tensor); the small structs themselves and the pointer
 *     arrays inside them live in HOST memory and are read during the call only.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without waiting.  The library allocates nothing
 *     and keeps no pointer after a call returns.
 *   - Every function returns an lp_status and never throws or aborts; a message
 *     for the last failure on the calling thread is available from lp_last_error().
 *   - All floating point is IEEE binary32, tensors are dense and C-contiguous.
 */
#ifndef LIGHTPLANE_H
#define LIGHTPLANE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LP_MAX_LAYERS 8    /* linear layers of a decoder MLP */
#define LP_MAX_FEATURES 16 /* rendered feature channels of the two-MLP decoder */

typedef enum {
    LP_OK = 0,
    LP_ERR_INVALID_ARG = 1, /* NULL required pointer, non-positive size, dims mismatch      */
    LP_ERR_UNSUPPORTED = 2, /* valid, but no kernel of this library covers the shape       */
    LP_ERR_HIP = 3,         /* the HIP runtime reported an error (launch, attribute query) */
    LP_ERR_WORKSPACE = 4    /* workspace missing or smaller than lp_bwd_workspace_bytes     */
} lp_status;

typedef enum { LP_GRID_VOXEL = 0, LP_GRID_TRIPLANE = 1, LP_GRID_HASH = 2, LP_GRID_HEXPLANE = 3 } lp_grid_kind;

/* Storage type of the values of a hash structure that is READ (Section 3.2 notes that the
   hashing scheme is where precision and layout can be traded).  Gradients and the Splatter's
   outputs are always fp32. */
typedef enum { LP_F32 = 0, LP_BF16 = 1, LP_F16 = 2 } lp_dtype;

/*
 * The 3D hash structure theta (Section 3.2), channel-last.
 *   voxel   : data[0] = [B][NX][NY][NZ][C]                       (data[1], data[2] ignored)
 *   triplane: data[0] = [B][NX][NY][C], data[1] = [B][NY][NZ][C], data[2] = [B][NZ][NX][C];
 *             a point (x,y,z) reads plane 0 at (x,y), plane 1 at (y,z), plane 2 at (z,x)
 *             bilinearly and SUMS the three feature vectors.
 *   hash    : data[0] = [B][hash_size][C], a hash table (Section 3.2 names hash tables among the
 *             structures; the paper defines none, this one is the single-resolution spatial hash
 *             of Teschner et al. 2003 that Instant-NGP uses): the point is interpolated
 *             trilinearly in a virtual NX x NY x NZ lattice as in a voxel grid, but lattice corner
 *             (ix, iy, iz) is stored in entry ((ix * 1) xor (iy * 2654435761) xor (iz * 805459861))
 *             mod hash_size (products and xor in 32-bit unsigned arithmetic); corners that collide
 *             share the entry and their gradients add.  The Splatter writes such tables too
 *             (colliding corners pool what is pushed into them).
 *             The matrix-core kernels take tables whose hash_size is a power of two (16 or 32
 *             channels, or 16 channels under the merged two-MLP decoder); every other table runs
 *             on the generic kernels.
 *   hexplane: a structure over space AND time (Section 3.2 names HexPlane among the structures;
 *             the definition is Cao & Johnson 2023's): data[0..2] as the triplane's planes, and
 *             data_t[p] = [B][N_c][NT][C] the space-time plane over (c, t), c being the spatial
 *             axis that plane p leaves out (z, x, y for p = 0, 1, 2).  A point (x,y,z) of a ray
 *             with time t reads both planes of a pair bilinearly, multiplies the two feature
 *             vectors channel by channel, and SUMS the three products.  Time t_min maps to index 0
 *             and t_max to index NT - 1 of the time axis, times outside are clamped; contract
 *             coordinates act on the spatial axes only.  The gradient has six tensors (d_grid[p]
 *             for data[p], d_grid[3 + p] for data_t[p]).  Renderer only (the Splatter refuses it).
 *             The matrix-core kernels take 16 or 32 channels (or 16 channels under the merged
 *             two-MLP decoder); every other shape runs on the generic kernels.
 * World coordinate aabb_min[a] maps to index 0 and aabb_max[a] to index N_a - 1 along axis
 * a; positions outside the box are clamped onto it.  B scenes share the MLP.
 * contract_a: 0 = off.  In (0, 2]: contract coordinates (appendix, "Experimental Details",
 * equation CC) with foreground scale a: every axis of a sample position is first mapped by
 * CC(x) = 0.5 a x for |x| <= 1 and 0.5 ((2 - a)(1 - 1/|x|) + a) sign(x) beyond (the paper
 * converts the axes independently), which sends the whole line into (-1, 1) and the unit
 * interval onto [-a/2, a/2]; the box mapping above then applies to the contracted position
 * (use the box [-1, 1]^3).  Sample spacing stays the world distance along the ray.
 */
typedef struct {
    int32_t kind; /* lp_grid_kind */
    int32_t B, C; /* scenes, feature channels (the paper's K) */
    int32_t NX, NY, NZ;
    const void* data[3]; /* device; elements of type `dtype` */
    float aabb_min[3], aabb_max[3];
    float contract_a;
    int32_t dtype; /* lp_dtype; LP_BF16 / LP_F16 halve the bytes a sample reads */
    int64_t hash_size; /* LP_GRID_HASH: entries of one scene's table, in [1, 2^31); else ignored */
    const void* data_t[3]; /* LP_GRID_HEXPLANE: device, the space-time planes; else ignored */
    int32_t NT;            /* LP_GRID_HEXPLANE: resolution of the time axis, >= 2 */
    float t_min, t_max;    /* LP_GRID_HEXPLANE: times of the first and last index, t_max > t_min */
} lp_grid;

/*
 * The tiny MLP g (Section 3.2): n_layers linear layers, ReLU after every layer but the
 * last.  dims[0] == C, dims[n_layers] == 4.  Output 0 through softplus is the density
 * sigma; outputs 1..3 through the logistic sigmoid are the colour.
 * W[l] = [dims[l+1]][dims[l]] row-major (out, in), b[l] = [dims[l+1]].
 */
typedef struct {
    int32_t n_layers;
    int32_t dims[LP_MAX_LAYERS + 1];
    const float* W[LP_MAX_LAYERS]; /* device */
    const float* b[LP_MAX_LAYERS]; /* device */
} lp_mlp;

/*
 * M rays with S samples each (the ray set of Section 3.3, whose R + 1 points per ray are read as S samples).  Sample j
 * (j = 1..S) sits at distance t_j = near + (j - 1/2) (far - near) / S from the origin along
 * the UNIT direction, so Delta = (far - near) / S is the world distance between samples.
 */
typedef struct {
    int64_t M;
    int32_t S;
    const float* origins; /* device [M][3] */
    const float* dirs;    /* device [M][3], unit length (not renormalised) */
    const float* near;    /* device [M] */
    const float* far;     /* device [M] */
    const int32_t* scene; /* device [M] scene index in [0,B), or NULL (all rays use scene 0) */
    const float* time;    /* device [M] time of every ray, or NULL (all rays at the grid's t_min);
                             read for LP_GRID_HEXPLANE only */
} lp_rays;

/* How the MLP contractions are evaluated by the matrix-core kernels. */
typedef enum {
    LP_MATH_DEFAULT = 0, /* the library's choice for the shape                            */
    LP_MATH_GENERIC = 1, /* scalar fp32 kernels for any layer widths (slow)               */
    LP_MATH_BF16X3 = 2   /* fp32 operands split into bf16 hi+lo, three MFMA products,
                            fp32 accumulation (matrix-core kernels; supported shapes only) */
} lp_math_mode;

/*
 * Forward (Eq. (1), Section 3.3).  With T_0 = 1, T_j = T_{j-1} exp(-sigma_j Delta),
 * w_j = T_{j-1} - T_j:
 *     rgb = sum_j w_j c_j + T_S bg,   alpha = 1 - T_S,   depth = sum_j w_j t_j.
 * Outputs (device, written, not accumulated): rgb [M][3], alpha [M], depth [M], and
 * ray_cache [M], the one scalar per ray the backward needs (Section 3.4; here the total
 * optical depth sum_j sigma_j Delta, opaque to the caller).  alpha, depth and ray_cache
 * may each be NULL if not wanted.  bg is a HOST array of 3 floats.  M == 0 is a no-op.
 */
lp_status lp_render_fwd(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                        const float bg[3], float* rgb, float* alpha, float* depth,
                        float* ray_cache, int32_t math_mode, void* stream);

/*
 * Backward (Eq. (2), Section 3.4): vector-Jacobian product of the forward for upstream
 * gradients d_rgb [M][3] (required), d_alpha [M], d_depth [M] (either may be NULL = zero),
 * all device.  Marches each ray in reverse, recomputes sampling and MLP, rebuilds the
 * transmittance from ray_cache (as written by lp_render_fwd for the SAME inputs), and
 * ACCUMULATES into (the caller zeroes or pre-loads them):
 *     d_grid[p] — same shape as grid->data[p] (device; triplane: all three required; HexPlane: six,
 *                 d_grid[3 + p] with the shape of grid->data_t[p]),
 *     dW[l], db[l] — same shapes as mlp->W[l], mlp->b[l] (device).
 * No gradient is produced for rays, near, far or bg.  `workspace` is device memory of at
 * least lp_bwd_workspace_bytes(...) bytes, 256-byte aligned, contents ignored on entry and
 * undefined on exit.  Grid gradients are summed with floating-point atomics, so they are
 * reproducible up to summation order only.
 */
lp_status lp_render_bwd(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                        const float bg[3], const float* d_rgb, const float* d_alpha,
                        const float* d_depth, const float* ray_cache, float* const d_grid[],
                        float* const dW[LP_MAX_LAYERS], float* const db[LP_MAX_LAYERS],
                        void* workspace, size_t workspace_bytes, int32_t math_mode,
                        void* stream);

/* Bytes of workspace lp_render_bwd needs for these shapes; independent of S and of M
   (it depends on the MLP size and the device's compute-unit count).  *bytes is written. */
lp_status lp_bwd_workspace_bytes(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                                 int32_t math_mode, size_t* bytes);

/*
 * lp_render_bwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and error behaviour as lp_render_bwd without `workspace`: the per-wave partial-sum
 * records of the MLP gradients go to a static device array of LP_STATIC_SCRATCH_BYTES that the
 * library holds on every GPU it runs on until the process ends.  The call allocates nothing.
 * A shape whose records need more (an MLP of more than about 8 000 parameters on the
 * matrix-core kernels) is refused with LP_ERR_UNSUPPORTED and a message that names both sizes.
 * All calls on one GPU share that array: calls that overlap on one GPU (different streams or
 * threads) race; calls that are ordered on one stream do not (the records are fully rewritten
 * by every call before they are read, nothing needs clearing).
 */
#define LP_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
lp_status lp_render_bwd_static(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                               const float bg[3], const float* d_rgb, const float* d_alpha,
                               const float* d_depth, const float* ray_cache, float* const d_grid[],
                               float* const dW[LP_MAX_LAYERS], float* const db[LP_MAX_LAYERS],
                               int32_t math_mode, void* stream);

/* 1 if the matrix-core (LP_MATH_BF16X3) kernels cover this grid kind / MLP shape, else 0. */
int32_t lp_has_fast_path(const lp_grid* grid, const lp_mlp* mlp);

/* ---- The Renderer with the paper's own decoder (Section 3.3, text below Eq. (1)) ----------
 *
 * Two MLPs instead of one: the opacity MLP g_sigma maps the sampled feature to the density
 * (one output, through softplus); the feature MLP g_v maps the sampled feature AND the
 * encoded view direction to the n_feat rendered features f_v ("e.g. colors"):
 *     sigma_j = softplus(g_sigma(h(x_j))),   f_j = act(g_v([h(x_j) ; enc(d)])),
 *     out = sum_j w_j f_j + T_S bg   (n_feat channels),   alpha, depth as in lp_render_fwd.
 * enc(d) = (d, sin(2^k pi d), cos(2^k pi d) for k = 0 .. n_freq-1), component by component:
 * 3 + 6 n_freq values (the paper does not give the form; n_freq = 0 is the raw direction).
 * act = logistic sigmoid (LP_FEAT_SIGMOID) or identity (LP_FEAT_IDENTITY).
 * opacity.dims[0] == C, last == 1; feature.dims[0] == C + 3 + 6 n_freq, last == n_feat;
 * both MLPs need at least one hidden layer (n_layers >= 2); 1 <= n_feat <= LP_MAX_FEATURES;
 * 0 <= n_freq <= 4.  No gradient is produced for the directions.
 */
typedef enum { LP_FEAT_SIGMOID = 0, LP_FEAT_IDENTITY = 1 } lp_feat_act;

typedef struct {
    lp_mlp opacity; /* g_sigma */
    lp_mlp feature; /* g_v */
    int32_t n_freq;
    int32_t n_feat;
    int32_t feat_act; /* lp_feat_act */
} lp_decoder;

/* Bytes of device workspace the two calls below need (either pointer may be NULL).
   Independent of S and M.  The workspace holds the two MLPs merged into one block-structured
   MLP (and, for the backward, its gradient and the partial-sum records). */
lp_status lp_dec_workspace_bytes(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                                 int32_t math_mode, size_t* fwd_bytes, size_t* bwd_bytes);

/* Forward.  out [M][n_feat], alpha [M], depth [M], ray_cache [M] (device; the last three may
   be NULL); bg is a HOST array of n_feat floats; workspace: device, 256-byte aligned, at least
   the fwd_bytes of lp_dec_workspace_bytes, contents ignored on entry, undefined on exit. */
lp_status lp_render_dec_fwd(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                            const float* bg, float* out, float* alpha, float* depth, float* ray_cache,
                            void* workspace, size_t workspace_bytes, int32_t math_mode, void* stream);

/* Backward: upstream gradients d_out [M][n_feat] (required), d_alpha, d_depth (may be NULL);
   ACCUMULATES into d_grid (as lp_render_bwd) and into dW_opacity[l], db_opacity[l],
   dW_feature[l], db_feature[l] (device, shapes of the decoder's weights and biases).
   workspace: at least the bwd_bytes of lp_dec_workspace_bytes. */
lp_status lp_render_dec_bwd(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                            const float* bg, const float* d_out, const float* d_alpha,
                            const float* d_depth, const float* ray_cache, float* const d_grid[],
                            float* const dW_opacity[LP_MAX_LAYERS], float* const db_opacity[LP_MAX_LAYERS],
                            float* const dW_feature[LP_MAX_LAYERS], float* const db_feature[LP_MAX_LAYERS],
                            void* workspace, size_t workspace_bytes, int32_t math_mode, void* stream);

/* 1 if the matrix-core kernels cover this grid kind / decoder shape, else 0.  Covered, for
   three features (sigmoid or identity) on grids of any storage type: 16 grid channels with a merged hidden width (opacity +
   feature MLP, layer by layer) of 32 or 64, one or two hidden layers, at most 16 direction
   inputs; and 16 or 32 grid channels with two 3-layer MLPs of width 64 each (the paper's
   experimental size, any n_freq), which run as two chains. */
int32_t lp_dec_has_fast_path(const lp_grid* grid, const lp_decoder* dec);

/* ---- Splatter (Section 3.3 "Splatter"; appendix "Normalization Process in Splatter") ---------
 *
 * The dual of the Renderer: M pixels with feature vectors are expanded into rays of S points
 * (placed like the Renderer's samples); every point pushes a feature vector into the target
 * hash structure with the interpolation weights the Renderer reads that cell with, and each
 * cell is finally divided by the sum of the weights that landed on it:
 *     theta[corner] += weight * vt_ij,  theta_w[corner] += weight,  out = theta / theta_w
 * (0 where nothing landed).  Naive Splatter (mlp == NULL, n_in == target->C): vt_ij = v_i.
 * With the MLP g_s: vt_ij = g_s([v_i ; h_prior(x_ij) ; enc(d_i)]) with h_prior the prior
 * structure read at the point (prior == NULL: none) and enc the direction encoding of the
 * two-MLP decoder above (n_freq = -1: none); ReLU hidden layers, linear output;
 * mlp->dims[0] == n_in + prior->C + (3 + 6 n_freq), mlp->dims[last] == target->C.
 * The prior has the target's kind, scene count, box and contraction; its own resolution (and,
 * for hash tables, its own hash_size).  Targets: voxel grids, triplanes and hash tables (a
 * HexPlane target is refused with LP_ERR_UNSUPPORTED).
 */
typedef struct {
    int32_t n_in;         /* channels of the pixel features */
    int32_t n_freq;       /* octaves of the direction encoding fed to the MLP, -1: none */
    const float* feats;   /* device [M][n_in] */
    const lp_grid* prior; /* NULL: none */
    const lp_mlp* mlp;    /* NULL: naive Splatter */
} lp_splat;

/* Forward.  target gives kind, B, C, resolution, box and contraction of the structure to
   build (its data pointers are ignored).  theta[p] (shape of the target's tensors) and
   theta_w[p] (same without the channel axis) are device buffers that are WRITTEN: the
   normalised structure and the weight sums (the backward needs the latter). */
lp_status lp_splat_fwd(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                       float* const theta[3], float* const theta_w[3], void* stream);

/* 1 if lp_splat_fwd (and, with an MLP, lp_splat_bwd) runs this target / splat on the
   wavefront-per-ray kernels, else 0 (generic kernels, same results).  Covered: targets of 16 or
   32 channels, with or without contract coordinates (voxel grids, triplanes and, for the naive
   Splatter, hash tables whose size is a power of two); with an MLP, voxel grids and triplanes
   with a prior of the same channel count and contraction in fp32, one or two hidden layers of
   width 64, and at most 48 pixel-feature plus direction-encoding inputs.  Nothing behind the
   device pointers is read. */
int32_t lp_splat_has_fast_path(const lp_grid* target, const lp_splat* splat);

/* Backward for d_theta[p] = dL/d(out) (device).  The weights depend on the ray geometry only,
   so dL/dtheta = d_theta / theta_w; the gradient of a pushed feature is that field read at
   the point.  d_feats [M][n_in] is WRITTEN; d_prior[p] (shapes of the prior's tensors),
   dW[l], db[l] are ACCUMULATED into (NULL lists are allowed where there is no prior / MLP).
   workspace: device, 256-byte aligned, lp_splat_bwd_workspace_bytes bytes. */
lp_status lp_splat_bwd(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                       const float* const theta_w[3], const float* const d_theta[3], float* d_feats,
                       float* const d_prior[3], float* const dW[LP_MAX_LAYERS],
                       float* const db[LP_MAX_LAYERS], void* workspace, size_t workspace_bytes,
                       void* stream);

lp_status lp_splat_bwd_workspace_bytes(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                                       size_t* bytes);

/* Diagnostics, not part of the method: how one SIMD of this GPU overlaps matrix instructions
   (32x32x16 bf16 products, 32 cycles each) with vector instructions (4 cycles each); the split of
   the Renderer's backward into two waves per ray follows from it.  ns_per_iteration (host, 10
   floats) receives nanoseconds per loop iteration of
     [0..3]  one wave per SIMD issuing one product followed by 0, 4, 8, 12 independent vector
             multiply-adds (a sum 32 + 4 K cycles means no overlap inside a wave);
     [4..6]  two waves per SIMD, waves w and w + 4 of a workgroup paired: the first issues 8 products
             per iteration, the second 64 multiply-adds; only the first works, only the second, both;
     [7..9]  the same with waves w and w + 1 paired.
   Allocates and frees a small device buffer; synchronises the stream. */
lp_status lp_diag_coexecution(float* ns_per_iteration, void* stream);

/* Diagnostics, not part of the method: the rate at which this GPU retires fp32 atomic adds that cover
   whole 64-byte lines (16 lanes per line), the unit the gradient scatter of the backward works in
   (Section 3.4: the backward adds every sample's feature gradient into the structure).
   lines_per_second (host, 6 floats): lines drawn at random from 256 MiB with 4, 2, 1 lines per
   instruction [0..2]; from 256 KiB with 4 lines per instruction [3]; neighbouring lines (a walk) in
   256 MiB and in 256 KiB [4..5].  Allocates and frees 256 MiB of device memory; synchronises the
   stream. */
lp_status lp_diag_atomic_rate(float* lines_per_second, void* stream);

/* Diagnostics of a MEASUREMENT build (the library compiled with -DLP_WS_PHASES; an ordinary build
   returns LP_ERR_UNSUPPORTED): cycles the two roles of the two-wave backward have spent in the
   phases of their steps since the last call, summed over all waves.  cycles (host, 32 values):
   [0..10] chain wave (step start, sampling issue, forward, hand-over of h1 and h2, Eq. (2), hand-over
   of the output gradients, first link of the input-gradient chain, hand-over of dZ2, second link,
   hand-over of the features, records and dZ1, interpolation of the next step's features),
   [16..26] weights wave (step start, h2 taken and transposed, wait for the output gradients, dWo, h1
   transposed, wait for dZ2, dW2, features taken and transposed, wait for dZ1, feature gradient and
   dW1, walk).  The sums are cleared by the call. */
lp_status lp_diag_ws_phases(unsigned long long* cycles);

/* Message of the last failure on this thread ("" if none).  Owned by the library. */
const char* lp_last_error(void);

/* Library version, major * 1000 + minor. */
int32_t lp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LIGHTPLANE_H */
