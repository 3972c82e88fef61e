// C-ABI entry points of the library: argument validation, translation of the host
// structs into device-side views, choice of kernel family, launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>

#include "lightplane.h"
#include "lp_kernels.h"

namespace {

thread_local std::string g_last_error;

lp_status fail(lp_status s, const std::string& msg)
{
    g_last_error = msg;
    return s;
}

constexpr size_t kMaxLds = 160 * 1024;   // LDS per compute unit on gfx950
constexpr int kGenericLanes = 64;
constexpr int kMaxDevices = 64;

int compute_units(int* out_n_cu, std::string* err)
{
    static int cached[kMaxDevices] = {0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { *err = std::string("hipGetDevice: ") + hipGetErrorString(e); return 1; }
    if (dev >= 0 && dev < kMaxDevices && cached[dev] > 0) { *out_n_cu = cached[dev]; return 0; }
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || n <= 0) {
        *err = std::string("hipDeviceGetAttribute(MultiprocessorCount): ") + hipGetErrorString(e);
        return 1;
    }
    if (dev >= 0 && dev < kMaxDevices) cached[dev] = n;
    *out_n_cu = n;
    return 0;
}

lp_status validate(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays)
{
    if (!grid || !mlp || !rays) return fail(LP_ERR_INVALID_ARG, "grid, mlp and rays must not be NULL");
    if (grid->kind != LP_GRID_VOXEL && grid->kind != LP_GRID_TRIPLANE && grid->kind != LP_GRID_HASH &&
        grid->kind != LP_GRID_HEXPLANE)
        return fail(LP_ERR_INVALID_ARG,
                    "grid->kind must be LP_GRID_VOXEL, LP_GRID_TRIPLANE, LP_GRID_HASH or LP_GRID_HEXPLANE");
    if (grid->kind == LP_GRID_HEXPLANE) {
        if (grid->NT < 2) return fail(LP_ERR_INVALID_ARG, "grid->NT must be >= 2 for a HexPlane");
        if (!std::isfinite(grid->t_min) || !std::isfinite(grid->t_max) || !(grid->t_max > grid->t_min))
            return fail(LP_ERR_INVALID_ARG, "grid->t_max must exceed grid->t_min (finite values)");
        for (int p = 0; p < 3; ++p)
            if (!grid->data_t[p]) return fail(LP_ERR_INVALID_ARG, "grid->data_t has a NULL tensor");
    }
    if (grid->kind == LP_GRID_HASH && (grid->hash_size < 1 || grid->hash_size >= (1ll << 31)))
        return fail(LP_ERR_INVALID_ARG, "grid->hash_size must be in [1, 2^31) for a hash table");
    if (grid->B < 1 || grid->C < 1) return fail(LP_ERR_INVALID_ARG, "grid->B and grid->C must be >= 1");
    if (grid->NX < 2 || grid->NY < 2 || grid->NZ < 2)
        return fail(LP_ERR_INVALID_ARG, "every grid resolution must be >= 2");
    const int n_planes = (grid->kind == LP_GRID_TRIPLANE || grid->kind == LP_GRID_HEXPLANE) ? 3 : 1;
    for (int p = 0; p < n_planes; ++p)
        if (!grid->data[p]) return fail(LP_ERR_INVALID_ARG, "grid->data has a NULL tensor");
    for (int a = 0; a < 3; ++a) {
        if (!std::isfinite(grid->aabb_min[a]) || !std::isfinite(grid->aabb_max[a]) ||
            !(grid->aabb_max[a] > grid->aabb_min[a]))
            return fail(LP_ERR_INVALID_ARG, "aabb_max must exceed aabb_min on every axis (finite values)");
    }
    if (grid->dtype != LP_F32 && grid->dtype != LP_BF16 && grid->dtype != LP_F16)
        return fail(LP_ERR_INVALID_ARG, "grid->dtype must be LP_F32, LP_BF16 or LP_F16");
    if (!(grid->contract_a >= 0.0f && grid->contract_a <= 2.0f))
        return fail(LP_ERR_INVALID_ARG, "grid->contract_a must be 0 (off) or in (0, 2]");
    if (mlp->n_layers < 1 || mlp->n_layers > LP_MAX_LAYERS)
        return fail(LP_ERR_INVALID_ARG, "mlp->n_layers must be in [1, LP_MAX_LAYERS]");
    for (int l = 0; l <= mlp->n_layers; ++l)
        if (mlp->dims[l] < 1) return fail(LP_ERR_INVALID_ARG, "mlp->dims entries must be >= 1");
    if (mlp->dims[0] != grid->C) return fail(LP_ERR_INVALID_ARG, "mlp->dims[0] must equal grid->C");
    if (mlp->dims[mlp->n_layers] != 4)
        return fail(LP_ERR_INVALID_ARG, "the last MLP layer must have 4 outputs (density + rgb)");
    for (int l = 0; l < mlp->n_layers; ++l)
        if (!mlp->W[l] || !mlp->b[l]) return fail(LP_ERR_INVALID_ARG, "mlp->W / mlp->b has a NULL layer");
    if (rays->M < 0) return fail(LP_ERR_INVALID_ARG, "rays->M must be >= 0");
    if (rays->S < 1) return fail(LP_ERR_INVALID_ARG, "rays->S must be >= 1");
    if (rays->M > 0 && (!rays->origins || !rays->dirs || !rays->near || !rays->far))
        return fail(LP_ERR_INVALID_ARG, "rays->origins, dirs, near and far must not be NULL");
    return LP_OK;
}

void to_device_views(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays, lp::GridDev* g,
                     lp::MlpDev* m, lp::RaysDev* r)
{
    std::memset(g, 0, sizeof(*g));
    g->kind = grid->kind; g->B = grid->B; g->C = grid->C;
    g->N[0] = grid->NX; g->N[1] = grid->NY; g->N[2] = grid->NZ;
    for (int p = 0; p < 3; ++p) g->data[p] = grid->data[p];
    for (int a = 0; a < 3; ++a) {
        g->amin[a] = (double)grid->aabb_min[a];
        g->scale[a] = (double)(g->N[a] - 1) / ((double)grid->aabb_max[a] - (double)grid->aabb_min[a]);
    }
    g->contract = (double)grid->contract_a;
    g->dtype = grid->dtype;
    g->hash_size = grid->kind == LP_GRID_HASH ? (unsigned)grid->hash_size : 0u;
    if (grid->kind == LP_GRID_HEXPLANE) {
        for (int p = 0; p < 3; ++p) g->data_t[p] = grid->data_t[p];
        g->NT = grid->NT;
        g->tmin = (double)grid->t_min;
        g->tscale = (double)(grid->NT - 1) / ((double)grid->t_max - (double)grid->t_min);
    }
    std::memset(m, 0, sizeof(*m));
    m->n_layers = mlp->n_layers;
    int off = 0, maxw = 0, act = 0;
    for (int l = 0; l <= mlp->n_layers; ++l) {
        m->dims[l] = mlp->dims[l];
        maxw = mlp->dims[l] > maxw ? mlp->dims[l] : maxw;
        act += mlp->dims[l];
    }
    for (int l = 0; l < mlp->n_layers; ++l) {
        m->W[l] = mlp->W[l];
        m->b[l] = mlp->b[l];
        m->w_off[l] = off; off += mlp->dims[l] * mlp->dims[l + 1];
        m->b_off[l] = off; off += mlp->dims[l + 1];
    }
    m->param_total = off;
    m->max_width = maxw;
    m->act_total = act;
    m->n_freq = 0; m->n_enc = 0; m->n_feat = 3; m->feat_act = 0;
    r->M = rays->M; r->S = rays->S;
    r->origins = rays->origins; r->dirs = rays->dirs; r->near = rays->near; r->far = rays->far;
    r->scene = rays->scene;
    r->time = rays->time;
}

enum class Path { Generic, Mfma };

lp_status choose_path(const lp::GridDev& g, const lp::MlpDev& m, int32_t mode, Path* path)
{
    const bool fast = lp::mfma_supported(g, m);
    switch (mode) {
        case LP_MATH_DEFAULT: *path = fast ? Path::Mfma : Path::Generic; return LP_OK;
        case LP_MATH_GENERIC: *path = Path::Generic; return LP_OK;
        case LP_MATH_BF16X3:
            if (!fast) return fail(LP_ERR_UNSUPPORTED, "no matrix-core kernel for this grid kind / MLP shape");
            *path = Path::Mfma;
            return LP_OK;
        default: return fail(LP_ERR_INVALID_ARG, "unknown math_mode");
    }
}

// LDS of the generic kernels for `lanes` rays per block: the parameters (the backward: a second
// copy as gradient accumulators unless they are accumulated in the records), then `columns` floats
// per ray (activations and the kernels' own per-ray columns).
size_t generic_lds(const lp::MlpDev& m, int param_copies, size_t columns, int lanes)
{
    return sizeof(float) * ((size_t)param_copies * (size_t)m.param_total + columns * (size_t)lanes);
}

// Rays per block (64, or a partial wavefront of 32 / 16 / 8 when the activation columns of 64 rays
// would not fit beside the weights) and, for a backward, whether the gradients are accumulated in
// the records instead of in a second LDS copy of the parameters.  Returns false if nothing fits.
struct GenericShape {
    int lanes;
    int acc_in_record;
    size_t lds;
};

bool generic_shape(const lp::MlpDev& m, size_t columns, bool backward, GenericShape* out)
{
    for (int lanes = kGenericLanes; lanes >= 8; lanes /= 2)
        for (int in_record = 0; in_record <= (backward ? 1 : 0); ++in_record) {
            const size_t lds = generic_lds(m, backward && !in_record ? 2 : 1, columns, lanes);
            if (lds <= kMaxLds) {
                out->lanes = lanes;
                out->acc_in_record = in_record;
                out->lds = lds;
                return true;
            }
        }
    return false;
}

int ws_stride(const lp::MlpDev& m) { return (m.param_total + 63) / 64 * 64; }

int generic_bwd_blocks(int n_cu) { return 4 * n_cu; }

lp_status hip_fail(const char* what, hipError_t e)
{
    return fail(LP_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

lp_status run_fwd(const lp::GridDev& g, const lp::MlpDev& m, const lp::RaysDev& r, const lp::FwdOut& out, Path path,
                  int n_cu, hipStream_t s)
{
    if (path == Path::Mfma) {
        hipError_t e = lp::launch_fwd_mfma(g, m, r, out, n_cu, s);
        if (e != hipSuccess) return hip_fail("forward matrix-core kernel launch", e);
        return LP_OK;
    }
    GenericShape shape;
    if (!generic_shape(m, (size_t)m.act_total + m.n_feat, false, &shape))
        return fail(LP_ERR_UNSUPPORTED, "MLP too large for the generic forward kernel's LDS budget");
    hipError_t e = hipFuncSetAttribute((const void*)lp::fwd_generic_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shape.lds);
    if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(fwd_generic_kernel)", e);
    const long long blocks = (r.M + shape.lanes - 1) / shape.lanes;
    if (blocks > 0x7fffffffLL) return fail(LP_ERR_UNSUPPORTED, "too many rays for one launch");
    hipLaunchKernelGGL(lp::fwd_generic_kernel, dim3((unsigned)blocks), dim3(shape.lanes), shape.lds, s, g, m, r, out);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("forward generic kernel launch", e);
    return LP_OK;
}

// Backward kernels plus the reduction of the per-wave / per-block records into io.dW / io.db.
lp_status run_bwd(const lp::GridDev& g, const lp::MlpDev& m, const lp::RaysDev& r, const lp::BwdIo& io_in,
                  bool fast_bwd, int max_records, int n_cu, hipStream_t s)
{
    if (fast_bwd) {
        hipError_t e = lp::launch_bwd_mfma(g, m, r, io_in, n_cu, s);
        if (e != hipSuccess) return hip_fail("backward matrix-core kernel launch", e);
        return LP_OK;
    }
    GenericShape shape;
    const size_t cell_columns = m.max_width >= lp::kGenericCellColumns ? 0 : lp::kGenericCellColumns;
    if (!generic_shape(m, (size_t)m.act_total + 2 * (size_t)m.max_width + m.n_feat + cell_columns, true, &shape))
        return fail(LP_ERR_UNSUPPORTED, "MLP too large for the generic backward kernel's LDS budget");
    lp::BwdIo io = io_in;
    io.acc_in_record = shape.acc_in_record;
    hipError_t e = hipFuncSetAttribute((const void*)lp::bwd_generic_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shape.lds);
    if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(bwd_generic_kernel)", e);
    const long long n_tiles = (r.M + shape.lanes - 1) / shape.lanes;
    const long long blocks = n_tiles < max_records ? n_tiles : max_records;
    const long long tiles_per_block = (n_tiles + blocks - 1) / blocks;
    if (tiles_per_block > 0x7fffffffLL) return fail(LP_ERR_UNSUPPORTED, "too many rays for one launch");
    // blocks whose first tile is past the end write an all-zero record
    hipLaunchKernelGGL(lp::bwd_generic_kernel, dim3((unsigned)blocks), dim3(shape.lanes), shape.lds, s, g, m, r, io,
                       (int)tiles_per_block);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("backward generic kernel launch", e);
    hipLaunchKernelGGL(lp::reduce_params_kernel, dim3((m.param_total + 63) / 64), dim3(lp::kReduceThreads), 0, s,
                       m, io, (int)blocks);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("parameter-gradient reduction launch", e);
    return LP_OK;
}

// ---- the two-MLP decoder ----------------------------------------------------------------

lp_status validate_mlp_ptrs(const lp_mlp& m, const char* name)
{
    if (m.n_layers < 2 || m.n_layers > LP_MAX_LAYERS)
        return fail(LP_ERR_UNSUPPORTED, std::string(name) + ": n_layers must be in [2, LP_MAX_LAYERS] (at least one hidden layer)");
    for (int l = 0; l <= m.n_layers; ++l)
        if (m.dims[l] < 1) return fail(LP_ERR_INVALID_ARG, std::string(name) + ": dims entries must be >= 1");
    for (int l = 0; l < m.n_layers; ++l)
        if (!m.W[l] || !m.b[l]) return fail(LP_ERR_INVALID_ARG, std::string(name) + ": W / b has a NULL layer");
    return LP_OK;
}

// Validates grid, decoder and rays and builds the device views: the merged MLP `m` (its W / b
// point into `packed`, which may be NULL when only sizes are wanted) and the layout `d`.
lp_status decoder_views(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays, float* packed,
                        lp::GridDev* g, lp::MlpDev* m, lp::RaysDev* r, lp::DecLayout* d)
{
    if (!dec) return fail(LP_ERR_INVALID_ARG, "dec must not be NULL");
    // grid and rays are checked by the single-MLP validator with a stand-in MLP of the right ends
    lp_mlp stand_in;
    std::memset(&stand_in, 0, sizeof(stand_in));
    stand_in.n_layers = 1;
    stand_in.dims[0] = grid ? grid->C : 1;
    stand_in.dims[1] = 4;
    static const float dummy = 0.0f;
    stand_in.W[0] = &dummy; stand_in.b[0] = &dummy;
    lp_status st = validate(grid, &stand_in, rays);
    if (st != LP_OK) return st;
    if ((st = validate_mlp_ptrs(dec->opacity, "dec->opacity")) != LP_OK) return st;
    if ((st = validate_mlp_ptrs(dec->feature, "dec->feature")) != LP_OK) return st;
    if (dec->n_freq < 0 || dec->n_freq > 4) return fail(LP_ERR_INVALID_ARG, "dec->n_freq must be in [0, 4]");
    if (dec->n_feat < 1 || dec->n_feat > LP_MAX_FEATURES)
        return fail(LP_ERR_INVALID_ARG, "dec->n_feat must be in [1, LP_MAX_FEATURES]");
    if (dec->feat_act != LP_FEAT_SIGMOID && dec->feat_act != LP_FEAT_IDENTITY)
        return fail(LP_ERR_INVALID_ARG, "dec->feat_act must be LP_FEAT_SIGMOID or LP_FEAT_IDENTITY");
    const int C = grid->C, E = 3 + 6 * dec->n_freq;
    if (dec->opacity.dims[0] != C || dec->opacity.dims[dec->opacity.n_layers] != 1)
        return fail(LP_ERR_INVALID_ARG, "dec->opacity must map grid->C inputs to 1 output");
    if (dec->feature.dims[0] != C + E || dec->feature.dims[dec->feature.n_layers] != dec->n_feat)
        return fail(LP_ERR_INVALID_ARG, "dec->feature must map grid->C + 3 + 6 n_freq inputs to n_feat outputs");

    lp_mlp none;
    std::memset(&none, 0, sizeof(none));
    none.n_layers = 1; none.dims[0] = C; none.dims[1] = 4;
    to_device_views(grid, &none, rays, g, m, r);   // fills g and r; m is rebuilt below

    std::memset(d, 0, sizeof(*d));
    d->Ls = dec->opacity.n_layers; d->Lv = dec->feature.n_layers;
    d->L = d->Ls > d->Lv ? d->Ls : d->Lv;
    d->C = C; d->E = E;
    for (int l = 0; l <= d->Ls; ++l) d->dims_s[l] = dec->opacity.dims[l];
    for (int l = 0; l <= d->Lv; ++l) d->dims_v[l] = dec->feature.dims[l];
    for (int l = 0; l < d->Ls; ++l) { d->Ws[l] = dec->opacity.W[l]; d->bs[l] = dec->opacity.b[l]; }
    for (int l = 0; l < d->Lv; ++l) { d->Wv[l] = dec->feature.W[l]; d->bv[l] = dec->feature.b[l]; }

    std::memset(m, 0, sizeof(*m));
    m->n_layers = d->L;
    // 16 grid channels: pad the inputs to 32 (zero columns), the width the matrix-core kernels take
    lp::dec_combined_dims(*d, (C == 16 && C + E <= 32) ? 32 : C + E, m->dims);
    int off = 0, maxw = 0, act = 0;
    for (int l = 0; l <= m->n_layers; ++l) {
        maxw = m->dims[l] > maxw ? m->dims[l] : maxw;
        act += m->dims[l];
    }
    for (int l = 0; l < m->n_layers; ++l) {
        m->w_off[l] = off; off += m->dims[l] * m->dims[l + 1];
        m->b_off[l] = off; off += m->dims[l + 1];
        m->W[l] = packed ? packed + m->w_off[l] : nullptr;
        m->b[l] = packed ? packed + m->b_off[l] : nullptr;
    }
    m->param_total = off;
    m->max_width = maxw;
    m->act_total = act;
    m->n_freq = dec->n_freq; m->n_enc = E; m->n_feat = dec->n_feat; m->feat_act = dec->feat_act;
    return LP_OK;
}

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

// ---- Splatter ---------------------------------------------------------------------------

long long plane_cells(const lp_grid* g, int p)
{
    if (g->kind == LP_GRID_VOXEL) return (long long)g->B * g->NX * g->NY * g->NZ;
    if (g->kind == LP_GRID_HASH) return (long long)g->B * g->hash_size;
    const long long n[3] = {(long long)g->NX * g->NY, (long long)g->NY * g->NZ, (long long)g->NZ * g->NX};
    return (long long)g->B * n[p];
}

// Validates the arguments of a Splatter call and builds the device views.
lp_status splat_views(const lp_grid* target, const lp_rays* rays, const lp_splat* sp, lp::GridDev* g,
                      lp::MlpDev* m, lp::RaysDev* r, lp::SplatDev* sd)
{
    if (!sp) return fail(LP_ERR_INVALID_ARG, "splat must not be NULL");
    lp_mlp stand_in;
    std::memset(&stand_in, 0, sizeof(stand_in));
    stand_in.n_layers = 1;
    stand_in.dims[0] = target ? target->C : 1;
    stand_in.dims[1] = 4;
    static const float dummy = 0.0f;
    stand_in.W[0] = &dummy; stand_in.b[0] = &dummy;
    lp_grid tgt_checked;
    if (target) {   // the target's data pointers are not used: give the validator something non-NULL
        tgt_checked = *target;
        for (int p = 0; p < 3; ++p) tgt_checked.data[p] = &dummy;
    }
    lp_status st = validate(target ? &tgt_checked : nullptr, &stand_in, rays);
    if (st != LP_OK) return st;
    if (target->kind == LP_GRID_HEXPLANE)
        return fail(LP_ERR_UNSUPPORTED, "the Splatter writes voxel grids, triplanes and hash tables, not HexPlanes");
    if (sp->n_in < 1) return fail(LP_ERR_INVALID_ARG, "splat->n_in must be >= 1");
    if (rays->M > 0 && !sp->feats) return fail(LP_ERR_INVALID_ARG, "splat->feats must not be NULL");
    if (sp->n_freq < -1 || sp->n_freq > 4) return fail(LP_ERR_INVALID_ARG, "splat->n_freq must be in [-1, 4]");
    const int E = sp->n_freq < 0 ? 0 : 3 + 6 * sp->n_freq;
    lp_mlp none;
    std::memset(&none, 0, sizeof(none));
    none.n_layers = 1; none.dims[0] = target->C; none.dims[1] = 4;
    to_device_views(&tgt_checked, &none, rays, g, m, r);
    for (int p = 0; p < 3; ++p) g->data[p] = nullptr;
    std::memset(sd, 0, sizeof(*sd));
    sd->n_in = sp->n_in;
    sd->feats = sp->feats;
    int Cp = 0;
    if (sp->prior) {
        if (!sp->mlp) return fail(LP_ERR_INVALID_ARG, "a prior structure needs the MLP that consumes it");
        if (sp->prior->kind != target->kind || sp->prior->B != target->B)
            return fail(LP_ERR_INVALID_ARG, "splat->prior must have the target's kind and scene count");
        lp_mlp pm = none;
        pm.dims[0] = sp->prior->C;
        lp_mlp stand_p = stand_in;
        stand_p.dims[0] = sp->prior->C;
        st = validate(sp->prior, &stand_p, rays);
        if (st != LP_OK) return st;
        lp::MlpDev tmp; lp::RaysDev tr;
        to_device_views(sp->prior, &pm, rays, &sd->prior, &tmp, &tr);
        sd->has_prior = 1;
        Cp = sp->prior->C;
    }
    std::memset(m, 0, sizeof(*m));
    if (!sp->mlp) {
        if (sp->n_in != target->C) return fail(LP_ERR_INVALID_ARG, "the naive Splatter needs splat->n_in == target->C");
        if (E) return fail(LP_ERR_INVALID_ARG, "a direction encoding needs the MLP that consumes it");
        m->n_layers = 0;
        m->dims[0] = target->C;
        m->max_width = target->C;
        m->act_total = target->C;
        return LP_OK;
    }
    const lp_mlp* mlp = sp->mlp;
    if (mlp->n_layers < 1 || mlp->n_layers > LP_MAX_LAYERS)
        return fail(LP_ERR_INVALID_ARG, "splat->mlp->n_layers must be in [1, LP_MAX_LAYERS]");
    for (int l = 0; l <= mlp->n_layers; ++l)
        if (mlp->dims[l] < 1) return fail(LP_ERR_INVALID_ARG, "splat->mlp->dims entries must be >= 1");
    for (int l = 0; l < mlp->n_layers; ++l)
        if (!mlp->W[l] || !mlp->b[l]) return fail(LP_ERR_INVALID_ARG, "splat->mlp W / b has a NULL layer");
    if (mlp->dims[0] != sp->n_in + Cp + E || mlp->dims[mlp->n_layers] != target->C)
        return fail(LP_ERR_INVALID_ARG, "splat->mlp must map n_in + prior->C + (3 + 6 n_freq) inputs to target->C outputs");
    m->n_layers = mlp->n_layers;
    int off = 0, maxw = 0, act = 0;
    for (int l = 0; l <= mlp->n_layers; ++l) {
        m->dims[l] = mlp->dims[l];
        maxw = mlp->dims[l] > maxw ? mlp->dims[l] : maxw;
        act += mlp->dims[l];
    }
    for (int l = 0; l < mlp->n_layers; ++l) {
        m->W[l] = mlp->W[l];
        m->b[l] = mlp->b[l];
        m->w_off[l] = off; off += mlp->dims[l] * mlp->dims[l + 1];
        m->b_off[l] = off; off += mlp->dims[l + 1];
    }
    m->param_total = off; m->max_width = maxw; m->act_total = act;
    m->n_freq = sp->n_freq < 0 ? 0 : sp->n_freq; m->n_enc = E; m->n_feat = target->C; m->feat_act = 1;
    return LP_OK;
}


// ---- static scratch of lp_render_bwd_static -----------------------------------------------
// Device memory of the library's own for callers that cannot allocate: every GPU the library
// runs on holds its own copy of this array, at its own address, until the process ends.  In
// host code the name `scratch` is only a handle for hipGetSymbolAddress: the address a kernel
// may use is looked up once per device, with that device current, and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[LP_STATIC_SCRATCH_BYTES];

lp_status static_scratch_ptr(void** out)
{
    static void* g_scratch_ptr[kMaxDevices] = {nullptr};
    static std::mutex g_scratch_mutex;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(LP_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(LP_ERR_UNSUPPORTED, "device index beyond the library's table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(LP_ERR_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LP_OK;
}

// lp_render_bwd with the partial-sum records in `workspace` (the caller's, or the static scratch)
lp_status render_bwd_with(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                          const float bg[3], const float* d_rgb, const float* d_alpha,
                          const float* d_depth, const float* ray_cache, float* const d_grid[],
                          float* const dW[LP_MAX_LAYERS], float* const db[LP_MAX_LAYERS],
                          void* workspace, size_t workspace_bytes, bool static_scratch, int32_t math_mode,
                          void* stream)
{
    lp_status st = validate(grid, mlp, rays);

    if (st != LP_OK) return st;
    if (!bg || !d_grid || !dW || !db) return fail(LP_ERR_INVALID_ARG, "bg, d_grid, dW and db must not be NULL");
    const bool hexplane = grid->kind == LP_GRID_HEXPLANE;   // six gradient tensors: d_grid[3 + p] for data_t[p]
    const int n_planes = (grid->kind == LP_GRID_TRIPLANE || hexplane) ? 3 : 1;
    for (int p = 0; p < (hexplane ? 6 : n_planes); ++p)
        if (!d_grid[p]) return fail(LP_ERR_INVALID_ARG, "d_grid has a NULL tensor");
    for (int l = 0; l < mlp->n_layers; ++l)
        if (!dW[l] || !db[l]) return fail(LP_ERR_INVALID_ARG, "dW / db has a NULL layer");
    if (rays->M > 0 && (!d_rgb || !ray_cache))
        return fail(LP_ERR_INVALID_ARG, "d_rgb and ray_cache must not be NULL");
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r;
    to_device_views(grid, mlp, rays, &g, &m, &r);
    Path path;
    st = choose_path(g, m, math_mode, &path);
    if (st != LP_OK) return st;
    if (rays->M == 0) return LP_OK;

    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    const bool fast_bwd = path == Path::Mfma && lp::mfma_bwd_records(n_cu) > 0;
    const int max_records = fast_bwd ? lp::mfma_bwd_records(n_cu) : generic_bwd_blocks(n_cu);
    const size_t need = sizeof(float) * (size_t)max_records * (size_t)ws_stride(m);
    if (static_scratch) {
        if (need > (size_t)LP_STATIC_SCRATCH_BYTES)
            return fail(LP_ERR_UNSUPPORTED, "lp_render_bwd_static: this MLP needs " + std::to_string(need) +
                        " bytes of partial-sum records, more than the library's static scratch of " +
                        std::to_string((size_t)LP_STATIC_SCRATCH_BYTES) +
                        " bytes (LP_STATIC_SCRATCH_BYTES); use lp_render_bwd with a workspace");
        st = static_scratch_ptr(&workspace);
        if (st != LP_OK) return st;
        workspace_bytes = (size_t)LP_STATIC_SCRATCH_BYTES;
    }
    if (!workspace || workspace_bytes < need)
        return fail(LP_ERR_WORKSPACE, "workspace is NULL or smaller than lp_bwd_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(LP_ERR_WORKSPACE, "workspace must be 256-byte aligned");

    lp::BwdIo io;
    std::memset(&io, 0, sizeof(io));
    io.d_rgb = d_rgb; io.d_alpha = d_alpha; io.d_depth = d_depth; io.cache = ray_cache;
    for (int p = 0; p < 3; ++p) io.d_grid[p] = p < n_planes ? d_grid[p] : nullptr;
    for (int p = 0; p < 3; ++p) io.d_grid_t[p] = hexplane ? d_grid[3 + p] : nullptr;
    for (int l = 0; l < mlp->n_layers; ++l) { io.dW[l] = dW[l]; io.db[l] = db[l]; }
    for (int c = 0; c < 3; ++c) io.bg[c] = bg[c];
    io.ws = (float*)workspace;
    io.ws_stride = ws_stride(m);
    hipStream_t s = (hipStream_t)stream;

    return run_bwd(g, m, r, io, fast_bwd, max_records, n_cu, s);
}

}  // namespace

extern "C" {

const char* lp_last_error(void) { return g_last_error.c_str(); }

int32_t lp_version(void) { return 1000; }

int32_t lp_has_fast_path(const lp_grid* grid, const lp_mlp* mlp)
{
    if (!grid || !mlp) return 0;
    lp_rays dummy;
    std::memset(&dummy, 0, sizeof(dummy));
    dummy.S = 1;
    if (validate(grid, mlp, &dummy) != LP_OK) return 0;
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r;
    to_device_views(grid, mlp, &dummy, &g, &m, &r);
    return lp::mfma_supported(g, m) ? 1 : 0;
}

lp_status lp_render_fwd(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                        const float bg[3], float* rgb, float* alpha, float* depth,
                        float* ray_cache, int32_t math_mode, void* stream)
{
    lp_status st = validate(grid, mlp, rays);
    if (st != LP_OK) return st;
    if (!bg) return fail(LP_ERR_INVALID_ARG, "bg must not be NULL");
    if (rays->M > 0 && !rgb) return fail(LP_ERR_INVALID_ARG, "rgb must not be NULL");
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r;
    to_device_views(grid, mlp, rays, &g, &m, &r);
    Path path;
    st = choose_path(g, m, math_mode, &path);
    if (st != LP_OK) return st;
    if (rays->M == 0) return LP_OK;

    lp::FwdOut out;
    out.rgb = rgb; out.alpha = alpha; out.depth = depth; out.cache = ray_cache;
    for (int c = 0; c < 3; ++c) out.bg[c] = bg[c];
    hipStream_t s = (hipStream_t)stream;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);

    return run_fwd(g, m, r, out, path, n_cu, s);
}

lp_status lp_bwd_workspace_bytes(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                                 int32_t math_mode, size_t* bytes)
{
    if (!bytes) return fail(LP_ERR_INVALID_ARG, "bytes must not be NULL");
    lp_status st = validate(grid, mlp, rays);
    if (st != LP_OK) return st;
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r;
    to_device_views(grid, mlp, rays, &g, &m, &r);
    Path path;
    st = choose_path(g, m, math_mode, &path);
    if (st != LP_OK) return st;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    const bool fast_bwd = path == Path::Mfma && lp::mfma_bwd_records(n_cu) > 0;
    const int records = fast_bwd ? lp::mfma_bwd_records(n_cu) : generic_bwd_blocks(n_cu);
    *bytes = sizeof(float) * (size_t)records * (size_t)ws_stride(m);
    return LP_OK;
}

lp_status lp_render_bwd(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                        const float bg[3], const float* d_rgb, const float* d_alpha,
                        const float* d_depth, const float* ray_cache, float* const d_grid[],
                        float* const dW[LP_MAX_LAYERS], float* const db[LP_MAX_LAYERS],
                        void* workspace, size_t workspace_bytes, int32_t math_mode, void* stream)
{
    return render_bwd_with(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, workspace,
                           workspace_bytes, /*static_scratch=*/false, math_mode, stream);
}

lp_status lp_render_bwd_static(const lp_grid* grid, const lp_mlp* mlp, const lp_rays* rays,
                               const float bg[3], const float* d_rgb, const float* d_alpha,
                               const float* d_depth, const float* ray_cache, float* const d_grid[],
                               float* const dW[LP_MAX_LAYERS], float* const db[LP_MAX_LAYERS],
                               int32_t math_mode, void* stream)
{
    return render_bwd_with(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, nullptr, 0,
                           /*static_scratch=*/true, math_mode, stream);
}

int32_t lp_dec_has_fast_path(const lp_grid* grid, const lp_decoder* dec)
{
    lp_rays dummy;
    std::memset(&dummy, 0, sizeof(dummy));
    dummy.S = 1;
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::DecLayout d;
    if (decoder_views(grid, dec, &dummy, nullptr, &g, &m, &r, &d) != LP_OK) return 0;
    return (lp::mfma_supported(g, m) || lp::dec2_supported(g, d, m.n_feat, m.feat_act)) ? 1 : 0;
}

// kernel family and number of partial-sum records for a decoder call
lp_status decoder_path(const lp::GridDev& g, const lp::MlpDev& m, const lp::DecLayout& d, int32_t math_mode,
                       Path* path, int* records, bool* two_chains)
{
    // two 3-layer MLPs of width 64 run as two chains on the matrix cores (the merged MLP would be
    // 128 wide, which only the generic kernels take)
    *two_chains = math_mode != LP_MATH_GENERIC && !lp::mfma_supported(g, m) &&
                  lp::dec2_supported(g, d, m.n_feat, m.feat_act);
    lp_status st = LP_OK;
    if (*two_chains) {
        if (math_mode != LP_MATH_DEFAULT && math_mode != LP_MATH_BF16X3) return fail(LP_ERR_INVALID_ARG, "unknown math_mode");
        *path = Path::Mfma;
    } else {
        st = choose_path(g, m, math_mode, path);
    }
    if (st != LP_OK) return st;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    *records = *path == Path::Mfma ? lp::mfma_bwd_records(n_cu) : generic_bwd_blocks(n_cu);
    return LP_OK;
}

lp_status lp_dec_workspace_bytes(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                                 int32_t math_mode, size_t* fwd_bytes, size_t* bwd_bytes)
{
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::DecLayout d;
    lp_status st = decoder_views(grid, dec, rays, nullptr, &g, &m, &r, &d);
    if (st != LP_OK) return st;
    Path path;
    int records = 0;
    // alignment of the grid tensors decides the path too; sizes take the larger record count
    bool two_chains = false;
    st = decoder_path(g, m, d, math_mode, &path, &records, &two_chains);
    if (st != LP_OK) return st;
    const size_t params = align256(sizeof(float) * (size_t)m.param_total);
    if (fwd_bytes) *fwd_bytes = params;
    if (bwd_bytes) *bwd_bytes = 2 * params + sizeof(float) * (size_t)records * (size_t)ws_stride(m);
    return LP_OK;
}

lp_status lp_render_dec_fwd(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                            const float* bg, float* out, float* alpha, float* depth, float* ray_cache,
                            void* workspace, size_t workspace_bytes, int32_t math_mode, void* stream)
{
    size_t need = 0;
    lp_status st = lp_dec_workspace_bytes(grid, dec, rays, math_mode, &need, nullptr);
    if (st != LP_OK) return st;
    if (!bg) return fail(LP_ERR_INVALID_ARG, "bg must not be NULL");
    if (rays->M > 0 && !out) return fail(LP_ERR_INVALID_ARG, "out must not be NULL");
    if (rays->M == 0) return LP_OK;
    if (!workspace || workspace_bytes < need)
        return fail(LP_ERR_WORKSPACE, "workspace is NULL or smaller than lp_dec_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(LP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::DecLayout d;
    st = decoder_views(grid, dec, rays, (float*)workspace, &g, &m, &r, &d);
    if (st != LP_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    lp::FwdOut fo;
    fo.rgb = out; fo.alpha = alpha; fo.depth = depth; fo.cache = ray_cache;
    for (int c = 0; c < LP_MAX_FEATURES; ++c) fo.bg[c] = c < dec->n_feat ? bg[c] : 0.0f;
    Path path;
    int records = 0;
    bool two_chains = false;
    st = decoder_path(g, m, d, math_mode, &path, &records, &two_chains);
    if (st != LP_OK) return st;
    if (two_chains) {   // nothing to merge
        hipError_t e2 = lp::launch_dec2_fwd(g, lp::dec2_view(d, m.feat_act), r, fo, n_cu, s);
        if (e2 != hipSuccess) return hip_fail("two-chain decoder forward kernel launch", e2);
        return LP_OK;
    }
    hipError_t e = lp::launch_dec_pack(d, m, (float*)workspace, nullptr, s);
    if (e != hipSuccess) return hip_fail("decoder merge kernel launch", e);
    return run_fwd(g, m, r, fo, path, n_cu, s);
}

lp_status lp_render_dec_bwd(const lp_grid* grid, const lp_decoder* dec, const lp_rays* rays,
                            const float* bg, const float* d_out, const float* d_alpha,
                            const float* d_depth, const float* ray_cache, float* const d_grid[],
                            float* const dW_opacity[LP_MAX_LAYERS], float* const db_opacity[LP_MAX_LAYERS],
                            float* const dW_feature[LP_MAX_LAYERS], float* const db_feature[LP_MAX_LAYERS],
                            void* workspace, size_t workspace_bytes, int32_t math_mode, void* stream)
{
    size_t need = 0;
    lp_status st = lp_dec_workspace_bytes(grid, dec, rays, math_mode, nullptr, &need);
    if (st != LP_OK) return st;
    if (!bg || !d_grid || !dW_opacity || !db_opacity || !dW_feature || !db_feature)
        return fail(LP_ERR_INVALID_ARG, "bg, d_grid and the four gradient lists must not be NULL");
    const bool hexplane = grid->kind == LP_GRID_HEXPLANE;   // six gradient tensors: d_grid[3 + p] for data_t[p]
    const int n_planes = (grid->kind == LP_GRID_TRIPLANE || hexplane) ? 3 : 1;
    for (int p = 0; p < (hexplane ? 6 : n_planes); ++p)
        if (!d_grid[p]) return fail(LP_ERR_INVALID_ARG, "d_grid has a NULL tensor");
    for (int l = 0; l < dec->opacity.n_layers; ++l)
        if (!dW_opacity[l] || !db_opacity[l]) return fail(LP_ERR_INVALID_ARG, "dW_opacity / db_opacity has a NULL layer");
    for (int l = 0; l < dec->feature.n_layers; ++l)
        if (!dW_feature[l] || !db_feature[l]) return fail(LP_ERR_INVALID_ARG, "dW_feature / db_feature has a NULL layer");
    if (rays->M > 0 && (!d_out || !ray_cache)) return fail(LP_ERR_INVALID_ARG, "d_out and ray_cache must not be NULL");
    if (rays->M == 0) return LP_OK;
    if (!workspace || workspace_bytes < need)
        return fail(LP_ERR_WORKSPACE, "workspace is NULL or smaller than lp_dec_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(LP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::DecLayout d;
    st = decoder_views(grid, dec, rays, (float*)workspace, &g, &m, &r, &d);
    if (st != LP_OK) return st;
    for (int l = 0; l < d.Ls; ++l) { d.dWs[l] = dW_opacity[l]; d.dbs[l] = db_opacity[l]; }
    for (int l = 0; l < d.Lv; ++l) { d.dWv[l] = dW_feature[l]; d.dbv[l] = db_feature[l]; }
    hipStream_t s = (hipStream_t)stream;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    // workspace: merged parameters | merged gradient (zeroed by the merge kernel) | records
    const size_t params = align256(sizeof(float) * (size_t)m.param_total);
    float* packed = (float*)workspace;
    float* grads = (float*)((char*)workspace + params);
    Path path;
    int records = 0;
    bool two_chains = false;
    st = decoder_path(g, m, d, math_mode, &path, &records, &two_chains);
    if (st != LP_OK) return st;
    if (two_chains) {   // the two MLPs as they are: their gradients are accumulated in place
        lp::BwdIo io2;
        std::memset(&io2, 0, sizeof(io2));
        io2.d_rgb = d_out; io2.d_alpha = d_alpha; io2.d_depth = d_depth; io2.cache = ray_cache;
        for (int p = 0; p < 3; ++p) io2.d_grid[p] = p < n_planes ? d_grid[p] : nullptr;
        for (int c = 0; c < dec->n_feat; ++c) io2.bg[c] = bg[c];
        io2.ws = (float*)((char*)workspace + 2 * params);
        io2.ws_stride = ws_stride(m);
        hipError_t e2 = lp::launch_dec2_bwd(g, lp::dec2_view(d, m.feat_act), r, io2, n_cu, s);
        if (e2 != hipSuccess) return hip_fail("two-chain decoder backward kernel launch", e2);
        return LP_OK;
    }
    hipError_t e = lp::launch_dec_pack(d, m, packed, grads, s);
    if (e != hipSuccess) return hip_fail("decoder merge kernel launch", e);

    lp::BwdIo io;
    std::memset(&io, 0, sizeof(io));
    io.d_rgb = d_out; io.d_alpha = d_alpha; io.d_depth = d_depth; io.cache = ray_cache;
    for (int p = 0; p < 3; ++p) io.d_grid[p] = p < n_planes ? d_grid[p] : nullptr;
    for (int p = 0; p < 3; ++p) io.d_grid_t[p] = hexplane ? d_grid[3 + p] : nullptr;
    for (int l = 0; l < m.n_layers; ++l) { io.dW[l] = grads + m.w_off[l]; io.db[l] = grads + m.b_off[l]; }
    for (int c = 0; c < dec->n_feat; ++c) io.bg[c] = bg[c];
    io.ws = (float*)((char*)workspace + 2 * params);
    io.ws_stride = ws_stride(m);
    st = run_bwd(g, m, r, io, path == Path::Mfma, records, n_cu, s);
    if (st != LP_OK) return st;
    e = lp::launch_dec_unpack(d, m, grads, s);
    if (e != hipSuccess) return hip_fail("decoder gradient hand-back kernel launch", e);
    return LP_OK;
}

lp_status lp_splat_fwd(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                       float* const theta[3], float* const theta_w[3], void* stream)
{
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::SplatDev sd;
    lp_status st = splat_views(target, rays, splat, &g, &m, &r, &sd);
    if (st != LP_OK) return st;
    if (!theta || !theta_w) return fail(LP_ERR_INVALID_ARG, "theta and theta_w must not be NULL");
    const int n_planes = target->kind == LP_GRID_TRIPLANE ? 3 : 1;
    for (int p = 0; p < n_planes; ++p) {
        if (!theta[p] || !theta_w[p]) return fail(LP_ERR_INVALID_ARG, "theta / theta_w has a NULL tensor");
        sd.theta[p] = theta[p];
        sd.theta_w[p] = theta_w[p];
    }
    hipStream_t s = (hipStream_t)stream;
    const int threads = 256;
    for (int p = 0; p < n_planes; ++p) {
        const long long cells = plane_cells(target, p);
        hipLaunchKernelGGL(lp::fill_zero_kernel, dim3((unsigned)((cells * target->C + threads - 1) / threads)),
                           dim3(threads), 0, s, theta[p], cells * target->C);
        hipLaunchKernelGGL(lp::fill_zero_kernel, dim3((unsigned)((cells + threads - 1) / threads)), dim3(threads), 0,
                           s, theta_w[p], cells);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("Splatter clear kernels", e);
    if (rays->M > 0 && m.n_layers == 0 && lp::splat_naive_supported(g)) {
        // naive Splatter with 16 or 32 channels: wavefront per ray, run-merged whole-line atomics
        std::string err;
        int n_cu = 0;
        if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
        e = lp::launch_splat_naive(g, r, sd, n_cu, s);
        if (e != hipSuccess) return hip_fail("Splatter forward kernel launch", e);
    } else if (rays->M > 0 && m.n_layers > 0 && lp::splat_mfma_supported(g, m, sd)) {
        // MLP of the covered shapes: wavefront per ray, MLP on the matrix cores, the same push
        std::string err;
        int n_cu = 0;
        if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
        e = lp::launch_splat_mfma(g, m, r, sd, n_cu, s);
        if (e != hipSuccess) return hip_fail("Splatter forward kernel launch", e);
    } else if (rays->M > 0) {
        GenericShape shape;
        if (!generic_shape(m, (size_t)m.act_total, false, &shape))
            return fail(LP_ERR_UNSUPPORTED, "MLP too large for the Splatter kernel's LDS budget");
        e = hipFuncSetAttribute((const void*)lp::splat_fwd_generic_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)shape.lds);
        if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(splat_fwd_generic_kernel)", e);
        const long long blocks = (rays->M + shape.lanes - 1) / shape.lanes;
        if (blocks > 0x7fffffffLL) return fail(LP_ERR_UNSUPPORTED, "too many rays for one launch");
        hipLaunchKernelGGL(lp::splat_fwd_generic_kernel, dim3((unsigned)blocks), dim3(shape.lanes), shape.lds, s, g, m,
                           r, sd);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail("Splatter forward kernel launch", e);
    }
    for (int p = 0; p < n_planes; ++p) {
        const long long cells = plane_cells(target, p);
        hipLaunchKernelGGL(lp::splat_normalise_kernel, dim3((unsigned)((cells * target->C + threads - 1) / threads)),
                           dim3(threads), 0, s, theta[p], theta_w[p], cells, target->C);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("Splatter normalisation kernel launch", e);
    return LP_OK;
}

int32_t lp_splat_has_fast_path(const lp_grid* target, const lp_splat* splat)
{
    lp_rays dummy;
    std::memset(&dummy, 0, sizeof(dummy));
    dummy.S = 1;
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::SplatDev sd;
    if (splat_views(target, &dummy, splat, &g, &m, &r, &sd) != LP_OK) return 0;
    if (m.n_layers == 0) return lp::splat_naive_supported(g) ? 1 : 0;
    return lp::splat_mfma_supported(g, m, sd) ? 1 : 0;
}

lp_status lp_splat_bwd_workspace_bytes(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                                       size_t* bytes)
{
    if (!bytes) return fail(LP_ERR_INVALID_ARG, "bytes must not be NULL");
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::SplatDev sd;
    lp_status st = splat_views(target, rays, splat, &g, &m, &r, &sd);
    if (st != LP_OK) return st;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    const bool fast = m.n_layers > 0 && lp::splat_mfma_supported(g, m, sd);
    const int records = fast ? lp::mfma_bwd_records(n_cu) : generic_bwd_blocks(n_cu);
    *bytes = align256(sizeof(float) * (size_t)records * (size_t)ws_stride(m)) + 256;
    return LP_OK;
}

lp_status lp_splat_bwd(const lp_grid* target, const lp_rays* rays, const lp_splat* splat,
                       const float* const theta_w[3], const float* const d_theta[3], float* d_feats,
                       float* const d_prior[3], float* const dW[LP_MAX_LAYERS],
                       float* const db[LP_MAX_LAYERS], void* workspace, size_t workspace_bytes,
                       void* stream)
{
    size_t need = 0;
    lp_status st = lp_splat_bwd_workspace_bytes(target, rays, splat, &need);
    if (st != LP_OK) return st;
    lp::GridDev g; lp::MlpDev m; lp::RaysDev r; lp::SplatDev sd;
    st = splat_views(target, rays, splat, &g, &m, &r, &sd);
    if (st != LP_OK) return st;
    if (!theta_w || !d_theta) return fail(LP_ERR_INVALID_ARG, "theta_w and d_theta must not be NULL");
    if (rays->M > 0 && !d_feats) return fail(LP_ERR_INVALID_ARG, "d_feats must not be NULL");
    const int n_planes = target->kind == LP_GRID_TRIPLANE ? 3 : 1;
    lp::BwdIo io;
    std::memset(&io, 0, sizeof(io));
    for (int p = 0; p < n_planes; ++p) {
        if (!theta_w[p] || !d_theta[p]) return fail(LP_ERR_INVALID_ARG, "theta_w / d_theta has a NULL tensor");
        sd.theta_w_in[p] = theta_w[p];
        sd.d_theta[p] = d_theta[p];
        if (sd.has_prior) {
            if (!d_prior || !d_prior[p]) return fail(LP_ERR_INVALID_ARG, "d_prior has a NULL tensor");
            io.d_grid[p] = d_prior[p];
        }
    }
    for (int l = 0; l < m.n_layers; ++l) {
        if (!dW || !db || !dW[l] || !db[l]) return fail(LP_ERR_INVALID_ARG, "dW / db has a NULL layer");
        io.dW[l] = dW[l];
        io.db[l] = db[l];
    }
    sd.d_feats = d_feats;
    if (rays->M == 0) return LP_OK;
    if (!workspace || workspace_bytes < need)
        return fail(LP_ERR_WORKSPACE, "workspace is NULL or smaller than lp_splat_bwd_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(LP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    io.ws = (float*)workspace;
    io.ws_stride = ws_stride(m);
    hipStream_t s = (hipStream_t)stream;
    std::string err;
    int n_cu = 0;
    if (compute_units(&n_cu, &err)) return fail(LP_ERR_HIP, err);
    if (m.n_layers > 0 && lp::splat_mfma_supported(g, m, sd)) {
        // covered MLP shapes: wavefront per ray, MLP forward and backward on the matrix cores
        hipError_t e = lp::launch_splat_mfma_bwd(g, m, r, sd, io, n_cu, s);
        if (e != hipSuccess) return hip_fail("Splatter backward kernel launch", e);
        return LP_OK;
    }
    GenericShape shape;
    if (!generic_shape(m, (size_t)m.act_total + 2 * (size_t)m.max_width + sd.n_in, true, &shape))
        return fail(LP_ERR_UNSUPPORTED, "MLP too large for the Splatter backward kernel's LDS budget");
    io.acc_in_record = shape.acc_in_record;
    hipError_t e = hipFuncSetAttribute((const void*)lp::splat_bwd_generic_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shape.lds);
    if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(splat_bwd_generic_kernel)", e);
    const int max_records = generic_bwd_blocks(n_cu);
    const long long n_tiles = (rays->M + shape.lanes - 1) / shape.lanes;
    const long long blocks = n_tiles < max_records ? n_tiles : max_records;
    const long long tiles_per_block = (n_tiles + blocks - 1) / blocks;
    if (tiles_per_block > 0x7fffffffLL) return fail(LP_ERR_UNSUPPORTED, "too many rays for one launch");
    hipLaunchKernelGGL(lp::splat_bwd_generic_kernel, dim3((unsigned)blocks), dim3(shape.lanes), shape.lds, s, g, m, r,
                       sd, io, (int)tiles_per_block);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("Splatter backward kernel launch", e);
    if (m.param_total > 0) {
        hipLaunchKernelGGL(lp::reduce_params_kernel, dim3((m.param_total + 63) / 64), dim3(lp::kReduceThreads), 0,
                           s, m, io, (int)blocks);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail("parameter-gradient reduction launch", e);
    }
    return LP_OK;
}

}  // extern "C"
