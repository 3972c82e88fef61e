// Generic Renderer kernels: any channel count and any MLP widths, scalar fp32.
//
// One lane marches one ray (the granularity of the paper's own kernels, Section 3.4): it
// samples, decodes and composites sample after sample, keeping only the running
// transmittance and the rendered features.  A block is a single wavefront; MLP weights
// live in LDS, activations in LDS columns indexed [feature][lane] (conflict free).
// The host launches a block with fewer than 64 lanes (a partial wavefront) when the
// activation columns of 64 rays would not fit in LDS beside the weights.
// These kernels are the fallback for shapes the matrix-core kernels do not cover.
#include "lp_device.h"
#include "lp_kernels.h"

namespace lp {

namespace {

constexpr int kMaxLanes = 64;

// rays (= lanes) of this block
__device__ __forceinline__ int block_lanes() { return (int)blockDim.x; }

// Copies all weights and biases into LDS at sW[w_off[l]...] / sW[b_off[l]...].
__device__ void stage_params(const MlpDev& m, float* sW)
{
    for (int l = 0; l < m.n_layers; ++l) {
        const int nw = m.dims[l] * m.dims[l + 1];
        for (int i = threadIdx.x; i < nw; i += blockDim.x) sW[m.w_off[l] + i] = m.W[l][i];
        for (int i = threadIdx.x; i < m.dims[l + 1]; i += blockDim.x) sW[m.b_off[l] + i] = m.b[l][i];
    }
}

struct Cell {
    int i[3];
    float f[3];
    float g[3];  // 1 - f, rounded from the fp64 index
    // the ray's time on the time axis of a HexPlane (unset for the other structures)
    int it;
    float ft, gt;
};

__device__ __forceinline__ Cell locate(const GridDev& g, double x, double y, double z)
{
    Cell c;
    if (g.contract > 0.0) axis_cell<true>(x, g.amin[0], g.scale[0], g.N[0], g.contract, c.i[0], c.f[0], c.g[0]);
    else axis_cell<false>(x, g.amin[0], g.scale[0], g.N[0], g.contract, c.i[0], c.f[0], c.g[0]);
    if (g.contract > 0.0) axis_cell<true>(y, g.amin[1], g.scale[1], g.N[1], g.contract, c.i[1], c.f[1], c.g[1]);
    else axis_cell<false>(y, g.amin[1], g.scale[1], g.N[1], g.contract, c.i[1], c.f[1], c.g[1]);
    if (g.contract > 0.0) axis_cell<true>(z, g.amin[2], g.scale[2], g.N[2], g.contract, c.i[2], c.f[2], c.g[2]);
    else axis_cell<false>(z, g.amin[2], g.scale[2], g.N[2], g.contract, c.i[2], c.f[2], c.g[2]);
    return c;
}

// Channels [k, k + 4) of h(x), for fp32 structures whose channel count is a multiple of four and whose
// tensors are 16-byte aligned: one 16-byte load per corner instead of four loads.
__device__ __forceinline__ void fma4(float4& acc, float w, const float4& v)
{
    acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
}

__device__ float4 gather_channels4(const GridDev& g, int scene, const Cell& c, int k)
{
    const int C = g.C;
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    auto at = [](const void* base, size_t idx) { return *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + idx); };
    if (g.kind == LP_GRID_VOXEL || g.kind == LP_GRID_HASH) {
        const size_t V = (size_t)scene * (g.kind == LP_GRID_VOXEL ? (size_t)g.N[0] * g.N[1] * g.N[2] : (size_t)g.hash_size) * C;
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            const size_t off = g.kind == LP_GRID_VOXEL
                ? (((size_t)(c.i[0] + dx) * g.N[1] + (c.i[1] + dy)) * g.N[2] + (c.i[2] + dz)) * C
                : (size_t)hash_slot(c.i[0] + dx, c.i[1] + dy, c.i[2] + dz, g.hash_size) * C;
            fma4(acc, w, at(g.data[0], V + off + k));
        }
    } else {
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
            const size_t P = (size_t)scene * g.N[a] * g.N[b] * C;
            float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f), u = s;
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                fma4(s, (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]),
                     at(g.data[p], P + ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C + k));
            }
            if (g.kind == LP_GRID_HEXPLANE) {
                const size_t Q = (size_t)scene * g.N[cc] * g.NT * C;
                for (int d = 0; d < 4; ++d) {
                    const int da = d >> 1, db = d & 1;
                    fma4(u, (da ? c.f[cc] : c.g[cc]) * (db ? c.ft : c.gt),
                         at(g.data_t[p], Q + ((size_t)(c.i[cc] + da) * g.NT + (c.it + db)) * C + k));
                }
                acc.x += s.x * u.x; acc.y += s.y * u.y; acc.z += s.z * u.z; acc.w += s.w * u.w;
            } else {
                acc.x += s.x; acc.y += s.y; acc.z += s.z; acc.w += s.w;
            }
        }
    }
    return acc;
}

// feat[k*lanes + lane] = h(x)[k], k < C  (Section 3.2)
__device__ void gather_feat(const GridDev& g, int scene, const Cell& c, float* feat, int lane)
{
    const int C = g.C;
    {
        uintptr_t bits = 0;
        const int n_planes = g.kind == LP_GRID_VOXEL || g.kind == LP_GRID_HASH ? 1 : 3;
        for (int p = 0; p < n_planes; ++p) bits |= (uintptr_t)g.data[p];
        if (g.kind == LP_GRID_HEXPLANE)
            for (int p = 0; p < 3; ++p) bits |= (uintptr_t)g.data_t[p];
        if (g.dtype == LP_F32 && (C & 3) == 0 && (bits & 15u) == 0) {
            for (int k = 0; k < C; k += 4) {
                const float4 v = gather_channels4(g, scene, c, k);
                feat[(k + 0) * block_lanes() + lane] = v.x;
                feat[(k + 1) * block_lanes() + lane] = v.y;
                feat[(k + 2) * block_lanes() + lane] = v.z;
                feat[(k + 3) * block_lanes() + lane] = v.w;
            }
            return;
        }
    }
    if (g.kind == LP_GRID_VOXEL) {
        const size_t V = (size_t)scene * g.N[0] * g.N[1] * g.N[2] * C;  // first element of the scene
        for (int k = 0; k < C; ++k) {
            float acc = 0.0f;
            for (int d = 0; d < 8; ++d) {
                const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
                const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                                (dz ? c.f[2] : c.g[2]);
                const size_t off =
                    (((size_t)(c.i[0] + dx) * g.N[1] + (c.i[1] + dy)) * g.N[2] + (c.i[2] + dz)) * C;
                acc += w * grid_load(g, g.data[0], V + off + k);
            }
            feat[k * block_lanes() + lane] = acc;
        }
    } else if (g.kind == LP_GRID_HASH) {
        // trilinear over the 8 lattice corners, each read from its table entry
        const size_t V = (size_t)scene * g.hash_size * C;
        for (int k = 0; k < C; ++k) {
            float acc = 0.0f;
            for (int d = 0; d < 8; ++d) {
                const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
                const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                                (dz ? c.f[2] : c.g[2]);
                const size_t off = (size_t)hash_slot(c.i[0] + dx, c.i[1] + dy, c.i[2] + dz, g.hash_size) * C;
                acc += w * grid_load(g, g.data[0], V + off + k);
            }
            feat[k * block_lanes() + lane] = acc;
        }
    } else if (g.kind == LP_GRID_HEXPLANE) {
        // pair p: the spatial plane over axes (a, b) = (0,1), (1,2), (2,0) times the space-time plane
        // over (c, time), c the third axis; the three products are added
        for (int k = 0; k < C; ++k) {
            float acc = 0.0f;
            for (int p = 0; p < 3; ++p) {
                const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
                const size_t P = (size_t)scene * g.N[a] * g.N[b] * C, Q = (size_t)scene * g.N[cc] * g.NT * C;
                float s = 0.0f, u = 0.0f;
                for (int d = 0; d < 4; ++d) {
                    const int da = d >> 1, db = d & 1;
                    s += (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]) *
                         grid_load(g, g.data[p], P + ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C + k);
                    u += (da ? c.f[cc] : c.g[cc]) * (db ? c.ft : c.gt) *
                         grid_load(g, g.data_t[p], Q + ((size_t)(c.i[cc] + da) * g.NT + (c.it + db)) * C + k);
                }
                acc += s * u;
            }
            feat[k * block_lanes() + lane] = acc;
        }
    } else {
        // plane p spans axes (a, b) = (0,1), (1,2), (2,0)
        for (int k = 0; k < C; ++k) {
            float acc = 0.0f;
            for (int p = 0; p < 3; ++p) {
                const int a = p, b = (p + 1) % 3;
                const size_t P = (size_t)scene * g.N[a] * g.N[b] * C;
                for (int d = 0; d < 4; ++d) {
                    const int da = d >> 1, db = d & 1;
                    const float w = (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]);
                    acc += w * grid_load(g, g.data[p], P + ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C + k);
                }
            }
            feat[k * block_lanes() + lane] = acc;
        }
    }
}

// d_grid[corner][k] += weight * df for ONE channel k: the transpose of gather_feat, same corners and
// weights.  (HexPlane: d_grid_t holds the gradients of the space-time planes; by the product rule each
// plane of a pair receives df times the other plane's read, which is formed again here.)
__device__ void scatter_channel(const GridDev& g, float* const d_grid[3], float* const d_grid_t[3], int scene,
                                const Cell& c, int k, float df)
{
    const int C = g.C;
    if (g.kind == LP_GRID_VOXEL) {
        float* V = d_grid[0] + (size_t)scene * g.N[0] * g.N[1] * g.N[2] * C;
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            const size_t off =
                (((size_t)(c.i[0] + dx) * g.N[1] + (c.i[1] + dy)) * g.N[2] + (c.i[2] + dz)) * C;
            atomicAdd(V + off + k, w * df);
        }
    } else if (g.kind == LP_GRID_HASH) {
        float* V = d_grid[0] + (size_t)scene * g.hash_size * C;
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            const size_t off = (size_t)hash_slot(c.i[0] + dx, c.i[1] + dy, c.i[2] + dz, g.hash_size) * C;
            atomicAdd(V + off + k, w * df);
        }
    } else if (g.kind == LP_GRID_HEXPLANE) {
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3, cc = (p + 2) % 3;
            const size_t Ps = (size_t)scene * g.N[a] * g.N[b] * C, Qs = (size_t)scene * g.N[cc] * g.NT * C;
            float* P = d_grid[p] + Ps;
            float* Q = d_grid_t[p] + Qs;
            float s = 0.0f, u = 0.0f;
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                s += (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]) *
                     grid_load(g, g.data[p], Ps + ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C + k);
                u += (da ? c.f[cc] : c.g[cc]) * (db ? c.ft : c.gt) *
                     grid_load(g, g.data_t[p], Qs + ((size_t)(c.i[cc] + da) * g.NT + (c.it + db)) * C + k);
            }
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                atomicAdd(P + ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C + k,
                          (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]) * (df * u));
                atomicAdd(Q + ((size_t)(c.i[cc] + da) * g.NT + (c.it + db)) * C + k,
                          (da ? c.f[cc] : c.g[cc]) * (db ? c.ft : c.gt) * (df * s));
            }
        }
    } else {
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            float* P = d_grid[p] + (size_t)scene * g.N[a] * g.N[b] * C;
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                const float w = (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]);
                const size_t off = ((size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db)) * C;
                atomicAdd(P + off + k, w * df);
            }
        }
    }
}

// the lane's own sample: every channel of dfeat[k * lanes + lane]
__device__ void scatter_feat(const GridDev& g, float* const d_grid[3], int scene, const Cell& c,
                             const float* dfeat, int lane, float* const d_grid_t[3] = nullptr)
{
    for (int k = 0; k < g.C; ++k) scatter_channel(g, d_grid, d_grid_t, scene, c, k, dfeat[k * block_lanes() + lane]);
}

// The samples of a whole tile, channel by channel ACROSS lanes: consecutive lanes add consecutive
// channels of one sample's corner, so that an atomic instruction covers whole lines of a few samples
// instead of one float of 64 samples' lines.  `cells` holds kCellColumns columns [field][lane] with every
// lane's cell (see publish_cell); dz the feature gradients [channel][lane].  All lanes call it.
static_assert(kGenericCellColumns >= 14, "a cell has 14 fields");

__device__ __forceinline__ void publish_cell(float* cells, int lane, const Cell& c, int scene, bool live)
{
    const int L = block_lanes();
    int* ci = reinterpret_cast<int*>(cells);
    for (int a = 0; a < 3; ++a) {
        ci[a * L + lane] = c.i[a];
        cells[(4 + a) * L + lane] = c.f[a];
        cells[(8 + a) * L + lane] = c.g[a];
    }
    ci[3 * L + lane] = c.it;
    cells[7 * L + lane] = c.ft;
    cells[11 * L + lane] = c.gt;
    ci[12 * L + lane] = scene;
    ci[13 * L + lane] = live ? 1 : 0;
}

__device__ void scatter_tile(const GridDev& g, float* const d_grid[3], float* const d_grid_t[3], const float* cells,
                             const float* dz, int lane)
{
    const int L = block_lanes(), C = g.C;
    const int* ci = reinterpret_cast<const int*>(cells);
    const int per_pass = C <= L ? L / C : 1;   // samples served by one pass over the lanes
    const int sub = C <= L ? lane / C : 0;
    for (int rb = 0; rb < L; rb += per_pass) {
        const int r = rb + sub;
        if (sub >= per_pass || r >= L || ci[13 * L + r] == 0) continue;
        Cell c;
        for (int a = 0; a < 3; ++a) {
            c.i[a] = ci[a * L + r];
            c.f[a] = cells[(4 + a) * L + r];
            c.g[a] = cells[(8 + a) * L + r];
        }
        c.it = ci[3 * L + r];
        c.ft = cells[7 * L + r];
        c.gt = cells[11 * L + r];
        const int scene = ci[12 * L + r];
        for (int k = C <= L ? lane - sub * C : lane; k < C; k += L)   // (C <= L: the one channel of this lane)
            scatter_channel(g, d_grid, d_grid_t, scene, c, k, dz[k * L + r]);
    }
}

// Runs the MLP on the lane's column.  acts holds act_total columns: the input features
// followed by every layer's output (post-ReLU for hidden layers, linear for the last).
__device__ void mlp_forward(const MlpDev& m, const float* sW, float* acts, int lane)
{
    int off_in = 0, off_out = m.dims[0];
    for (int l = 0; l < m.n_layers; ++l) {
        const int nin = m.dims[l], nout = m.dims[l + 1];
        const float* W = sW + m.w_off[l];
        const float* B = sW + m.b_off[l];
        const bool hidden = l + 1 < m.n_layers;
        if ((nin & 3) == 0 && (m.w_off[l] & 3) == 0) {
            // eight outputs at a time, four inputs per step: the lane's four activations are read once
            // for eight rows of weights, and a row's four weights come as one 16-byte broadcast read
            // (three LDS reads per eight multiply-adds instead of sixteen)
            for (int o0 = 0; o0 < nout; o0 += 8) {
                float z[8];
                const float* row[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int o = min(o0 + i, nout - 1);   // rows beyond the layer repeat its last row; not stored
                    z[i] = B[o];
                    row[i] = W + o * nin;
                }
                for (int k = 0; k < nin; k += 4) {
                    const float a0 = acts[(off_in + k + 0) * block_lanes() + lane];
                    const float a1 = acts[(off_in + k + 1) * block_lanes() + lane];
                    const float a2 = acts[(off_in + k + 2) * block_lanes() + lane];
                    const float a3 = acts[(off_in + k + 3) * block_lanes() + lane];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float4 w = *reinterpret_cast<const float4*>(row[i] + k);
                        z[i] += w.x * a0 + w.y * a1 + w.z * a2 + w.w * a3;
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (o0 + i < nout) acts[(off_out + o0 + i) * block_lanes() + lane] = hidden ? fmaxf(z[i], 0.0f) : z[i];
            }
        } else {
            for (int o = 0; o < nout; ++o) {
                float z = B[o];
                for (int k = 0; k < nin; ++k) z += W[o * nin + k] * acts[(off_in + k) * block_lanes() + lane];
                acts[(off_out + o) * block_lanes() + lane] = hidden ? fmaxf(z, 0.0f) : z;
            }
        }
        off_in = off_out;
        off_out += nout;
    }
}

struct RayRegs {
    float o[3], d[3], near, delta;
    double delta64;
    int scene;
    float time;  // read by a HexPlane only
};

// cell of sample j: position in fp64 from the fp32 ray
__device__ __forceinline__ Cell sample_cell(const GridDev& g, const RayRegs& q, int j)
{
    const double t = (double)q.near + ((double)j + 0.5) * q.delta64;
    Cell c = locate(g, (double)q.o[0] + t * (double)q.d[0], (double)q.o[1] + t * (double)q.d[1],
                    (double)q.o[2] + t * (double)q.d[2]);
    // the time axis is not contracted
    if (g.kind == LP_GRID_HEXPLANE) axis_cell<false>((double)q.time, g.tmin, g.tscale, g.NT, 0.0, c.it, c.ft, c.gt);
    return c;
}

__device__ __forceinline__ RayRegs load_ray(const RaysDev& r, long long ray)
{
    RayRegs q;
    for (int a = 0; a < 3; ++a) {
        q.o[a] = r.origins[3 * ray + a];
        q.d[a] = r.dirs[3 * ray + a];
    }
    q.near = r.near[ray];
    q.delta64 = ((double)r.far[ray] - (double)q.near) / (double)r.S;
    q.delta = (float)q.delta64;
    q.scene = r.scene ? r.scene[ray] : 0;
    q.time = r.time ? r.time[ray] : -INFINITY;  // no times given: clamps onto the first index, the grid's t_min
    return q;
}

// Reverse of mlp_forward for the 64 columns of a tile.  dz holds dL/d(output) of the last layer
// (rows [0, dims[n_layers])), dz_next is scratch of the same size (max_width rows).  Adds the
// weight / bias gradients of the tile into sdW and returns the buffer that holds dL/d(input)
// (rows [0, dims[0])).  Every lane of the block must call it (it synchronises).
__device__ float* mlp_backward(const MlpDev& m, const float* sW, float* sdW, const float* acts, float* dz,
                               float* dz_next, int lane)
{
    int off_out = m.act_total - m.dims[m.n_layers];
    for (int l = m.n_layers - 1; l >= 0; --l) {
        const int nin = m.dims[l], nout = m.dims[l + 1];
        const int off_in = off_out - nin;
        const float* W = sW + m.w_off[l];
        __syncthreads();
        // weight and bias gradients: each lane owns a strided set of weights and sums
        // the outer product over the 64 rays of the tile
        // (every lane walks the rays of the tile starting at its own lane number: the lanes read
        // different rows at the same moment, and rows are a multiple of the LDS banks apart, so a
        // common starting ray would put all of them on one bank)
        const int L = block_lanes();
        if ((nin & 3) == 0 && (nout & 3) == 0 && (L & 3) == 0 && (((uintptr_t)acts | (uintptr_t)dz) & 15u) == 0) {
            // a lane owns 4 x 4 blocks of the weight matrix and reads four rays of a row at a time:
            // eight 16-byte reads per 64 multiply-adds
            const int tiles_k = nin >> 2, n_tiles = (nout >> 2) * tiles_k;
            for (int tile = lane; tile < n_tiles; tile += L) {
                const int o0 = (tile / tiles_k) << 2, k0 = (tile % tiles_k) << 2;
                float acc[4][4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
                const int r0 = (4 * lane) % L;
                for (int t = 0; t < L; t += 4) {
                    int r = r0 + t;
                    if (r >= L) r -= L;
                    float4 d[4], a[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        d[i] = *reinterpret_cast<const float4*>(dz + (o0 + i) * L + r);
                        a[i] = *reinterpret_cast<const float4*>(acts + (off_in + k0 + i) * L + r);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[i][j] += d[i].x * a[j].x + d[i].y * a[j].y + d[i].z * a[j].z + d[i].w * a[j].w;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) sdW[m.w_off[l] + (o0 + i) * nin + k0 + j] += acc[i][j];
            }
        } else {
            for (int idx = lane; idx < nin * nout; idx += L) {
                const int o = idx / nin, k = idx - o * nin;
                float s = 0.0f;
                for (int t = 0; t < L; ++t) {
                    int r = lane + t;
                    if (r >= L) r -= L;
                    s += dz[o * L + r] * acts[(off_in + k) * L + r];
                }
                sdW[m.w_off[l] + idx] += s;
            }
        }
        for (int o = lane; o < nout; o += block_lanes()) {
            float s = 0.0f;
            for (int t = 0; t < block_lanes(); ++t) {
                int r = lane + t;
                if (r >= block_lanes()) r -= block_lanes();
                s += dz[o * block_lanes() + r];
            }
            sdW[m.b_off[l] + o] += s;
        }
        // input gradient of the lane's own column, through the ReLU of the layer below
        if ((nin & 3) == 0 && (m.w_off[l] & 3) == 0) {
            // four inputs at a time: one 16-byte broadcast read of a weight row's four entries per output
            for (int k = 0; k < nin; k += 4) {
                float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
                for (int o = 0; o < nout; ++o) {
                    const float d = dz[o * block_lanes() + lane];
                    const float4 w = *reinterpret_cast<const float4*>(W + o * nin + k);
                    s0 += w.x * d; s1 += w.y * d; s2 += w.z * d; s3 += w.w * d;
                }
                const float sk[4] = {s0, s1, s2, s3};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool off = l > 0 && !(acts[(off_in + k + i) * block_lanes() + lane] > 0.0f);
                    dz_next[(k + i) * block_lanes() + lane] = off ? 0.0f : sk[i];
                }
            }
        } else {
            for (int k = 0; k < nin; ++k) {
                float s = 0.0f;
                for (int o = 0; o < nout; ++o) s += W[o * nin + k] * dz[o * block_lanes() + lane];
                if (l > 0 && !(acts[(off_in + k) * block_lanes() + lane] > 0.0f)) s = 0.0f;
                dz_next[k * block_lanes() + lane] = s;
            }
        }
        __syncthreads();
        float* tmp = dz; dz = dz_next; dz_next = tmp;
        off_out = off_in;
    }
    return dz;
}

// Inputs of the MLP beyond the grid channels: the encoded view direction of the lane's ray
// (constant along the ray), then zero padding up to dims[0].
__device__ void set_direction_inputs(const GridDev& g, const MlpDev& m, const RayRegs& q, float* acts, int lane)
{
    for (int e = g.C; e < m.dims[0]; ++e)
        acts[e * block_lanes() + lane] = e - g.C < m.n_enc ? dir_encoding(q.d, e - g.C) : 0.0f;
}

// rendered feature from the MLP output: logistic sigmoid (colours) or identity
__device__ __forceinline__ float feature_act(const MlpDev& m, float z)
{
    return m.feat_act == 0 ? logistic_f(z) : z;
}

// ---- Splatter (Section 3.3 "Splatter"; appendix "Normalization Process in Splatter") ----------
// One lane per pixel / ray, like the generic Renderer kernels.  Forward: every point of the ray
// pushes its feature vector (the pixel's, or the MLP's output for [pixel feature ; prior
// structure read at the point ; direction encoding]) into the target structure with the
// Renderer's interpolation weights, and the weight itself into a one-channel structure; a
// second kernel divides.  Backward: the gradient of a pushed feature is the normalised output
// gradient READ at the point; from there through the MLP as in the Renderer's backward.

// d_w[corner] += weight   (one channel, same cells and weights as scatter_feat)
__device__ void scatter_weight(const GridDev& g, float* const d_w[3], int scene, const Cell& c)
{
    if (g.kind == LP_GRID_HASH) {
        float* V = d_w[0] + (size_t)scene * g.hash_size;
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            atomicAdd(V + hash_slot(c.i[0] + dx, c.i[1] + dy, c.i[2] + dz, g.hash_size), w);
        }
    } else if (g.kind == LP_GRID_VOXEL) {
        float* V = d_w[0] + (size_t)scene * g.N[0] * g.N[1] * g.N[2];
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            atomicAdd(V + ((size_t)(c.i[0] + dx) * g.N[1] + (c.i[1] + dy)) * g.N[2] + (c.i[2] + dz), w);
        }
    } else {
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            float* P = d_w[p] + (size_t)scene * g.N[a] * g.N[b];
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                const float w = (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]);
                atomicAdd(P + (size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db), w);
            }
        }
    }
}

// feat[k*lanes + lane] = sum_corners weight * G[corner][k] / W[corner]   (0 where W == 0), k < C:
// the normalised output gradient read at the point
__device__ void gather_normalised(const GridDev& g, const float* const G[3], const float* const Wt[3], int scene,
                                  const Cell& c, float* feat, int lane)
{
    const int C = g.C;
    for (int k = 0; k < C; ++k) feat[k * block_lanes() + lane] = 0.0f;
    if (g.kind == LP_GRID_HASH) {
        const size_t cells = (size_t)scene * g.hash_size;
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            const size_t cell = cells + hash_slot(c.i[0] + dx, c.i[1] + dy, c.i[2] + dz, g.hash_size);
            const float ws = Wt[0][cell];
            const float s = ws > 0.0f ? w / ws : 0.0f;
            for (int k = 0; k < C; ++k) feat[k * block_lanes() + lane] += s * G[0][cell * C + k];
        }
    } else if (g.kind == LP_GRID_VOXEL) {
        const size_t cells = (size_t)scene * g.N[0] * g.N[1] * g.N[2];
        for (int d = 0; d < 8; ++d) {
            const int dx = d >> 2, dy = (d >> 1) & 1, dz = d & 1;
            const float w = (dx ? c.f[0] : c.g[0]) * (dy ? c.f[1] : c.g[1]) *
                            (dz ? c.f[2] : c.g[2]);
            const size_t cell = cells + ((size_t)(c.i[0] + dx) * g.N[1] + (c.i[1] + dy)) * g.N[2] + (c.i[2] + dz);
            const float ws = Wt[0][cell];
            const float s = ws > 0.0f ? w / ws : 0.0f;
            for (int k = 0; k < C; ++k) feat[k * block_lanes() + lane] += s * G[0][cell * C + k];
        }
    } else {
        for (int p = 0; p < 3; ++p) {
            const int a = p, b = (p + 1) % 3;
            const size_t cells = (size_t)scene * g.N[a] * g.N[b];
            for (int d = 0; d < 4; ++d) {
                const int da = d >> 1, db = d & 1;
                const float w = (da ? c.f[a] : c.g[a]) * (db ? c.f[b] : c.g[b]);
                const size_t cell = cells + (size_t)(c.i[a] + da) * g.N[b] + (c.i[b] + db);
                const float ws = Wt[p][cell];
                const float s = ws > 0.0f ? w / ws : 0.0f;
                for (int k = 0; k < C; ++k) feat[k * block_lanes() + lane] += s * G[p][cell * C + k];
            }
        }
    }
}

// per-ray inputs of the Splatter's MLP: the pixel feature (columns [0, n_in)) and the direction
// encoding (columns after the prior's channels)
__device__ void set_splat_ray_inputs(const SplatDev& sp, const MlpDev& m, const RayRegs& q, long long ray,
                                     float* acts, int lane)
{
    for (int k = 0; k < sp.n_in; ++k) acts[k * block_lanes() + lane] = sp.feats[(size_t)ray * sp.n_in + k];
    const int e0 = sp.n_in + (sp.has_prior ? sp.prior.C : 0);
    for (int e = 0; e < m.n_enc; ++e) acts[(e0 + e) * block_lanes() + lane] = dir_encoding(q.d, e);
}

}  // namespace

__global__ __launch_bounds__(kMaxLanes) void splat_fwd_generic_kernel(GridDev tgt, MlpDev m, RaysDev rays, SplatDev sp)
{
    extern __shared__ __align__(16) float smem[];
    float* sW = smem;
    float* acts = smem + m.param_total;
    stage_params(m, sW);
    __syncthreads();
    const int lane = threadIdx.x;
    const long long ray_raw = (long long)blockIdx.x * block_lanes() + lane;
    const bool live = ray_raw < rays.M;
    const long long ray = live ? ray_raw : rays.M - 1;
    const RayRegs q = load_ray(rays, ray);
    const int out_off = m.act_total - tgt.C;
    set_splat_ray_inputs(sp, m, q, ray, acts, lane);
    for (int j = 0; j < rays.S; ++j) {
        const Cell c = sample_cell(tgt, q, j);
        if (m.n_layers > 0) {
            if (sp.has_prior) gather_feat(sp.prior, q.scene, sample_cell(sp.prior, q, j), acts + sp.n_in * block_lanes(), lane);
            mlp_forward(m, sW, acts, lane);
        }
        if (live) {
            scatter_feat(tgt, sp.theta, q.scene, c, acts + out_off * block_lanes(), lane);
            scatter_weight(tgt, sp.theta_w, q.scene, c);
        }
    }
}

// theta[cell][k] /= theta_w[cell] (0 where nothing landed); one thread per element
__global__ void splat_normalise_kernel(float* theta, const float* theta_w, long long cells, int C)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cells * C) return;
    const float w = theta_w[i / C];
    theta[i] = w > 0.0f ? theta[i] / w : 0.0f;
}

__global__ void fill_zero_kernel(float* p, long long n)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// LDS: params | dparams accumulators | acts (act_total columns) | dz (2 * max_width columns) |
// pixel-feature gradients (n_in columns)
__global__ __launch_bounds__(kMaxLanes) void splat_bwd_generic_kernel(GridDev tgt, MlpDev m, RaysDev rays, SplatDev sp,
                                                                   BwdIo io, int tiles_per_block)
{
    extern __shared__ __align__(16) float smem[];
    float* sW = smem;
    // gradient accumulators of the block: in LDS, or (MLPs whose two copies do not fit) directly in
    // the block's record in the workspace; every element has one owner lane either way
    float* rec = io.ws + (size_t)blockIdx.x * io.ws_stride;
    float* sdW = io.acc_in_record ? rec : sW + m.param_total;
    float* acts = sW + (io.acc_in_record ? 1 : 2) * m.param_total;
    float* dz0 = acts + m.act_total * block_lanes();
    float* dz1 = dz0 + m.max_width * block_lanes();
    stage_params(m, sW);
    for (int i = threadIdx.x; i < m.param_total; i += blockDim.x) sdW[i] = 0.0f;
    __syncthreads();
    const int lane = threadIdx.x;
    const long long n_tiles = (rays.M + block_lanes() - 1) / block_lanes();

    for (int it = 0; it < tiles_per_block; ++it) {
        const long long tile = (long long)blockIdx.x * tiles_per_block + it;
        if (tile >= n_tiles) break;  // uniform over the block
        const long long ray_raw = tile * block_lanes() + lane;
        const bool live = ray_raw < rays.M;
        const long long ray = live ? ray_raw : rays.M - 1;
        const RayRegs q = load_ray(rays, ray);
        set_splat_ray_inputs(sp, m, q, ray, acts, lane);
        // gradient of the pixel feature, summed over the points of the ray: n_in columns after dz1
        float* dfe = dz1 + m.max_width * block_lanes();
        for (int k = 0; k < sp.n_in; ++k) dfe[k * block_lanes() + lane] = 0.0f;
        for (int j = 0; j < rays.S; ++j) {
            const Cell c = sample_cell(tgt, q, j);
            float* dz = dz0;
            gather_normalised(tgt, sp.d_theta, sp.theta_w_in, q.scene, c, dz, lane);
            if (!live)
                for (int k = 0; k < tgt.C; ++k) dz[k * block_lanes() + lane] = 0.0f;
            if (m.n_layers > 0) {
                Cell cp = c;
                if (sp.has_prior) {
                    cp = sample_cell(sp.prior, q, j);
                    gather_feat(sp.prior, q.scene, cp, acts + sp.n_in * block_lanes(), lane);
                }
                mlp_forward(m, sW, acts, lane);
                dz = mlp_backward(m, sW, sdW, acts, dz, dz1, lane);
                if (live && sp.has_prior) scatter_feat(sp.prior, io.d_grid, q.scene, cp, dz + sp.n_in * block_lanes(), lane);
            }
            for (int k = 0; k < sp.n_in; ++k) dfe[k * block_lanes() + lane] += dz[k * block_lanes() + lane];
        }
        if (live)
            for (int k = 0; k < sp.n_in; ++k) sp.d_feats[(size_t)ray * sp.n_in + k] = dfe[k * block_lanes() + lane];
    }
    __syncthreads();
    if (!io.acc_in_record)
        for (int i = threadIdx.x; i < m.param_total; i += blockDim.x) rec[i] = sdW[i];
}

namespace {

}  // namespace

__global__ __launch_bounds__(kMaxLanes) void fwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays,
                                                             FwdOut out)
{
    extern __shared__ __align__(16) float smem[];
    float* sW = smem;
    float* acts = smem + m.param_total;
    stage_params(m, sW);
    __syncthreads();

    const int lane = threadIdx.x;
    const long long ray_raw = (long long)blockIdx.x * block_lanes() + lane;
    const bool live = ray_raw < rays.M;
    const long long ray = live ? ray_raw : rays.M - 1;
    const RayRegs q = load_ray(rays, ray);
    const int F = m.n_feat, out_off = m.act_total - (1 + F);
    float* racc = acts + m.act_total * block_lanes();  // F columns: the rendered features
    set_direction_inputs(g, m, q, acts, lane);
    for (int ch = 0; ch < F; ++ch) racc[ch * block_lanes() + lane] = 0.0f;

    float T = 1.0f, tau = 0.0f, depth = 0.0f;
    for (int j = 0; j < rays.S; ++j) {
        const float t = q.near + ((float)j + 0.5f) * q.delta;
        const Cell c = sample_cell(g, q, j);
        gather_feat(g, q.scene, c, acts, lane);
        mlp_forward(m, sW, acts, lane);
        const float sigma = softplus_f(acts[(out_off + 0) * block_lanes() + lane]);
        const float sd = sigma * q.delta;
        const float Tn = T * expf(-sd);
        const float w = T - Tn;
        for (int ch = 0; ch < F; ++ch)
            racc[ch * block_lanes() + lane] += w * feature_act(m, acts[(out_off + 1 + ch) * block_lanes() + lane]);
        depth += w * t;
        tau += sd;
        T = Tn;
    }
    if (live) {
        for (int ch = 0; ch < F; ++ch) out.rgb[F * ray + ch] = racc[ch * block_lanes() + lane] + T * out.bg[ch];
        if (out.alpha) out.alpha[ray] = 1.0f - T;
        if (out.depth) out.depth[ray] = depth;
        if (out.cache) out.cache[ray] = tau;
    }
}

// Backward: reverse march with recomputation (Section 3.4).  Per sample q, from last to
// first:  tau_{q-1} = tau_q - sigma_q Delta,  T = exp(-tau)  (the paper's
// T_{q-1} = T_q exp(Delta sigma_q), kept in the log domain so that it survives T_S
// underflowing), then Eq. (2) with the running suffix sum of w_j a_j.
// LDS: params | dparams accumulators | acts (act_total columns) | dz (2 * max_width columns) |
// upstream feature gradients (n_feat columns) | the lanes' cells (kGenericCellColumns columns; only for
// MLPs narrower than that: otherwise the cells go into the dz buffer that the MLP backward leaves free).
__global__ __launch_bounds__(kMaxLanes) void bwd_generic_kernel(GridDev g, MlpDev m, RaysDev rays,
                                                             BwdIo io, int tiles_per_block)
{
    extern __shared__ __align__(16) float smem[];
    float* sW = smem;
    // gradient accumulators of the block: in LDS, or (MLPs whose two copies do not fit) directly in
    // the block's record in the workspace; every element has one owner lane either way
    float* rec = io.ws + (size_t)blockIdx.x * io.ws_stride;
    float* sdW = io.acc_in_record ? rec : sW + m.param_total;
    float* acts = sW + (io.acc_in_record ? 1 : 2) * m.param_total;
    float* dz0 = acts + m.act_total * block_lanes();
    float* dz1 = dz0 + m.max_width * block_lanes();
    float* pcol = dz1 + m.max_width * block_lanes();
    float* cells_extra = pcol + m.n_feat * block_lanes();   // present when max_width < kGenericCellColumns
    stage_params(m, sW);
    for (int i = threadIdx.x; i < m.param_total; i += blockDim.x) sdW[i] = 0.0f;
    __syncthreads();

    const int lane = threadIdx.x;
    const int F = m.n_feat, out_off = m.act_total - (1 + F);
    const long long n_tiles = (rays.M + block_lanes() - 1) / block_lanes();

    for (int it = 0; it < tiles_per_block; ++it) {
        const long long tile = (long long)blockIdx.x * tiles_per_block + it;
        if (tile >= n_tiles) break;  // uniform over the block
        const long long ray_raw = tile * block_lanes() + lane;
        const bool live = ray_raw < rays.M;
        const long long ray = live ? ray_raw : rays.M - 1;
        const RayRegs q = load_ray(rays, ray);
        set_direction_inputs(g, m, q, acts, lane);
        float pbg = 0.0f;  // p . bg
        for (int ch = 0; ch < F; ++ch) {
            const float p = live ? io.d_rgb[F * ray + ch] : 0.0f;
            pcol[ch * block_lanes() + lane] = p;
            pbg += p * io.bg[ch];
        }
        const float p_alpha = (live && io.d_alpha) ? io.d_alpha[ray] : 0.0f;
        const float p_depth = (live && io.d_depth) ? io.d_depth[ray] : 0.0f;
        const float tau_S = io.cache[ray];
        const float T_S = expf(-tau_S);
        // d(loss)/dT_S through alpha = 1 - T_S and the background term
        const float kS = T_S * (p_alpha - pbg);
        float tau = tau_S;   // optical depth up to and including the current sample
        float suffix = 0.0f; // sum_{j>q} w_j a_j

        for (int j = rays.S - 1; j >= 0; --j) {
            const float t = q.near + ((float)j + 0.5f) * q.delta;
            const Cell c = sample_cell(g, q, j);
            gather_feat(g, q.scene, c, acts, lane);
            mlp_forward(m, sW, acts, lane);
            const float z0 = acts[(out_off + 0) * block_lanes() + lane];
            const float sigma = softplus_f(z0);
            const float sd = sigma * q.delta;
            const float Tq = expf(-tau);          // T_q
            const float tau_prev = tau - sd;
            const float Tprev = expf(-tau_prev);  // T_{q-1}
            const float w = Tprev - Tq;
            float a = p_depth * t;
            for (int ch = 0; ch < F; ++ch)
                a += pcol[ch * block_lanes() + lane] * feature_act(m, acts[(out_off + 1 + ch) * block_lanes() + lane]);
            const float dsigma = q.delta * (Tq * a - suffix + kS);
            suffix += w * a;
            tau = tau_prev;

            // heads
            float* dz = dz0;
            float* dz_next = dz1;
            dz[0 * block_lanes() + lane] = live ? dsigma * logistic_f(z0) : 0.0f;
            for (int ch = 0; ch < F; ++ch) {
                const float f = feature_act(m, acts[(out_off + 1 + ch) * block_lanes() + lane]);
                const float df = m.feat_act == 0 ? f * (1.0f - f) : 1.0f;
                dz[(1 + ch) * block_lanes() + lane] = live ? w * pcol[ch * block_lanes() + lane] * df : 0.0f;
            }

            dz = mlp_backward(m, sW, sdW, acts, dz, dz_next, lane);
            // (the MLP backward alternates between dz0 and dz1; the one it did not return is free now)
            float* cells = m.max_width >= kGenericCellColumns ? (dz == dz0 ? dz1 : dz0) : cells_extra;
            publish_cell(cells, lane, c, q.scene, live);
            __syncthreads();
            scatter_tile(g, io.d_grid, io.d_grid_t, cells, dz, lane);
            __syncthreads();   // the next sample overwrites cells and dz
        }
    }
    __syncthreads();
    // this block's partial sums; a second kernel adds all records into dW / db
    if (!io.acc_in_record)
        for (int i = threadIdx.x; i < m.param_total; i += blockDim.x) rec[i] = sdW[i];
}

// dW[l] += sum over records, db[l] likewise.  A block of 1024 threads handles 64 consecutive
// parameters: thread (p, q) sums records q, q + 16, q + 32, ... of parameter p in fp64, then the
// 16 partial sums of a parameter are added in a fixed order (deterministic).
__global__ __launch_bounds__(kReduceThreads) void reduce_params_kernel(MlpDev m, BwdIo io, int n_records)
{
    __shared__ double part[kReduceThreads];
    const int p = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + p;
    double s = 0.0;
    if (i < m.param_total)
        for (int r = q; r < n_records; r += kReduceThreads / 64) s += (double)io.ws[(size_t)r * io.ws_stride + i];
    part[threadIdx.x] = s;
    __syncthreads();
    if (q != 0 || i >= m.param_total) return;
    for (int k = 1; k < kReduceThreads / 64; ++k) s += part[k * 64 + p];
    for (int l = 0; l < m.n_layers; ++l) {
        const int nw = m.dims[l] * m.dims[l + 1];
        if (i >= m.w_off[l] && i < m.w_off[l] + nw) {
            io.dW[l][i - m.w_off[l]] += (float)s;
            return;
        }
        if (i >= m.b_off[l] && i < m.b_off[l] + m.dims[l + 1]) {
            io.db[l][i - m.b_off[l]] += (float)s;
            return;
        }
    }
}

}  // namespace lp
