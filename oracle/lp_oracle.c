/*
 * lp_oracle.c — CPU oracle for the Lightplane Renderer.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the Renderer computes: the "naive"
 * renderer the paper contrasts itself with (Section 3.1), which materialises every
 * per-sample quantity of a ray, composites with the emission-absorption sum of
 * Eq. (1) (Section 3.3), and differentiates that stored computation by ordinary
 * reverse-mode, operation by operation.  The paper's Renderer is exact (it changes
 * what is stored, not what is computed), so this definition is its oracle.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this
 * file.  It shares no code with the HIP library and includes none of its headers.
 *
 * Conventions fixed where the paper is silent (each is one reading, listed in the
 * design notes of the repository):
 *   - T_0 = 1 and T_j = T_{j-1} exp(-sigma_j Delta); Eq. (1)'s inner sum is read as
 *     running over n = 1..j.
 *   - S samples at the midpoints of S equal bins of [near, far]; Delta = (far-near)/S.
 *   - world -> grid: index 0 is at aabb_min, index N-1 at aabb_max; positions outside
 *     the box are clamped to it (border).
 *   - axis x <-> first spatial dim, y <-> second, z <-> third; channels innermost
 *     (Section 3.2: voxel HxWxDxK; planes at (x,y), (y,z), (z,x), summed).
 *   - one MLP C -> ... -> 4: ReLU hidden layers, linear last layer; output 0 through
 *     softplus is the density, outputs 1..3 through the logistic sigmoid are the colour.
 *   - depth = sum_j w_j t_j (a rendered feature like any other); rgb gets + T_S * bg.
 *   - contract coordinates (appendix, "Experimental Details", the equation CC(x)): when the
 *     scale a is positive, every axis of a sample position goes through CC on its own (the
 *     text says the axes are converted independently, so ||x|| and x/||x|| are |x| and
 *     sign(x)) before the box mapping; sample spacing Delta stays the world distance.
 *   - further structures h that Section 3.2 names without defining them: a hash table (one level
 *     of the spatial hash of Teschner et al. 2003 with Instant-NGP's primes, trilinear over a
 *     virtual lattice) and a HexPlane (Cao & Johnson 2023: three pairs of a spatial and a
 *     space-time plane, the reads of a pair multiplied, the three products added; one time per
 *     ray).  Both are pinned like the other structures (tests/test_oracle_hash.py,
 *     tests/test_oracle_hexplane.py); no function of this file is parity-unpinned.
 *
 * All arithmetic is double.  Parallel over rays only (OpenMP); grid gradients are
 * added with atomic updates, weight gradients in per-thread buffers summed at the end.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LPO_VOXEL 0
#define LPO_TRIPLANE 1
#define LPO_HASH 2
#define LPO_HEXPLANE 3
#define LPO_MAX_LAYERS 8

typedef struct {
    int32_t kind, B, C, NX, NY, NZ;
    const double* data[3];
    double aabb_min[3], aabb_max[3];
    double contract_a; /* 0: no contraction; else the foreground scale a of CC */
    int64_t hash_size; /* LPO_HASH: entries T of the table of one scene, data[0] = [B][T][C] */
    /* LPO_HEXPLANE: data[p] as the triplane's planes; data_t[p] = [B][N_c][NT][C] is the space-time
       plane over (c, t), c the spatial axis that plane p leaves out (z, x, y for p = 0, 1, 2); time
       t_min maps to index 0 and t_max to index NT - 1 */
    const double* data_t[3];
    int32_t NT;
    double t_min, t_max;
} lpo_grid;

typedef struct {
    int32_t n_layers;
    int32_t dims[LPO_MAX_LAYERS + 1];
    const double* W[LPO_MAX_LAYERS]; /* [dims[l+1]][dims[l]] */
    const double* b[LPO_MAX_LAYERS]; /* [dims[l+1]] */
} lpo_mlp;

typedef struct {
    int64_t M;
    int32_t S;
    const double* origins; /* [M][3] */
    const double* dirs;    /* [M][3] unit */
    const double* near;    /* [M] */
    const double* far;     /* [M] */
    const int32_t* scene;  /* [M] or NULL */
    const double* time;    /* [M] or NULL (every ray at the grid's t_min); read by LPO_HEXPLANE only */
} lpo_rays;

static double ray_time(const lpo_grid* g, const lpo_rays* rays, int64_t i)
{
    return rays->time ? rays->time[i] : g->t_min;
}

/* ---- Section 3.2: the hashing scheme h (bi/tri-linear interpolation) ---------- */

/* CC of one coordinate: 0.5 a x inside the unit interval; outside, magnitude
 * 0.5 ((2 - a)(1 - 1/|x|) + a) with the sign of x.  Maps the real line into (-1, 1). */
static double contract_axis(double x, double a)
{
    double m = fabs(x);
    if (m <= 1.0) return 0.5 * a * x;
    double r = 0.5 * ((2.0 - a) * (1.0 - 1.0 / m) + a);
    return x < 0.0 ? -r : r;
}

/* position the hash structure is read at: the sample position, contracted if asked for */
static void grid_position(const lpo_grid* g, const double x[3], double y[3])
{
    for (int a = 0; a < 3; ++a) y[a] = g->contract_a > 0.0 ? contract_axis(x[a], g->contract_a) : x[a];
}

/* continuous index along one axis -> cell index i in [0, N-2] and fraction f in [0,1] */
static void axis_cell(double x, double lo, double hi, int N, int* i, double* f)
{
    double u = (x - lo) / (hi - lo) * (double)(N - 1);
    if (u < 0.0) u = 0.0;
    if (u > (double)(N - 1)) u = (double)(N - 1);
    int c = (int)floor(u);
    if (c > N - 2) c = N - 2;
    *i = c;
    *f = u - (double)c;
}

/* bilinear read of a [NA][NB][C] plane at cell (ia, ib), fractions (fa, fb); adds into feat */
static void plane_gather(const double* P, int NB, int C, int ia, int ib, double fa, double fb,
                         double* feat)
{
    for (int da = 0; da < 2; ++da)
        for (int db = 0; db < 2; ++db) {
            double w = (da ? fa : 1.0 - fa) * (db ? fb : 1.0 - fb);
            const double* v = P + ((int64_t)(ia + da) * NB + (ib + db)) * C;
            for (int k = 0; k < C; ++k) feat[k] += w * v[k];
        }
}

static void plane_scatter(double* P, int NB, int C, int ia, int ib, double fa, double fb,
                          const double* dfeat)
{
    for (int da = 0; da < 2; ++da)
        for (int db = 0; db < 2; ++db) {
            double w = (da ? fa : 1.0 - fa) * (db ? fb : 1.0 - fb);
            double* v = P + ((int64_t)(ia + da) * NB + (ib + db)) * C;
            for (int k = 0; k < C; ++k) {
                double add = w * dfeat[k];
#pragma omp atomic
                v[k] += add;
            }
        }
}

/* Hash-table structure (Section 3.2 names hash tables among the structures h; the paper gives no
   definition, this is the single-resolution spatial hash of Teschner et al. 2003 as Instant-NGP
   uses it): lattice corner (ix, iy, iz) of the virtual NX x NY x NZ grid lives in entry
   ((ix * 1) xor (iy * 2654435761) xor (iz * 805459861)) mod T, products and xor in 32-bit unsigned
   arithmetic; corners that collide share the entry. */
int64_t lpo_hash_slot(int32_t ix, int32_t iy, int32_t iz, int64_t T)
{
    const uint32_t h = ((uint32_t)ix * 1u) ^ ((uint32_t)iy * 2654435761u) ^ ((uint32_t)iz * 805459861u);
    return (int64_t)((uint64_t)h % (uint64_t)T);
}

/* HexPlane (Section 3.2 names it among the structures h; the definition is Cao & Johnson 2023's):
   six planes in three complementary pairs, (x,y) with (z,t), (y,z) with (x,t), (z,x) with (y,t).
   Both planes of a pair are read bilinearly, the two feature vectors are multiplied channel by
   channel, and the three products are added (the fusion that keeps C channels, as the triplane's sum
   does).  s[p], u[p]: the reads of the spatial and of the space-time plane of pair p. */
static void hexplane_reads(const lpo_grid* g, int b, const int i[3], const double f[3], double t,
                           double* s /* [3][C] */, double* u /* [3][C] */, int* it, double* ft)
{
    const int N[3] = {g->NX, g->NY, g->NZ};
    const int C = g->C;
    axis_cell(t, g->t_min, g->t_max, g->NT, it, ft);
    for (int k = 0; k < 3 * C; ++k) s[k] = u[k] = 0.0;
    for (int p = 0; p < 3; ++p) {
        const int a = p, bb = (p + 1) % 3, c = (p + 2) % 3;
        plane_gather(g->data[p] + (int64_t)b * N[a] * N[bb] * C, N[bb], C, i[a], i[bb], f[a], f[bb], s + p * C);
        plane_gather(g->data_t[p] + (int64_t)b * N[c] * g->NT * C, g->NT, C, i[c], *it, f[c], *ft, u + p * C);
    }
}

/* h(x): feature of world point x (at time t, which only a HexPlane reads) in scene b */
static void grid_gather(const lpo_grid* g, int b, const double x[3], double t, double* feat)
{
    int i[3];
    double f[3], y[3];
    const int N[3] = {g->NX, g->NY, g->NZ};
    grid_position(g, x, y);
    for (int a = 0; a < 3; ++a) axis_cell(y[a], g->aabb_min[a], g->aabb_max[a], N[a], &i[a], &f[a]);
    const int C = g->C;
    for (int k = 0; k < C; ++k) feat[k] = 0.0;
    if (g->kind == LPO_VOXEL) {
        const double* V = g->data[0] + (int64_t)b * g->NX * g->NY * g->NZ * C;
        for (int dx = 0; dx < 2; ++dx)
            for (int dy = 0; dy < 2; ++dy)
                for (int dz = 0; dz < 2; ++dz) {
                    double w = (dx ? f[0] : 1.0 - f[0]) * (dy ? f[1] : 1.0 - f[1]) *
                               (dz ? f[2] : 1.0 - f[2]);
                    const double* v =
                        V + (((int64_t)(i[0] + dx) * g->NY + (i[1] + dy)) * g->NZ + (i[2] + dz)) * C;
                    for (int k = 0; k < C; ++k) feat[k] += w * v[k];
                }
    } else if (g->kind == LPO_HASH) {
        /* trilinear over the 8 lattice corners of the cell, each read from its table entry */
        const double* V = g->data[0] + (int64_t)b * g->hash_size * C;
        for (int dx = 0; dx < 2; ++dx)
            for (int dy = 0; dy < 2; ++dy)
                for (int dz = 0; dz < 2; ++dz) {
                    double w = (dx ? f[0] : 1.0 - f[0]) * (dy ? f[1] : 1.0 - f[1]) *
                               (dz ? f[2] : 1.0 - f[2]);
                    const double* v = V + lpo_hash_slot(i[0] + dx, i[1] + dy, i[2] + dz, g->hash_size) * C;
                    for (int k = 0; k < C; ++k) feat[k] += w * v[k];
                }
    } else if (g->kind == LPO_HEXPLANE) {
        int it;
        double ft;
        double* s = (double*)malloc(sizeof(double) * 6 * (size_t)C);
        double* u = s + 3 * C;
        hexplane_reads(g, b, i, f, t, s, u, &it, &ft);
        for (int p = 0; p < 3; ++p)
            for (int k = 0; k < C; ++k) feat[k] += s[p * C + k] * u[p * C + k];
        free(s);
    } else {
        /* planes sampled at (x,y), (y,z), (z,x) and summed */
        plane_gather(g->data[0] + (int64_t)b * g->NX * g->NY * C, g->NY, C, i[0], i[1], f[0], f[1], feat);
        plane_gather(g->data[1] + (int64_t)b * g->NY * g->NZ * C, g->NZ, C, i[1], i[2], f[1], f[2], feat);
        plane_gather(g->data[2] + (int64_t)b * g->NZ * g->NX * C, g->NX, C, i[2], i[0], f[2], f[0], feat);
    }
}

/* transpose of grid_gather: d_grid[corner] += weight * dfeat, same corners and weights */
/* (a HexPlane has six gradient tensors: d_grid[p] for data[p], d_grid[3 + p] for data_t[p]).
   dfeat_neg: NULL, or -- when dfeat is one side of the kink envelope of the feature gradient -- the
   other side, which a HexPlane uses wherever the feature gradient is multiplied by a NEGATIVE plane
   read (the upper bound of a product with a negative factor comes from the lower bound). */
static void grid_scatter(const lpo_grid* g, double* const d_grid[], int b, const double x[3], double t,
                         const double* dfeat, const double* dfeat_neg)
{
    int i[3];
    double f[3], y[3];
    const int N[3] = {g->NX, g->NY, g->NZ};
    grid_position(g, x, y);
    for (int a = 0; a < 3; ++a) axis_cell(y[a], g->aabb_min[a], g->aabb_max[a], N[a], &i[a], &f[a]);
    const int C = g->C;
    if (g->kind == LPO_VOXEL) {
        double* V = d_grid[0] + (int64_t)b * g->NX * g->NY * g->NZ * C;
        for (int dx = 0; dx < 2; ++dx)
            for (int dy = 0; dy < 2; ++dy)
                for (int dz = 0; dz < 2; ++dz) {
                    double w = (dx ? f[0] : 1.0 - f[0]) * (dy ? f[1] : 1.0 - f[1]) *
                               (dz ? f[2] : 1.0 - f[2]);
                    double* v =
                        V + (((int64_t)(i[0] + dx) * g->NY + (i[1] + dy)) * g->NZ + (i[2] + dz)) * C;
                    for (int k = 0; k < C; ++k) {
                        double add = w * dfeat[k];
#pragma omp atomic
                        v[k] += add;
                    }
                }
    } else if (g->kind == LPO_HASH) {
        double* V = d_grid[0] + (int64_t)b * g->hash_size * C;
        for (int dx = 0; dx < 2; ++dx)
            for (int dy = 0; dy < 2; ++dy)
                for (int dz = 0; dz < 2; ++dz) {
                    double w = (dx ? f[0] : 1.0 - f[0]) * (dy ? f[1] : 1.0 - f[1]) *
                               (dz ? f[2] : 1.0 - f[2]);
                    double* v = V + lpo_hash_slot(i[0] + dx, i[1] + dy, i[2] + dz, g->hash_size) * C;
                    for (int k = 0; k < C; ++k) {
                        double add = w * dfeat[k];
#pragma omp atomic
                        v[k] += add;
                    }
                }
    } else if (g->kind == LPO_HEXPLANE) {
        /* product rule: the spatial plane of a pair receives dfeat times the space-time plane's read,
           and the other way round */
        int it;
        double ft;
        double* s = (double*)malloc(sizeof(double) * 7 * (size_t)C);
        double* u = s + 3 * C;
        double* tmp = s + 6 * C;
        hexplane_reads(g, b, i, f, t, s, u, &it, &ft);
        for (int p = 0; p < 3; ++p) {
            const int a = p, bb = (p + 1) % 3, c = (p + 2) % 3;
            for (int k = 0; k < C; ++k) tmp[k] = ((u[p * C + k] < 0.0 && dfeat_neg) ? dfeat_neg[k] : dfeat[k]) * u[p * C + k];
            plane_scatter(d_grid[p] + (int64_t)b * N[a] * N[bb] * C, N[bb], C, i[a], i[bb], f[a], f[bb], tmp);
            for (int k = 0; k < C; ++k) tmp[k] = ((s[p * C + k] < 0.0 && dfeat_neg) ? dfeat_neg[k] : dfeat[k]) * s[p * C + k];
            plane_scatter(d_grid[3 + p] + (int64_t)b * N[c] * g->NT * C, g->NT, C, i[c], it, f[c], ft, tmp);
        }
        free(s);
    } else {
        plane_scatter(d_grid[0] + (int64_t)b * g->NX * g->NY * C, g->NY, C, i[0], i[1], f[0], f[1], dfeat);
        plane_scatter(d_grid[1] + (int64_t)b * g->NY * g->NZ * C, g->NZ, C, i[1], i[2], f[1], f[2], dfeat);
        plane_scatter(d_grid[2] + (int64_t)b * g->NZ * g->NX * C, g->NX, C, i[2], i[0], f[2], f[0], dfeat);
    }
}

/* ---- Section 3.2: the tiny MLP g ------------------------------------------------ */

static int mlp_act_total(const lpo_mlp* m)
{
    int n = 0;
    for (int l = 0; l <= m->n_layers; ++l) n += m->dims[l];
    return n;
}

/* act holds the input (dims[0]) followed by every layer's post-activation output;
   pre holds every layer's pre-activation (offset as act minus dims[0]). */
static void mlp_forward(const lpo_mlp* m, double* act, double* pre)
{
    int off_in = 0, off_out = m->dims[0];
    for (int l = 0; l < m->n_layers; ++l) {
        const int nin = m->dims[l], nout = m->dims[l + 1];
        const double* W = m->W[l];
        const double* bb = m->b[l];
        for (int o = 0; o < nout; ++o) {
            double z = bb[o];
            for (int k = 0; k < nin; ++k) z += W[(int64_t)o * nin + k] * act[off_in + k];
            pre[off_out - m->dims[0] + o] = z;
            act[off_out + o] = (l + 1 < m->n_layers) ? (z > 0.0 ? z : 0.0) : z;
        }
        off_in = off_out;
        off_out += nout;
    }
}

static double softplus(double z) { return (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z))); }
static double logistic(double z) { return 1.0 / (1.0 + exp(-z)); }

/* ---- per-ray record of the stored forward computation ------------------------- */

typedef struct {
    int S, nact, C;
    double delta;
    double* t;     /* [S]   distance of sample j along the ray            */
    double* x;     /* [S][3] world position                               */
    double* act;   /* [S][nact] feature + every layer's output            */
    double* pre;   /* [S][nact - C] pre-activations                       */
    double* sigma; /* [S]                                                  */
    double* col;   /* [S][3]                                               */
    double* e;     /* [S]   exp(-sigma_j Delta)                           */
    double* T;     /* [S+1] T[0] = 1                                       */
    double* w;     /* [S]   T[j-1] - T[j]                                  */
} ray_tape;

static int tape_alloc(ray_tape* r, int S, int nact, int C)
{
    memset(r, 0, sizeof(*r));
    r->S = S; r->nact = nact; r->C = C;
    r->t = (double*)malloc(sizeof(double) * S);
    r->x = (double*)malloc(sizeof(double) * S * 3);
    r->act = (double*)malloc(sizeof(double) * (size_t)S * nact);
    r->pre = (double*)malloc(sizeof(double) * (size_t)S * (nact - C));
    r->sigma = (double*)malloc(sizeof(double) * S);
    r->col = (double*)malloc(sizeof(double) * S * 3);
    r->e = (double*)malloc(sizeof(double) * S);
    r->T = (double*)malloc(sizeof(double) * (S + 1));
    r->w = (double*)malloc(sizeof(double) * S);
    return r->t && r->x && r->act && r->pre && r->sigma && r->col && r->e && r->T && r->w;
}

static void tape_free(ray_tape* r)
{
    free(r->t); free(r->x); free(r->act); free(r->pre); free(r->sigma);
    free(r->col); free(r->e); free(r->T); free(r->w);
}

/* Forward of one ray, everything stored (Section 3.1's naive renderer; Eq. (1)). */
static void ray_forward(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays, int64_t i,
                        const double bg[3], ray_tape* r, double rgb[3], double* alpha, double* depth)
{
    const int S = r->S, nact = r->nact, C = r->C;
    const double* o = rays->origins + 3 * i;
    const double* d = rays->dirs + 3 * i;
    const double nr = rays->near[i], fr = rays->far[i];
    const int b = rays->scene ? rays->scene[i] : 0;
    const int nl = m->n_layers;
    const int out_off = nact - m->dims[nl]; /* offset of the last layer's output in act */
    r->delta = (fr - nr) / (double)S;
    r->T[0] = 1.0;
    rgb[0] = rgb[1] = rgb[2] = 0.0;
    *depth = 0.0;
    for (int j = 0; j < S; ++j) {
        const double t = nr + ((double)j + 0.5) * r->delta;
        r->t[j] = t;
        for (int a = 0; a < 3; ++a) r->x[3 * j + a] = o[a] + t * d[a];
        double* act = r->act + (size_t)j * nact;
        grid_gather(g, b, r->x + 3 * j, ray_time(g, rays, i), act);
        mlp_forward(m, act, r->pre + (size_t)j * (nact - C));
        const double* out = act + out_off;
        r->sigma[j] = softplus(out[0]);
        for (int c = 0; c < 3; ++c) r->col[3 * j + c] = logistic(out[1 + c]);
        r->e[j] = exp(-r->sigma[j] * r->delta);
        r->T[j + 1] = r->T[j] * r->e[j];
        r->w[j] = r->T[j] - r->T[j + 1];
        for (int c = 0; c < 3; ++c) rgb[c] += r->w[j] * r->col[3 * j + c];
        *depth += r->w[j] * t;
    }
    for (int c = 0; c < 3; ++c) rgb[c] += r->T[S] * bg[c];
    *alpha = 1.0 - r->T[S];
}

static int check_args(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays)
{
    if (!g || !m || !rays) return 1;
    if (g->B < 1 || g->C < 1 || g->NX < 2 || g->NY < 2 || g->NZ < 2) return 1;
    if (g->kind == LPO_HEXPLANE && (g->NT < 2 || !(g->t_max > g->t_min))) return 1;
    if (m->n_layers < 1 || m->n_layers > LPO_MAX_LAYERS) return 1;
    if (m->dims[0] != g->C || m->dims[m->n_layers] != 4) return 1;
    if (rays->M < 0 || rays->S < 1) return 1;
    return 0;
}

int lpo_render_fwd(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays, const double bg[3],
                   double* rgb, double* alpha, double* depth)
{
    if (check_args(g, m, rays)) return 1;
    const int nact = mlp_act_total(m);
    int fail = 0;
#pragma omp parallel
    {
        ray_tape r;
        if (!tape_alloc(&r, rays->S, nact, g->C)) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i)
                ray_forward(g, m, rays, i, bg, &r, rgb + 3 * i, alpha + i, depth + i);
        }
        tape_free(&r);
    }
    return fail ? 2 : 0;
}

/* Rounding-error scale of a hidden unit's pre-activation: |b| + sum_k |W_k x_k|. */
static double unit_scale(const lpo_mlp* m, int l, int o, const double* in)
{
    const int nin = m->dims[l];
    double mag = fabs(m->b[l][o]);
    for (int k = 0; k < nin; ++k) mag += fabs(m->W[l][(int64_t)o * nin + k] * in[k]);
    return mag;
}

#define LPO_MAX_KINKS 6

/* Hidden units of this sample whose pre-activation lies within band * scale of the ReLU kink:
   writes up to LPO_MAX_KINKS (layer, unit) pairs, returns how many. */
static int sample_kinks(const lpo_mlp* m, const double* act, const double* pre, int C, double band,
                        int* kl, int* ko)
{
    int n = 0, off_in = 0, off_out = m->dims[0];
    for (int l = 0; l + 1 < m->n_layers; ++l) {
        for (int o = 0; o < m->dims[l + 1]; ++o)
            if (fabs(pre[off_out - C + o]) < band * unit_scale(m, l, o, act + off_in) && n < LPO_MAX_KINKS) {
                kl[n] = l;
                ko[n] = o;
                ++n;
            }
        off_in = off_out;
        off_out += m->dims[l + 1];
    }
    return n;
}

/* Reverse-mode through the MLP of one sample.  dact holds dL/d(output) in its last 4
   entries on entry and dL/d(feature) in its first C entries on exit; dW, db are added to.
   ReLU' = 1 iff pre-activation > 0, except for the n_over listed units (kl, ko), whose
   derivative is bit i of `mask`. */
static void sample_mlp_backward(const lpo_mlp* m, const double* act, const double* pre, int C,
                                int nact, double* dact, double* const dW[], double* const db[],
                                int n_over, const int* kl, const int* ko, unsigned mask)
{
    const int nl = m->n_layers;
    for (int k = 0; k < nact - 4; ++k) dact[k] = 0.0;
    int off_out = nact - 4;
    for (int l = nl - 1; l >= 0; --l) {
        const int nin = m->dims[l], nout = m->dims[l + 1];
        const int off_in = off_out - nin;
        const double* W = m->W[l];
        for (int o = 0; o < nout; ++o) {
            double dz = dact[off_out + o];
            if (l + 1 < nl) {
                int on = pre[off_out - C + o] > 0.0;
                for (int i = 0; i < n_over; ++i)
                    if (kl[i] == l && ko[i] == o) on = (mask >> i) & 1u;
                if (!on) dz = 0.0;
            }
            if (dz == 0.0) continue;
            db[l][o] += dz;
            for (int k = 0; k < nin; ++k) {
                dW[l][(int64_t)o * nin + k] += dz * act[off_in + k];
                dact[off_in + k] += dz * W[(int64_t)o * nin + k];
            }
        }
        off_out = off_in;
    }
}

/* Scratch of the kink envelope: [0] running minimum, [1] running maximum, [2] current choice. */
typedef struct {
    double* W[3][LPO_MAX_LAYERS];
    double* b[3][LPO_MAX_LAYERS];
    double* dact[3];
} kink_tmp;

/* Reverse-mode over one ray's stored forward.  The forward operations, in order:
     e_j = exp(-sigma_j Delta); T_j = T_{j-1} e_j; w_j = T_{j-1} - T_j;
     rgb = sum_j w_j c_j + T_S bg; alpha = 1 - T_S; depth = sum_j w_j t_j.
   Each is reversed individually; nothing is simplified algebraically.
   dsig_out (optional) receives dL/dsigma_j, dcol_out (optional) dL/dc_j.
   side = 0: the definition.  side = +1 / -1 (with band > 0 and kt != NULL): for every sample
   with hidden pre-activations inside the kink band, the sample's contribution is the
   elementwise maximum / minimum over all on/off choices for those units. */
static void ray_backward(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays, int64_t i,
                         const double bg[3], const ray_tape* r, const double p_rgb[3],
                         double p_alpha, double p_depth, double* const d_grid[],
                         double* const dW[], double* const db[], double* scratch,
                         double* dsig_out, double* dcol_out, double band, int side, kink_tmp* kt)
{
    const int S = r->S, nact = r->nact, C = r->C, nl = m->n_layers;
    const int b = rays->scene ? rays->scene[i] : 0;
    double* dT = scratch;            /* [S+1] */
    double* dact = scratch + (S + 1); /* [nact] */
    for (int j = 0; j <= S; ++j) dT[j] = 0.0;
    /* alpha = 1 - T_S ; rgb += T_S bg */
    dT[S] += -p_alpha;
    for (int c = 0; c < 3; ++c) dT[S] += p_rgb[c] * bg[c];
    /* w_j = T_{j-1} - T_j enters rgb and depth */
    for (int j = 0; j < S; ++j) {
        double dw = p_depth * r->t[j];
        for (int c = 0; c < 3; ++c) dw += p_rgb[c] * r->col[3 * j + c];
        dT[j] += dw;
        dT[j + 1] -= dw;
    }
    /* T_j = T_{j-1} e_j, reversed from the last sample to the first */
    for (int j = S - 1; j >= 0; --j) {
        const double de = dT[j + 1] * r->T[j];
        dT[j] += dT[j + 1] * r->e[j];
        const double dsigma = de * (-r->delta) * r->e[j];
        double dcol[3];
        for (int c = 0; c < 3; ++c) dcol[c] = r->w[j] * p_rgb[c];
        if (dsig_out) dsig_out[j] = dsigma;
        if (dcol_out)
            for (int c = 0; c < 3; ++c) dcol_out[3 * j + c] = dcol[c];
        /* heads: sigma = softplus(out0), c = logistic(out1..3) */
        const double* act = r->act + (size_t)j * nact;
        const double* pre = r->pre + (size_t)j * (nact - C);
        const int out_off = nact - 4;
        double dout[4];
        dout[0] = dsigma * logistic(act[out_off + 0]);
        for (int c = 0; c < 3; ++c) {
            const double cc = r->col[3 * j + c];
            dout[1 + c] = dcol[c] * cc * (1.0 - cc);
        }
        int kl[LPO_MAX_KINKS], ko[LPO_MAX_KINKS];
        const int nk = (side != 0 && kt) ? sample_kinks(m, act, pre, C, band, kl, ko) : 0;
        const double* dact_neg = NULL;
        if (nk > 0) {
            for (unsigned mask = 0; mask < (1u << nk); ++mask) {
                for (int l = 0; l < nl; ++l) {
                    memset(kt->W[2][l], 0, sizeof(double) * (size_t)m->dims[l] * m->dims[l + 1]);
                    memset(kt->b[2][l], 0, sizeof(double) * (size_t)m->dims[l + 1]);
                }
                for (int c = 0; c < 4; ++c) kt->dact[2][out_off + c] = dout[c];
                sample_mlp_backward(m, act, pre, C, nact, kt->dact[2], kt->W[2], kt->b[2], nk, kl, ko, mask);
                for (int l = 0; l < nl; ++l) {
                    const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
                    for (int64_t k = 0; k < n; ++k) {
                        const double v = kt->W[2][l][k];
                        kt->W[0][l][k] = mask ? fmin(kt->W[0][l][k], v) : v;
                        kt->W[1][l][k] = mask ? fmax(kt->W[1][l][k], v) : v;
                    }
                    for (int k = 0; k < m->dims[l + 1]; ++k) {
                        const double v = kt->b[2][l][k];
                        kt->b[0][l][k] = mask ? fmin(kt->b[0][l][k], v) : v;
                        kt->b[1][l][k] = mask ? fmax(kt->b[1][l][k], v) : v;
                    }
                }
                for (int k = 0; k < C; ++k) {
                    const double v = kt->dact[2][k];
                    kt->dact[0][k] = mask ? fmin(kt->dact[0][k], v) : v;
                    kt->dact[1][k] = mask ? fmax(kt->dact[1][k], v) : v;
                }
            }
            const int pick = side > 0 ? 1 : 0;
            for (int l = 0; l < nl; ++l) {
                const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
                for (int64_t k = 0; k < n; ++k) dW[l][k] += kt->W[pick][l][k];
                for (int k = 0; k < m->dims[l + 1]; ++k) db[l][k] += kt->b[pick][l][k];
            }
            /* interpolation weights are non-negative, so the envelope of weight * dfeat is the
               weight times the envelope of dfeat (a HexPlane also multiplies by signed plane reads
               and takes the other side there, see grid_scatter) */
            for (int k = 0; k < C; ++k) dact[k] = kt->dact[pick][k];
            dact_neg = kt->dact[1 - pick];
        } else {
            for (int c = 0; c < 4; ++c) dact[out_off + c] = dout[c];
            sample_mlp_backward(m, act, pre, C, nact, dact, dW, db, 0, NULL, NULL, 0u);
        }
        grid_scatter(g, d_grid, b, r->x + 3 * j, ray_time(g, rays, i), dact, dact_neg);
    }
}

static int kink_alloc(kink_tmp* kt, const lpo_mlp* m, int nact)
{
    int ok = 1;
    memset(kt, 0, sizeof(*kt));
    for (int v = 0; v < 3; ++v) {
        for (int l = 0; l < m->n_layers; ++l) {
            kt->W[v][l] = (double*)calloc((size_t)m->dims[l] * m->dims[l + 1], sizeof(double));
            kt->b[v][l] = (double*)calloc((size_t)m->dims[l + 1], sizeof(double));
            ok = ok && kt->W[v][l] && kt->b[v][l];
        }
        kt->dact[v] = (double*)calloc((size_t)nact, sizeof(double));
        ok = ok && kt->dact[v];
    }
    return ok;
}

static void kink_free(kink_tmp* kt)
{
    for (int v = 0; v < 3; ++v) {
        for (int l = 0; l < LPO_MAX_LAYERS; ++l) { free(kt->W[v][l]); free(kt->b[v][l]); }
        free(kt->dact[v]);
    }
}

/* d_grid, dW, db are ACCUMULATED into (the caller zeroes them).
   side = 0 is the definition (ReLU' = 1 iff z > 0; band is ignored).
   side = +1 / -1 returns the upper / lower ENVELOPE of the gradients over the choices a
   finite-precision evaluation may legitimately make where a hidden pre-activation z lies
   within band * (|b| + sum_k |W_k x_k|) of the kink (there either one-sided derivative is
   a correct answer): every on/off combination of a sample's banded units (at most
   LPO_MAX_KINKS of them) is evaluated; samples are independent, so per-sample envelopes
   add.  The forward is never affected. */
int lpo_render_bwd(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays, const double bg[3],
                   const double* p_rgb, const double* p_alpha, const double* p_depth,
                   double* const d_grid[], double* const dW[], double* const db[], double band,
                   int side)
{
    if (check_args(g, m, rays)) return 1;
    if (side != 0 && !(band > 0.0)) return 1;
    const int nact = mlp_act_total(m);
    const int nl = m->n_layers;
    int fail = 0;
#pragma omp parallel
    {
        ray_tape r;
        kink_tmp kt;
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(rays->S + 1 + nact));
        double* tW[LPO_MAX_LAYERS];
        double* tb[LPO_MAX_LAYERS];
        int ok = tape_alloc(&r, rays->S, nact, g->C) && scratch;
        ok = kink_alloc(&kt, m, nact) && ok;
        for (int l = 0; l < nl; ++l) {
            tW[l] = (double*)calloc((size_t)m->dims[l] * m->dims[l + 1], sizeof(double));
            tb[l] = (double*)calloc((size_t)m->dims[l + 1], sizeof(double));
            ok = ok && tW[l] && tb[l];
        }
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i) {
                double rgb[3], alpha, depth;
                ray_forward(g, m, rays, i, bg, &r, rgb, &alpha, &depth);
                ray_backward(g, m, rays, i, bg, &r, p_rgb + 3 * i, p_alpha ? p_alpha[i] : 0.0,
                             p_depth ? p_depth[i] : 0.0, d_grid, tW, tb, scratch, NULL, NULL, band,
                             side, &kt);
            }
#pragma omp critical
            {
                for (int l = 0; l < nl; ++l) {
                    const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
                    for (int64_t k = 0; k < n; ++k) dW[l][k] += tW[l][k];
                    for (int k = 0; k < m->dims[l + 1]; ++k) db[l][k] += tb[l][k];
                }
            }
        }
        for (int l = 0; l < nl; ++l) { free(tW[l]); free(tb[l]); }
        free(scratch);
        kink_free(&kt);
        tape_free(&r);
    }
    return fail ? 2 : 0;
}

/* Per-sample quantities of ONE ray, for the pins: t [S], x [S][3], feat [S][C], sigma [S],
   col [S][3], T [S+1], w [S]; and, when p_rgb is given, dL/dsigma [S] and dL/dcol [S][3]
   of that ray alone (gradient buffers are scratch and discarded).  Any output may be NULL. */
int lpo_ray_trace(const lpo_grid* g, const lpo_mlp* m, const lpo_rays* rays, const double bg[3],
                  int64_t ray, const double* p_rgb, double p_alpha, double p_depth,
                  double* t, double* x, double* feat, double* sigma, double* col, double* T,
                  double* w, double* dsigma, double* dcol)
{
    if (check_args(g, m, rays) || ray < 0 || ray >= rays->M) return 1;
    const int nact = mlp_act_total(m), S = rays->S, C = g->C, nl = m->n_layers;
    ray_tape r;
    if (!tape_alloc(&r, S, nact, C)) { tape_free(&r); return 2; }
    double rgb[3], alpha, depth;
    ray_forward(g, m, rays, ray, bg, &r, rgb, &alpha, &depth);
    if (t) memcpy(t, r.t, sizeof(double) * S);
    if (x) memcpy(x, r.x, sizeof(double) * S * 3);
    if (feat)
        for (int j = 0; j < S; ++j) memcpy(feat + (size_t)j * C, r.act + (size_t)j * nact, sizeof(double) * C);
    if (sigma) memcpy(sigma, r.sigma, sizeof(double) * S);
    if (col) memcpy(col, r.col, sizeof(double) * S * 3);
    if (T) memcpy(T, r.T, sizeof(double) * (S + 1));
    if (w) memcpy(w, r.w, sizeof(double) * S);
    int rc = 0;
    if (p_rgb && (dsigma || dcol)) {
        /* throw-away gradient buffers */
        int64_t gsz[6] = {0, 0, 0, 0, 0, 0};
        if (g->kind == LPO_VOXEL) gsz[0] = (int64_t)g->B * g->NX * g->NY * g->NZ * C;
        else if (g->kind == LPO_HASH) gsz[0] = (int64_t)g->B * g->hash_size * C;
        else {
            gsz[0] = (int64_t)g->B * g->NX * g->NY * C;
            gsz[1] = (int64_t)g->B * g->NY * g->NZ * C;
            gsz[2] = (int64_t)g->B * g->NZ * g->NX * C;
            if (g->kind == LPO_HEXPLANE) {
                gsz[3] = (int64_t)g->B * g->NZ * g->NT * C;
                gsz[4] = (int64_t)g->B * g->NX * g->NT * C;
                gsz[5] = (int64_t)g->B * g->NY * g->NT * C;
            }
        }
        double* dg[6] = {NULL, NULL, NULL, NULL, NULL, NULL};
        double* tW[LPO_MAX_LAYERS] = {NULL};
        double* tb[LPO_MAX_LAYERS] = {NULL};
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(S + 1 + nact));
        int ok = scratch != NULL;
        for (int p = 0; p < 6; ++p)
            if (gsz[p]) { dg[p] = (double*)calloc((size_t)gsz[p], sizeof(double)); ok = ok && dg[p]; }
        for (int l = 0; l < nl; ++l) {
            tW[l] = (double*)calloc((size_t)m->dims[l] * m->dims[l + 1], sizeof(double));
            tb[l] = (double*)calloc((size_t)m->dims[l + 1], sizeof(double));
            ok = ok && tW[l] && tb[l];
        }
        if (ok)
            ray_backward(g, m, rays, ray, bg, &r, p_rgb, p_alpha, p_depth, dg, tW, tb, scratch,
                         dsigma, dcol, 0.0, 0, NULL);
        else rc = 2;
        for (int p = 0; p < 6; ++p) free(dg[p]);
        for (int l = 0; l < nl; ++l) { free(tW[l]); free(tb[l]); }
        free(scratch);
    }
    tape_free(&r);
    return rc;
}

int lpo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ==== The Renderer with the paper's own decoder (Section 3.3, below Eq. (1)) =================
 *
 * Two MLPs read the feature sampled at a point: the opacity MLP g_sigma gives the density, and a
 * second MLP g_v, which also receives the view direction, gives the feature f_v that is rendered;
 * that feature is a vector of any width (colours and depths are the paper's examples).
 *
 *   sigma_j = softplus( g_sigma( h(x_j) )[0] )                 g_sigma : C -> ... -> 1
 *   f_j     = act( g_v( [ h(x_j) ; enc(d) ] ) )                g_v     : C + E -> ... -> F
 *   v       = sum_j w_j f_j + T_S bg            (F channels),  alpha, depth as before.
 *
 * Readings (the paper does not say): enc(d) is the view direction followed by n_freq octaves
 * of sin / cos, enc = (d, sin(2^0 pi d), cos(2^0 pi d), ..., sin(2^{L-1} pi d), cos(2^{L-1} pi d)),
 * each applied per component, E = 3 + 6 L (L = 0: the raw direction); act is the logistic
 * sigmoid (colours, as in the single-MLP decoder) or the identity (feat_act = 1); the same
 * sampled feature feeds both MLPs; no gradient with respect to the direction.
 */

typedef struct {
    lpo_mlp opacity;  /* g_sigma */
    lpo_mlp color;    /* g_v */
    int32_t n_freq;   /* L */
    int32_t n_feat;   /* F */
    int32_t feat_act; /* 0 logistic sigmoid, 1 identity */
} lpo_decoder;

static const double LPO_PI = 3.14159265358979323846264338327950288;

static void dir_encode(const double d[3], int L, double* enc)
{
    for (int a = 0; a < 3; ++a) enc[a] = d[a];
    double f = LPO_PI;
    for (int k = 0; k < L; ++k) {
        for (int a = 0; a < 3; ++a) {
            enc[3 + 6 * k + a] = sin(f * d[a]);
            enc[3 + 6 * k + 3 + a] = cos(f * d[a]);
        }
        f *= 2.0;
    }
}

typedef struct {
    int S, C, E, F, na_s, na_v; /* na_*: act_total of the two MLPs */
    double delta;
    double *t, *x;
    double *act_s, *pre_s; /* [S][na_s], [S][na_s - C]       */
    double *act_v, *pre_v; /* [S][na_v], [S][na_v - (C + E)] */
    double *sigma, *feat;  /* [S], [S][F] (after act)        */
    double *e, *T, *w;
} dec_tape;

static int dec_tape_alloc(dec_tape* r, int S, int C, int E, int F, int na_s, int na_v)
{
    memset(r, 0, sizeof(*r));
    r->S = S; r->C = C; r->E = E; r->F = F; r->na_s = na_s; r->na_v = na_v;
    r->t = (double*)malloc(sizeof(double) * S);
    r->x = (double*)malloc(sizeof(double) * S * 3);
    r->act_s = (double*)malloc(sizeof(double) * (size_t)S * na_s);
    r->pre_s = (double*)malloc(sizeof(double) * (size_t)S * na_s);
    r->act_v = (double*)malloc(sizeof(double) * (size_t)S * na_v);
    r->pre_v = (double*)malloc(sizeof(double) * (size_t)S * na_v);
    r->sigma = (double*)malloc(sizeof(double) * S);
    r->feat = (double*)malloc(sizeof(double) * (size_t)S * F);
    r->e = (double*)malloc(sizeof(double) * S);
    r->T = (double*)malloc(sizeof(double) * (S + 1));
    r->w = (double*)malloc(sizeof(double) * S);
    return r->t && r->x && r->act_s && r->pre_s && r->act_v && r->pre_v && r->sigma && r->feat &&
           r->e && r->T && r->w;
}

static void dec_tape_free(dec_tape* r)
{
    free(r->t); free(r->x); free(r->act_s); free(r->pre_s); free(r->act_v); free(r->pre_v);
    free(r->sigma); free(r->feat); free(r->e); free(r->T); free(r->w);
}

static int dec_check(const lpo_grid* g, const lpo_decoder* dc, const lpo_rays* rays)
{
    if (!g || !dc || !rays) return 1;
    if (g->B < 1 || g->C < 1 || g->NX < 2 || g->NY < 2 || g->NZ < 2) return 1;
    if (g->kind == LPO_HEXPLANE && (g->NT < 2 || !(g->t_max > g->t_min))) return 1;
    const lpo_mlp* ms = &dc->opacity;
    const lpo_mlp* mv = &dc->color;
    if (ms->n_layers < 1 || ms->n_layers > LPO_MAX_LAYERS) return 1;
    if (mv->n_layers < 1 || mv->n_layers > LPO_MAX_LAYERS) return 1;
    if (dc->n_freq < 0 || dc->n_feat < 1) return 1;
    if (ms->dims[0] != g->C || ms->dims[ms->n_layers] != 1) return 1;
    if (mv->dims[0] != g->C + 3 + 6 * dc->n_freq || mv->dims[mv->n_layers] != dc->n_feat) return 1;
    if (rays->M < 0 || rays->S < 1) return 1;
    return 0;
}

/* forward of one ray, everything stored */
static void dec_ray_forward(const lpo_grid* g, const lpo_decoder* dc, const lpo_rays* rays, int64_t i,
                            const double* bg, dec_tape* r, double* out, double* alpha, double* depth)
{
    const int S = r->S, C = r->C, E = r->E, F = r->F;
    const double* o = rays->origins + 3 * i;
    const double* d = rays->dirs + 3 * i;
    const double nr = rays->near[i], fr = rays->far[i];
    const int b = rays->scene ? rays->scene[i] : 0;
    const int out_s = r->na_s - 1, out_v = r->na_v - F;
    r->delta = (fr - nr) / (double)S;
    r->T[0] = 1.0;
    for (int k = 0; k < F; ++k) out[k] = 0.0;
    *depth = 0.0;
    for (int j = 0; j < S; ++j) {
        const double t = nr + ((double)j + 0.5) * r->delta;
        r->t[j] = t;
        for (int a = 0; a < 3; ++a) r->x[3 * j + a] = o[a] + t * d[a];
        double* as = r->act_s + (size_t)j * r->na_s;
        double* av = r->act_v + (size_t)j * r->na_v;
        grid_gather(g, b, r->x + 3 * j, ray_time(g, rays, i), as);
        for (int k = 0; k < C; ++k) av[k] = as[k];
        dir_encode(d, dc->n_freq, av + C);
        mlp_forward(&dc->opacity, as, r->pre_s + (size_t)j * r->na_s);
        mlp_forward(&dc->color, av, r->pre_v + (size_t)j * r->na_v);
        r->sigma[j] = softplus(as[out_s]);
        for (int k = 0; k < F; ++k)
            r->feat[(size_t)j * F + k] = dc->feat_act == 0 ? logistic(av[out_v + k]) : av[out_v + k];
        r->e[j] = exp(-r->sigma[j] * r->delta);
        r->T[j + 1] = r->T[j] * r->e[j];
        r->w[j] = r->T[j] - r->T[j + 1];
        for (int k = 0; k < F; ++k) out[k] += r->w[j] * r->feat[(size_t)j * F + k];
        *depth += r->w[j] * t;
    }
    for (int k = 0; k < F; ++k) out[k] += r->T[S] * bg[k];
    *alpha = 1.0 - r->T[S];
    (void)E;
}

int lpo_render2_fwd(const lpo_grid* g, const lpo_decoder* dc, const lpo_rays* rays, const double* bg,
                    double* out, double* alpha, double* depth)
{
    if (dec_check(g, dc, rays)) return 1;
    const int na_s = mlp_act_total(&dc->opacity), na_v = mlp_act_total(&dc->color);
    const int E = 3 + 6 * dc->n_freq, F = dc->n_feat;
    int fail = 0;
#pragma omp parallel
    {
        dec_tape r;
        if (!dec_tape_alloc(&r, rays->S, g->C, E, F, na_s, na_v)) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i)
                dec_ray_forward(g, dc, rays, i, bg, &r, out + (size_t)F * i, alpha + i, depth + i);
        }
        dec_tape_free(&r);
    }
    return fail ? 2 : 0;
}

/* Reverse-mode through one MLP of one sample, any number of outputs.  dact holds
   dL/d(output) in its last n_out entries on entry and dL/d(input) in its first dims[0]
   entries on exit; dW, db are added to.  pre is indexed like act minus dims[0].
   ReLU' = 1 iff pre-activation > 0, except for the listed units, whose derivative is bit i
   of `mask`. */
static void mlp_backward_sample(const lpo_mlp* m, const double* act, const double* pre, int nact,
                                double* dact, double* const dW[], double* const db[], int n_over,
                                const int* kl, const int* ko, unsigned mask)
{
    const int nl = m->n_layers, n_in = m->dims[0], n_out = m->dims[nl];
    for (int k = 0; k < nact - n_out; ++k) dact[k] = 0.0;
    int off_out = nact - n_out;
    for (int l = nl - 1; l >= 0; --l) {
        const int nin = m->dims[l], nout = m->dims[l + 1];
        const int off_in = off_out - nin;
        const double* W = m->W[l];
        for (int o = 0; o < nout; ++o) {
            double dz = dact[off_out + o];
            if (l + 1 < nl) {
                int on = pre[off_out - n_in + o] > 0.0;
                for (int i = 0; i < n_over; ++i)
                    if (kl[i] == l && ko[i] == o) on = (mask >> i) & 1u;
                if (!on) dz = 0.0;
            }
            if (dz == 0.0) continue;
            db[l][o] += dz;
            for (int k = 0; k < nin; ++k) {
                dW[l][(int64_t)o * nin + k] += dz * act[off_in + k];
                dact[off_in + k] += dz * W[(int64_t)o * nin + k];
            }
        }
        off_out = off_in;
    }
}

/* One MLP of one sample: the definition (side = 0) or the upper / lower envelope over the
   on/off choices of its hidden units inside the kink band (see lpo_render_bwd).  dout holds
   the n_out output gradients.  Adds to dW, db; writes dL/d(input) to din[0 .. dims[0]). */
static void mlp_backward_choice(const lpo_mlp* m, const double* act, const double* pre, int nact,
                                const double* dout, double band, int side, kink_tmp* kt,
                                double* const dW[], double* const db[], double* dact, double* din,
                                double* din_other /* the other side of the envelope of din (= din for side 0) */)
{
    const int nl = m->n_layers, n_in = m->dims[0], n_out = m->dims[nl];
    int kl[LPO_MAX_KINKS], ko[LPO_MAX_KINKS];
    const int nk = (side != 0 && kt) ? sample_kinks(m, act, pre, n_in, band, kl, ko) : 0;
    if (nk == 0) {
        for (int c = 0; c < n_out; ++c) dact[nact - n_out + c] = dout[c];
        mlp_backward_sample(m, act, pre, nact, dact, dW, db, 0, NULL, NULL, 0u);
        for (int k = 0; k < n_in; ++k) din[k] = din_other[k] = dact[k];
        return;
    }
    for (unsigned mask = 0; mask < (1u << nk); ++mask) {
        for (int l = 0; l < nl; ++l) {
            memset(kt->W[2][l], 0, sizeof(double) * (size_t)m->dims[l] * m->dims[l + 1]);
            memset(kt->b[2][l], 0, sizeof(double) * (size_t)m->dims[l + 1]);
        }
        for (int c = 0; c < n_out; ++c) kt->dact[2][nact - n_out + c] = dout[c];
        mlp_backward_sample(m, act, pre, nact, kt->dact[2], kt->W[2], kt->b[2], nk, kl, ko, mask);
        for (int l = 0; l < nl; ++l) {
            const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
            for (int64_t k = 0; k < n; ++k) {
                const double v = kt->W[2][l][k];
                kt->W[0][l][k] = mask ? fmin(kt->W[0][l][k], v) : v;
                kt->W[1][l][k] = mask ? fmax(kt->W[1][l][k], v) : v;
            }
            for (int k = 0; k < m->dims[l + 1]; ++k) {
                const double v = kt->b[2][l][k];
                kt->b[0][l][k] = mask ? fmin(kt->b[0][l][k], v) : v;
                kt->b[1][l][k] = mask ? fmax(kt->b[1][l][k], v) : v;
            }
        }
        for (int k = 0; k < n_in; ++k) {
            const double v = kt->dact[2][k];
            kt->dact[0][k] = mask ? fmin(kt->dact[0][k], v) : v;
            kt->dact[1][k] = mask ? fmax(kt->dact[1][k], v) : v;
        }
    }
    const int pick = side > 0 ? 1 : 0;
    for (int l = 0; l < nl; ++l) {
        const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
        for (int64_t k = 0; k < n; ++k) dW[l][k] += kt->W[pick][l][k];
        for (int k = 0; k < m->dims[l + 1]; ++k) db[l][k] += kt->b[pick][l][k];
    }
    for (int k = 0; k < n_in; ++k) { din[k] = kt->dact[pick][k]; din_other[k] = kt->dact[1 - pick][k]; }
}

/* Reverse of dec_ray_forward, operation by operation.  The two MLPs of a sample choose their
   kink units independently, and the sample's feature gradient is the sum of the two input
   gradients, so the envelope of the sum is the sum of the envelopes. */
static void dec_ray_backward(const lpo_grid* g, const lpo_decoder* dc, const lpo_rays* rays, int64_t i,
                             const double* bg, const dec_tape* r, const double* p_out, double p_alpha,
                             double p_depth, double* const d_grid[], double* const dWs[],
                             double* const dbs[], double* const dWv[], double* const dbv[],
                             double* scratch, double band, int side, kink_tmp* kts, kink_tmp* ktv)
{
    const int S = r->S, C = r->C, F = r->F;
    const int b = rays->scene ? rays->scene[i] : 0;
    double* dT = scratch;                    /* [S+1]  */
    double* dact_s = dT + (S + 1);           /* [na_s] */
    double* dact_v = dact_s + r->na_s;       /* [na_v] */
    double* din_s = dact_v + r->na_v;        /* [C]     */
    double* din_v = din_s + C;               /* [C + E] */
    double* dout_v = din_v + (C + r->E);     /* [F]     */
    double* oth_s = dout_v + F;              /* [C]     the other side of the envelope of din_s */
    double* oth_v = oth_s + C;               /* [C + E] ... of din_v */
    for (int j = 0; j <= S; ++j) dT[j] = 0.0;
    dT[S] += -p_alpha;
    for (int k = 0; k < F; ++k) dT[S] += p_out[k] * bg[k];
    for (int j = 0; j < S; ++j) {
        double dw = p_depth * r->t[j];
        for (int k = 0; k < F; ++k) dw += p_out[k] * r->feat[(size_t)j * F + k];
        dT[j] += dw;
        dT[j + 1] -= dw;
    }
    for (int j = S - 1; j >= 0; --j) {
        const double de = dT[j + 1] * r->T[j];
        dT[j] += dT[j + 1] * r->e[j];
        const double dsigma = de * (-r->delta) * r->e[j];
        const double* as = r->act_s + (size_t)j * r->na_s;
        const double* av = r->act_v + (size_t)j * r->na_v;
        const double dout_s = dsigma * logistic(as[r->na_s - 1]);
        for (int k = 0; k < F; ++k) {
            const double df = r->w[j] * p_out[k];
            const double f = r->feat[(size_t)j * F + k];
            dout_v[k] = dc->feat_act == 0 ? df * f * (1.0 - f) : df;
        }
        mlp_backward_choice(&dc->opacity, as, r->pre_s + (size_t)j * r->na_s, r->na_s, &dout_s, band, side,
                            kts, dWs, dbs, dact_s, din_s, oth_s);
        mlp_backward_choice(&dc->color, av, r->pre_v + (size_t)j * r->na_v, r->na_v, dout_v, band, side,
                            ktv, dWv, dbv, dact_v, din_v, oth_v);
        for (int k = 0; k < C; ++k) { din_s[k] += din_v[k]; oth_s[k] += oth_v[k]; }
        grid_scatter(g, d_grid, b, r->x + 3 * j, ray_time(g, rays, i), din_s, side != 0 ? oth_s : NULL);
    }
}

/* d_grid and the four gradient lists are ACCUMULATED into.  band / side as in lpo_render_bwd. */
int lpo_render2_bwd(const lpo_grid* g, const lpo_decoder* dc, const lpo_rays* rays, const double* bg,
                    const double* p_out, const double* p_alpha, const double* p_depth,
                    double* const d_grid[], double* const dWs[], double* const dbs[],
                    double* const dWv[], double* const dbv[], double band, int side)
{
    if (dec_check(g, dc, rays)) return 1;
    if (side != 0 && !(band > 0.0)) return 1;
    const lpo_mlp* ms = &dc->opacity;
    const lpo_mlp* mv = &dc->color;
    const int na_s = mlp_act_total(ms), na_v = mlp_act_total(mv);
    const int C = g->C, E = 3 + 6 * dc->n_freq, F = dc->n_feat;
    int fail = 0;
#pragma omp parallel
    {
        dec_tape r;
        kink_tmp kts, ktv;
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(rays->S + 1 + na_s + na_v + 4 * C + 2 * E + F));
        double* tWs[LPO_MAX_LAYERS] = {NULL};
        double* tbs[LPO_MAX_LAYERS] = {NULL};
        double* tWv[LPO_MAX_LAYERS] = {NULL};
        double* tbv[LPO_MAX_LAYERS] = {NULL};
        int ok = dec_tape_alloc(&r, rays->S, C, E, F, na_s, na_v) && scratch;
        ok = kink_alloc(&kts, ms, na_s) && ok;
        ok = kink_alloc(&ktv, mv, na_v) && ok;
        for (int l = 0; l < ms->n_layers; ++l) {
            tWs[l] = (double*)calloc((size_t)ms->dims[l] * ms->dims[l + 1], sizeof(double));
            tbs[l] = (double*)calloc((size_t)ms->dims[l + 1], sizeof(double));
            ok = ok && tWs[l] && tbs[l];
        }
        for (int l = 0; l < mv->n_layers; ++l) {
            tWv[l] = (double*)calloc((size_t)mv->dims[l] * mv->dims[l + 1], sizeof(double));
            tbv[l] = (double*)calloc((size_t)mv->dims[l + 1], sizeof(double));
            ok = ok && tWv[l] && tbv[l];
        }
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
            double* out = (double*)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i) {
                double alpha, depth;
                dec_ray_forward(g, dc, rays, i, bg, &r, out, &alpha, &depth);
                dec_ray_backward(g, dc, rays, i, bg, &r, p_out + (size_t)F * i, p_alpha ? p_alpha[i] : 0.0,
                                 p_depth ? p_depth[i] : 0.0, d_grid, tWs, tbs, tWv, tbv, scratch, band, side,
                                 &kts, &ktv);
            }
            free(out);
#pragma omp critical
            {
                for (int l = 0; l < ms->n_layers; ++l) {
                    const int64_t n = (int64_t)ms->dims[l] * ms->dims[l + 1];
                    for (int64_t k = 0; k < n; ++k) dWs[l][k] += tWs[l][k];
                    for (int k = 0; k < ms->dims[l + 1]; ++k) dbs[l][k] += tbs[l][k];
                }
                for (int l = 0; l < mv->n_layers; ++l) {
                    const int64_t n = (int64_t)mv->dims[l] * mv->dims[l + 1];
                    for (int64_t k = 0; k < n; ++k) dWv[l][k] += tWv[l][k];
                    for (int k = 0; k < mv->dims[l + 1]; ++k) dbv[l][k] += tbv[l][k];
                }
            }
        }
        for (int l = 0; l < LPO_MAX_LAYERS; ++l) { free(tWs[l]); free(tbs[l]); free(tWv[l]); free(tbv[l]); }
        free(scratch);
        kink_free(&kts);
        kink_free(&ktv);
        dec_tape_free(&r);
    }
    return fail ? 2 : 0;
}

/* enc(d) of one direction, for the pins: enc has 3 + 6 L entries */
int lpo_dir_encode(const double d[3], int n_freq, double* enc)
{
    if (!d || !enc || n_freq < 0) return 1;
    dir_encode(d, n_freq, enc);
    return 0;
}

/* ==== Splatter (Section 3.3, "Splatter"; appendix "Normalization Process in Splatter") ========
 *
 * The dual of the Renderer: M pixels with feature vectors v_i are expanded into rays of S
 * points (the same placement as the Renderer's samples); every point pushes a feature vector
 * into the hash cell that contains it, with the SAME bi/tri-linear weights the Renderer uses to
 * read that cell, and every cell is finally divided by the sum of the weights that landed on it:
 *     theta[corner]   += weight * vt_ij        theta_w[corner] += weight        (all i, j)
 *     out = theta / theta_w    (0 where nothing landed)
 * naive Splatter:  vt_ij = v_i.   With the MLP g_s (the paper's Eq. for the splatted feature):
 *     vt_ij = g_s( [ v_i ; h_prior(x_ij) ; enc(d_i) ] )
 * with h_prior the prior hash structure read by interpolation and enc the direction encoding
 * (n_freq = -1: no direction input; form as for the Renderer's decoder).  g_s: ReLU hidden
 * layers, linear output of the target's channel count.
 *
 * Backward, given G = dL/d(out): the weights depend on the ray geometry only, so
 * dL/dtheta = G / theta_w (the appendix: theta_w is kept to normalise the gradients), the
 * gradient of a splatted feature is that field READ at the point (the Renderer's forward
 * read), and from there ordinary reverse mode through g_s: dW, db, d(prior) (scattered like
 * the Renderer's grid gradient) and d(v_i) summed over the points of the ray.
 */

typedef struct {
    int32_t n_in;          /* channels of the pixel features */
    int32_t n_freq;        /* octaves of the direction encoding, -1: none */
    const double* feats;   /* [M][n_in] */
    const lpo_grid* prior; /* NULL: none */
    const lpo_mlp* mlp;    /* NULL: naive Splatter (n_in == target channels) */
} lpo_splat;

static int64_t grid_elems(const lpo_grid* g, int p)
{
    if (g->kind == LPO_VOXEL) return p == 0 ? (int64_t)g->B * g->NX * g->NY * g->NZ : 0;
    if (g->kind == LPO_HASH) return p == 0 ? (int64_t)g->B * g->hash_size : 0;
    const int64_t n[3] = {(int64_t)g->NX * g->NY, (int64_t)g->NY * g->NZ, (int64_t)g->NZ * g->NX};
    return (int64_t)g->B * n[p];
}

static int splat_check(const lpo_grid* tgt, const lpo_rays* rays, const lpo_splat* sp)
{
    if (!tgt || !rays || !sp || !sp->feats) return 1;
    if (tgt->B < 1 || tgt->C < 1 || tgt->NX < 2 || tgt->NY < 2 || tgt->NZ < 2) return 1;
    if (rays->M < 0 || rays->S < 1 || sp->n_in < 1 || sp->n_freq < -1) return 1;
    const int E = sp->n_freq < 0 ? 0 : 3 + 6 * sp->n_freq;
    const int Cp = sp->prior ? sp->prior->C : 0;
    if (tgt->kind == LPO_HEXPLANE) return 1; /* the Splatter writes voxel grids, triplanes and hash tables */
    if (tgt->kind == LPO_HASH && tgt->hash_size < 1) return 1;
    if (sp->prior && (sp->prior->kind != tgt->kind || sp->prior->B != tgt->B)) return 1;
    if (!sp->mlp) return (sp->n_in != tgt->C || sp->prior || E) ? 1 : 0;
    if (sp->mlp->n_layers < 1 || sp->mlp->n_layers > LPO_MAX_LAYERS) return 1;
    if (sp->mlp->dims[0] != sp->n_in + Cp + E || sp->mlp->dims[sp->mlp->n_layers] != tgt->C) return 1;
    return 0;
}

/* inputs of g_s for point x of ray i: [v_i ; h_prior(x) ; enc(d_i)] */
static void splat_inputs(const lpo_rays* rays, const lpo_splat* sp, int64_t i, int b, const double x[3],
                         double* in)
{
    int n = 0;
    for (int k = 0; k < sp->n_in; ++k) in[n++] = sp->feats[(size_t)i * sp->n_in + k];
    if (sp->prior) {
        grid_gather(sp->prior, b, x, 0.0, in + n);
        n += sp->prior->C;
    }
    if (sp->n_freq >= 0) dir_encode(rays->dirs + 3 * i, sp->n_freq, in + n);
}

/* theta [p] and theta_w [p] are written (normalised features, weight sums); shapes of the
   target grid with C and 1 channels. */
int lpo_splat_fwd(const lpo_grid* tgt, const lpo_rays* rays, const lpo_splat* sp, double* const theta[3],
                  double* const theta_w[3])
{
    if (splat_check(tgt, rays, sp)) return 1;
    const int C = tgt->C, S = rays->S, np = tgt->kind == LPO_TRIPLANE ? 3 : 1;
    lpo_grid wgrid = *tgt;
    wgrid.C = 1;
    for (int p = 0; p < np; ++p) {
        memset(theta[p], 0, sizeof(double) * (size_t)grid_elems(tgt, p) * C);
        memset(theta_w[p], 0, sizeof(double) * (size_t)grid_elems(tgt, p));
    }
    const int nact = sp->mlp ? mlp_act_total(sp->mlp) : 0;
    int fail = 0;
#pragma omp parallel
    {
        double* act = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        double* pre = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        if (!act || !pre) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i) {
                const double* o = rays->origins + 3 * i;
                const double* d = rays->dirs + 3 * i;
                const double nr = rays->near[i], delta = (rays->far[i] - nr) / (double)S;
                const int b = rays->scene ? rays->scene[i] : 0;
                const double one = 1.0;
                for (int j = 0; j < S; ++j) {
                    const double t = nr + ((double)j + 0.5) * delta;
                    const double x[3] = {o[0] + t * d[0], o[1] + t * d[1], o[2] + t * d[2]};
                    const double* vt = sp->feats + (size_t)i * sp->n_in;
                    if (sp->mlp) {
                        splat_inputs(rays, sp, i, b, x, act);
                        mlp_forward(sp->mlp, act, pre);
                        vt = act + nact - C;
                    }
                    grid_scatter(tgt, theta, b, x, 0.0, vt, NULL);
                    grid_scatter(&wgrid, theta_w, b, x, 0.0, &one, NULL);
                }
            }
        }
        free(act);
        free(pre);
    }
    if (fail) return 2;
    for (int p = 0; p < np; ++p) {
        const int64_t n = grid_elems(tgt, p);
        for (int64_t c = 0; c < n; ++c) {
            const double w = theta_w[p][c];
            for (int k = 0; k < C; ++k) theta[p][c * C + k] = w > 0.0 ? theta[p][c * C + k] / w : 0.0;
        }
    }
    return 0;
}

/* d_feats [M][n_in] is written; d_prior, dW, db are ACCUMULATED into (d_prior may be NULL
   without a prior, dW / db without an MLP).  band / side as in lpo_render_bwd. */
int lpo_splat_bwd(const lpo_grid* tgt, const lpo_rays* rays, const lpo_splat* sp,
                  const double* const theta_w[3], const double* const d_out[3], double* d_feats,
                  double* const d_prior[3], double* const dW[], double* const db[], double band, int side)
{
    if (splat_check(tgt, rays, sp)) return 1;
    if (side != 0 && !(band > 0.0)) return 1;
    const int C = tgt->C, S = rays->S, np = tgt->kind == LPO_TRIPLANE ? 3 : 1;
    /* dL/dtheta = G / theta_w as a grid that is then read by interpolation */
    lpo_grid ggrid = *tgt;
    double* gbuf[3] = {NULL, NULL, NULL};
    for (int p = 0; p < np; ++p) {
        const int64_t n = grid_elems(tgt, p);
        gbuf[p] = (double*)malloc(sizeof(double) * (size_t)n * C);
        if (!gbuf[p]) { for (int q = 0; q < 3; ++q) free(gbuf[q]); return 2; }
        for (int64_t c = 0; c < n; ++c) {
            const double w = theta_w[p][c];
            for (int k = 0; k < C; ++k) gbuf[p][c * C + k] = w > 0.0 ? d_out[p][c * C + k] / w : 0.0;
        }
        ggrid.data[p] = gbuf[p];
    }
    const lpo_mlp* m = sp->mlp;
    const int nact = m ? mlp_act_total(m) : 0, n_in = sp->n_in;
    const int Cp = sp->prior ? sp->prior->C : 0;
    memset(d_feats, 0, sizeof(double) * (size_t)rays->M * n_in);
    int fail = 0;
#pragma omp parallel
    {
        kink_tmp kt;
        memset(&kt, 0, sizeof(kt));
        double* act = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        double* pre = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        double* dact = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        double* din = (double*)malloc(sizeof(double) * (size_t)(nact + 1));
        double* din_other = (double*)malloc(sizeof(double) * (size_t)(nact + 1)); /* unused: no HexPlane here */
        double* dvt = (double*)malloc(sizeof(double) * (size_t)C);
        double* tW[LPO_MAX_LAYERS] = {NULL};
        double* tb[LPO_MAX_LAYERS] = {NULL};
        int ok = act && pre && dact && din && dvt;
        if (m) {
            ok = kink_alloc(&kt, m, nact) && ok;
            for (int l = 0; l < m->n_layers; ++l) {
                tW[l] = (double*)calloc((size_t)m->dims[l] * m->dims[l + 1], sizeof(double));
                tb[l] = (double*)calloc((size_t)m->dims[l + 1], sizeof(double));
                ok = ok && tW[l] && tb[l];
            }
        }
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 16)
            for (int64_t i = 0; i < rays->M; ++i) {
                const double* o = rays->origins + 3 * i;
                const double* d = rays->dirs + 3 * i;
                const double nr = rays->near[i], delta = (rays->far[i] - nr) / (double)S;
                const int b = rays->scene ? rays->scene[i] : 0;
                for (int j = 0; j < S; ++j) {
                    const double t = nr + ((double)j + 0.5) * delta;
                    const double x[3] = {o[0] + t * d[0], o[1] + t * d[1], o[2] + t * d[2]};
                    grid_gather(&ggrid, b, x, 0.0, dvt); /* dL/d(vt_ij) */
                    if (!m) {
                        for (int k = 0; k < n_in; ++k) d_feats[(size_t)i * n_in + k] += dvt[k];
                        continue;
                    }
                    splat_inputs(rays, sp, i, b, x, act);
                    mlp_forward(m, act, pre);
                    mlp_backward_choice(m, act, pre, nact, dvt, band, side, &kt, tW, tb, dact, din, din_other);
                    for (int k = 0; k < n_in; ++k) d_feats[(size_t)i * n_in + k] += din[k];
                    if (sp->prior) grid_scatter(sp->prior, d_prior, b, x, 0.0, din + n_in, NULL);
                }
            }
            if (m) {
#pragma omp critical
                for (int l = 0; l < m->n_layers; ++l) {
                    const int64_t n = (int64_t)m->dims[l] * m->dims[l + 1];
                    for (int64_t k = 0; k < n; ++k) dW[l][k] += tW[l][k];
                    for (int k = 0; k < m->dims[l + 1]; ++k) db[l][k] += tb[l][k];
                }
            }
        }
        for (int l = 0; l < LPO_MAX_LAYERS; ++l) { free(tW[l]); free(tb[l]); }
        free(act); free(pre); free(dact); free(din); free(din_other); free(dvt);
        if (m) kink_free(&kt);
    }
    for (int p = 0; p < 3; ++p) free(gbuf[p]);
    (void)Cp;
    return fail ? 2 : 0;
}
