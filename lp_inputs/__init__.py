"""Seeded synthetic inputs for the Lightplane Renderer path.

This module serves BOTH the CPU oracle and the HIP library with identical host
buffers.  It holds camera geometry, random-number draws and the table of
workloads; it holds none of the method's arithmetic (no sampling of grids, no
MLP, no compositing), so neither side can inherit a mistake from it.

Every array is a C-contiguous numpy array; floats are float32, the precision of
the library's inputs.  The layouts follow the hybrid representation of the
paper (Section 3.2): a voxel grid is `[B][NX][NY][NZ][C]`, a triplane is three
tensors `[B][NX][NY][C]`, `[B][NY][NZ][C]`, `[B][NZ][NX][C]` (channels
innermost), and MLP layer `l` is a matrix `[out][in]` plus a bias `[out]`.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Tuple

import numpy as np

VOXEL = 0
TRIPLANE = 1
HASH = 2        # hash table: one [B][T][C] tensor; res is the virtual lattice whose corners are hashed into it
HEXPLANE = 3    # three spatial planes as a triplane's + three space-time planes [B][N_c][NT][C]


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic workload: the shapes of a benchmark configuration."""
    name: str
    kind: int                 # VOXEL or TRIPLANE
    n_scenes: int             # B
    channels: int             # C (the paper's K)
    res: Tuple[int, int, int]  # NX, NY, NZ
    grid_std: float
    mlp_dims: Tuple[int, ...]  # C, hidden..., 4
    image: int                # square image side
    n_cameras: int            # views per scene
    samples: int              # S (the paper's R)
    near: float = 1.0
    far: float = 4.0
    aabb: float = 2.75        # grid spans [-aabb, aabb]^3
    cfg_id: int = 0
    contract_a: float = 0.0   # > 0: contract coordinates with this foreground scale (grid spans [-1, 1]^3)
    dec_hidden: Optional[Tuple[Tuple[int, ...], Tuple[int, ...]]] = None  # two-MLP decoder: hidden widths (opacity, feature)
    dec_freq: int = 0         # octaves of its view-direction encoding
    hash_size: int = 0        # kind HASH: entries of the table per scene
    n_time: int = 0           # kind HEXPLANE: resolution of the time axis (times run over [0, 1])

    @property
    def rays(self) -> int:
        return self.n_scenes * self.n_cameras * self.image * self.image

    @property
    def ray_samples(self) -> int:
        return self.rays * self.samples

    @property
    def corners(self) -> int:
        return {TRIPLANE: 12, HEXPLANE: 24}.get(self.kind, 8)

    @property
    def gather_bytes_per_sample(self) -> int:
        """Algorithmic bytes one sample reads from the grid (corners x C x 4)."""
        return self.corners * self.channels * 4

    @property
    def mlp_flop_per_sample(self) -> int:
        d = self.mlp_dims
        return 2 * sum(d[i] * d[i + 1] for i in range(len(d) - 1))


# The five benchmark configurations (tiny, single scene, voxel, batched, large).
WORKLOADS = {
    "tiny": Workload("tiny", TRIPLANE, 1, 16, (32, 32, 32), 0.1, (16, 32, 4),
                     32, 1, 64, cfg_id=1),
    "single_scene": Workload("single_scene", TRIPLANE, 1, 32, (128, 128, 128), 0.1,
                             (32, 64, 64, 4), 128, 1, 128, cfg_id=2),
    "voxel": Workload("voxel", VOXEL, 1, 32, (64, 64, 64), 0.1, (32, 64, 4),
                      256, 4, 256, cfg_id=3),
    "batched": Workload("batched", TRIPLANE, 8, 32, (256, 256, 256), 0.1,
                        (32, 64, 64, 4), 256, 4, 192, cfg_id=4),
    "large": Workload("large", VOXEL, 1, 16, (256, 256, 256), 0.05,
                      (16, 64, 64, 4), 800, 1, 512, cfg_id=5),
    # The Renderer shape of the paper's experiments (appendix, "Experimental Details"): 160^3 voxel
    # grid with 32 features, 3-layer MLP of width 64, 256^2 image, 384 points per ray, contract
    # coordinates (unbounded scene: the rays run far beyond the unit cube).
    "contract": Workload("contract", VOXEL, 1, 32, (160, 160, 160), 0.1, (32, 64, 64, 4),
                         256, 1, 384, near=0.5, far=12.0, aabb=1.0, cfg_id=6, contract_a=1.0),
    # The paper's decoder (opacity MLP + view-dependent feature MLP, Section 3.3) at a size the
    # matrix-core kernels take: 16 grid channels, two hidden layers of 32 + 32, 15 direction inputs.
    "decoder": Workload("decoder", VOXEL, 1, 16, (128, 128, 128), 0.1, (16, 64, 64, 4),
                        256, 1, 256, cfg_id=7, dec_hidden=((32, 32), (32, 32)), dec_freq=2),
    # The same decoder at the size of the paper's experiments (appendix, "Experimental Details":
    # 160^3 voxels with 32 channels, two 3-layer MLPs of width 64, 256^2 image, 384 points per ray,
    # contract coordinates): the two MLPs run as two chains on the matrix cores.
    "decoder_paper": Workload("decoder_paper", VOXEL, 1, 32, (160, 160, 160), 0.1, (32, 64, 64, 4),
                              256, 1, 384, near=0.5, far=12.0, aabb=1.0, cfg_id=10, contract_a=1.0,
                              dec_hidden=((64, 64), (64, 64)), dec_freq=2),
    # A hash table (one level of Instant-NGP's spatial hash, 2^19 entries of 16 channels over a 128^3
    # lattice) under the largest configuration's MLP.
    "hash": Workload("hash", HASH, 1, 16, (128, 128, 128), 0.1, (16, 64, 64, 4), 128, 1, 128, cfg_id=11,
                     hash_size=1 << 19),
    # A HexPlane (three 128^2 spatial planes and three 128 x 16 space-time planes of 16 channels), rays
    # of one view with a frame time each.
    "hexplane": Workload("hexplane", HEXPLANE, 1, 16, (128, 128, 128), 0.1, (16, 64, 64, 4), 128, 1, 128, cfg_id=12,
                         n_time=16),
}
WORKLOAD_ORDER = ["tiny", "single_scene", "voxel", "batched", "large"]


def _seed(cfg_id: int, what: int, extra: int = 0) -> int:
    # what: 0 grid, 1 weights, 2 target, 3 upstream alpha/depth grads
    return 1000 * cfg_id + what + 10 * extra


def camera_pose(azimuth_deg: float, elevation_deg: float, radius: float):
    """Camera-to-world rotation (columns right, up, back) and position of a
    camera on a sphere, looking at the origin with +y up."""
    az = math.radians(azimuth_deg)
    el = math.radians(elevation_deg)
    pos = np.array([radius * math.cos(el) * math.sin(az),
                    radius * math.sin(el),
                    radius * math.cos(el) * math.cos(az)], dtype=np.float64)
    back = pos / np.linalg.norm(pos)          # camera looks along -back
    up0 = np.array([0.0, 1.0, 0.0])
    right = np.cross(up0, back)
    right /= np.linalg.norm(right)
    up = np.cross(back, right)
    rot = np.stack([right, up, back], axis=1)  # world = rot @ cam
    return rot, pos


def pinhole_rays(width: int, rot: np.ndarray, pos: np.ndarray, fov_deg: float = 60.0):
    """Unit ray directions through pixel centres of a square pinhole image.
    Returns (origins [W*W,3], dirs [W*W,3]) float32, row-major over (v, u)."""
    f = (width / 2.0) / math.tan(math.radians(fov_deg) / 2.0)
    u = (np.arange(width, dtype=np.float64) + 0.5 - width / 2.0) / f
    uu, vv = np.meshgrid(u, u, indexing="xy")
    cam = np.stack([uu, -vv, -np.ones_like(uu)], axis=-1).reshape(-1, 3)
    cam /= np.linalg.norm(cam, axis=1, keepdims=True)
    world = cam @ rot.T
    # normalise once more in float32 so that |d| = 1 to float32 rounding
    world = world.astype(np.float32)
    world /= np.linalg.norm(world.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    origins = np.broadcast_to(pos.astype(np.float32), world.shape).copy()
    return origins, np.ascontiguousarray(world)


def cameras_for(w: Workload):
    if w.n_cameras == 1:
        return [camera_pose(0.0, 0.0, 2.5)]
    return [camera_pose(45.0 + 90.0 * k, 20.0, 2.5) for k in range(w.n_cameras)]


@dataclasses.dataclass
class Decoder:
    """The paper's two-MLP decoder: opacity MLP C -> ... -> 1 and feature MLP
    (C + E) -> ... -> F with E = 3 + 6 n_freq encoded view-direction inputs."""
    dims_s: Tuple[int, ...]
    weights_s: List[np.ndarray]
    biases_s: List[np.ndarray]
    dims_v: Tuple[int, ...]
    weights_v: List[np.ndarray]
    biases_v: List[np.ndarray]
    n_freq: int
    n_feat: int
    feat_act: int = 0                 # 0: logistic sigmoid, 1: identity

    @property
    def n_enc(self) -> int:
        return 3 + 6 * self.n_freq


def make_decoder(channels: int, hidden_s, hidden_v, n_freq: int, n_feat: int, seed: int,
                 bias_std: float = 0.0, feat_act: int = 0) -> Decoder:
    """He-normal weights for both MLPs; hidden_s / hidden_v are the hidden widths."""
    dims_s = (channels, *hidden_s, 1)
    dims_v = (channels + 3 + 6 * n_freq, *hidden_v, n_feat)
    ws, bs = make_mlp(dims_s, seed, bias_std)
    wv, bv = make_mlp(dims_v, seed + 1, bias_std)
    return Decoder(dims_s=tuple(dims_s), weights_s=ws, biases_s=bs, dims_v=tuple(dims_v), weights_v=wv,
                   biases_v=bv, n_freq=n_freq, n_feat=n_feat, feat_act=feat_act)


@dataclasses.dataclass
class Inputs:
    """Host buffers for one call of the Renderer."""
    kind: int
    n_scenes: int
    channels: int
    res: Tuple[int, int, int]
    grid: List[np.ndarray]            # 1 (voxel, hash table), 3 (triplane) or 6 (HexPlane) float32 arrays
    aabb_min: Tuple[float, float, float]
    aabb_max: Tuple[float, float, float]
    mlp_dims: Tuple[int, ...]
    weights: List[np.ndarray]         # [out][in] float32 per layer
    biases: List[np.ndarray]          # [out] float32 per layer
    origins: np.ndarray               # [M][3] float32
    dirs: np.ndarray                  # [M][3] float32, unit length
    near: np.ndarray                  # [M] float32
    far: np.ndarray                   # [M] float32
    scene: Optional[np.ndarray]       # [M] int32 or None when n_scenes == 1
    samples: int
    bg: Tuple[float, float, float]
    target: Optional[np.ndarray] = None  # [M][3] float32 (for the MSE loss)
    contract_a: float = 0.0           # > 0: contract coordinates with this foreground scale
    decoder: Optional[Decoder] = None  # set: the two-MLP decoder is used (bg / target have n_feat channels)
    time: Optional[np.ndarray] = None  # [M] float32: the time of every ray (read by a HexPlane only)
    t_range: Tuple[float, float] = (0.0, 1.0)   # times that map to the first and last index of the time axis

    @property
    def n_time(self) -> int:
        """Resolution of the time axis of a HexPlane, else 0."""
        return int(self.grid[3].shape[2]) if self.kind == HEXPLANE else 0

    @property
    def n_rays(self) -> int:
        return int(self.origins.shape[0])

    @property
    def hash_size(self) -> int:
        """Entries per scene of a hash table (kind HASH), else 0."""
        return int(self.grid[0].shape[1]) if self.kind == HASH else 0

    def subset(self, idx: np.ndarray) -> "Inputs":
        """The same scene with only rays `idx` (rays are independent units)."""
        idx = np.asarray(idx)
        return dataclasses.replace(
            self,
            origins=np.ascontiguousarray(self.origins[idx]),
            dirs=np.ascontiguousarray(self.dirs[idx]),
            near=np.ascontiguousarray(self.near[idx]),
            far=np.ascontiguousarray(self.far[idx]),
            scene=None if self.scene is None else np.ascontiguousarray(self.scene[idx]),
            target=None if self.target is None else np.ascontiguousarray(self.target[idx]),
            time=None if self.time is None else np.ascontiguousarray(self.time[idx]),
        )


def grid_shapes(kind: int, n_scenes: int, res, channels: int, hash_size: Optional[int] = None,
                n_time: Optional[int] = None):
    nx, ny, nz = res
    if kind == VOXEL:
        return [(n_scenes, nx, ny, nz, channels)]
    if kind == HASH:
        assert hash_size is not None and hash_size >= 1
        return [(n_scenes, int(hash_size), channels)]
    planes = [(n_scenes, nx, ny, channels), (n_scenes, ny, nz, channels), (n_scenes, nz, nx, channels)]
    if kind == HEXPLANE:
        # the space-time plane of pair p spans (the spatial axis plane p leaves out, time)
        assert n_time is not None and n_time >= 2
        planes += [(n_scenes, nz, int(n_time), channels), (n_scenes, nx, int(n_time), channels),
                   (n_scenes, ny, int(n_time), channels)]
    return planes


def make_grid(kind, n_scenes, res, channels, std, seed, hash_size=None, n_time=None) -> List[np.ndarray]:
    """Entries N(0, std); the space-time planes of a HexPlane N(1, std), so that the products of a
    pair keep the scale of the spatial planes."""
    out = []
    shapes = grid_shapes(kind, n_scenes, res, channels, hash_size, n_time)
    per_scene = [np.empty(s, dtype=np.float32) for s in shapes]
    for b in range(n_scenes):
        rng = np.random.default_rng(seed + 10 * b)
        for p, s in enumerate(shapes):
            blk = rng.standard_normal(s[1:], dtype=np.float32)
            blk *= np.float32(std)
            if kind == HEXPLANE and p >= 3:
                blk += np.float32(1.0)
            per_scene[p][b] = blk
    out.extend(per_scene)
    return out


def make_mlp(dims, seed, bias_std: float = 0.0):
    """He-normal weights N(0, sqrt(2/fan_in)); zero biases unless bias_std > 0."""
    rng = np.random.default_rng(seed)
    ws, bs = [], []
    for l in range(len(dims) - 1):
        fan_in, fan_out = dims[l], dims[l + 1]
        w = rng.standard_normal((fan_out, fan_in)).astype(np.float32)
        w *= np.float32(math.sqrt(2.0 / fan_in))
        b = (rng.standard_normal(fan_out) * bias_std).astype(np.float32)
        ws.append(np.ascontiguousarray(w))
        bs.append(np.ascontiguousarray(b))
    return ws, bs


def make_rays(w: Workload):
    """Rays of every camera of every scene, scene-major then camera then pixel."""
    per_cam = [pinhole_rays(w.image, rot, pos) for rot, pos in cameras_for(w)]
    o1 = np.concatenate([o for o, _ in per_cam], axis=0)
    d1 = np.concatenate([d for _, d in per_cam], axis=0)
    origins = np.tile(o1, (w.n_scenes, 1))
    dirs = np.tile(d1, (w.n_scenes, 1))
    m = origins.shape[0]
    near = np.full(m, w.near, dtype=np.float32)
    far = np.full(m, w.far, dtype=np.float32)
    scene = None
    if w.n_scenes > 1:
        scene = np.repeat(np.arange(w.n_scenes, dtype=np.int32), o1.shape[0])
    return (np.ascontiguousarray(origins), np.ascontiguousarray(dirs), near, far, scene)


def make_inputs(name: str, aabb: Optional[float] = None, with_grid: bool = True) -> Inputs:
    """All host buffers of workload `name` (see WORKLOADS)."""
    w = WORKLOADS[name]
    a = w.aabb if aabb is None else aabb
    grid = (make_grid(w.kind, w.n_scenes, w.res, w.channels, w.grid_std, _seed(w.cfg_id, 0), w.hash_size or None,
                      w.n_time or None)
            if with_grid else [])
    ws, bs = make_mlp(w.mlp_dims, _seed(w.cfg_id, 1))
    origins, dirs, near, far, scene = make_rays(w)
    rng = np.random.default_rng(_seed(w.cfg_id, 2))
    target = rng.random((origins.shape[0], 3), dtype=np.float32)
    decoder = None
    if w.dec_hidden is not None:
        decoder = make_decoder(w.channels, w.dec_hidden[0], w.dec_hidden[1], w.dec_freq, 3, _seed(w.cfg_id, 3))
    time = None
    if w.kind == HEXPLANE:   # a training batch of a dynamic scene: every ray from a frame drawn at random
        time = np.random.default_rng(_seed(w.cfg_id, 4)).random(origins.shape[0], dtype=np.float32)
    return Inputs(time=time, kind=w.kind, n_scenes=w.n_scenes, channels=w.channels, res=w.res, grid=grid, decoder=decoder,
                  aabb_min=(-a, -a, -a), aabb_max=(a, a, a), mlp_dims=w.mlp_dims,
                  weights=ws, biases=bs, origins=origins, dirs=dirs, near=near, far=far,
                  scene=scene, samples=w.samples, bg=(1.0, 1.0, 1.0), target=target,
                  contract_a=w.contract_a)


def strided_ray_subset(n_rays: int, n_keep: int, offset: int = 0) -> np.ndarray:
    """Deterministic subset: every (n_rays // n_keep)-th ray, starting at offset."""
    n_keep = min(n_keep, n_rays)
    stride = max(1, n_rays // n_keep)
    return (np.arange(n_keep, dtype=np.int64) * stride + offset) % n_rays


def make_small(kind: int, *, n_scenes=1, channels=4, res=(5, 4, 6), mlp_dims=(4, 8, 4),
               n_rays=6, samples=7, seed=0, grid_std=0.5, bias_std=0.3,
               aabb_min=(-1.0, -1.0, -1.0), aabb_max=(1.0, 1.0, 1.0),
               near=(0.3, 0.9), far=(2.2, 3.7), origin_radius=2.0,
               bg=(0.9, 0.5, 0.2), hash_size=None, n_time=None, t_range=(0.0, 1.0)) -> Inputs:
    """A small random problem for pins and edge cases: rays from random points on a
    sphere towards random points near the origin, per-ray near/far, non-cubic grid,
    non-zero biases, coloured background."""
    rng = np.random.default_rng(seed)
    grid = make_grid(kind, n_scenes, res, channels, grid_std, seed + 1, hash_size, n_time)
    ws, bs = make_mlp(mlp_dims, seed + 2, bias_std=bias_std)
    p = rng.standard_normal((n_rays, 3))
    p /= np.linalg.norm(p, axis=1, keepdims=True)
    origins = (origin_radius * p).astype(np.float32)
    look = rng.uniform(-0.6, 0.6, size=(n_rays, 3))
    d = look - origins
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    d = d.astype(np.float32)
    d /= np.linalg.norm(d.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    nr = rng.uniform(near[0], near[1], size=n_rays).astype(np.float32)
    fr = rng.uniform(far[0], far[1], size=n_rays).astype(np.float32)
    scene = None
    if n_scenes > 1:
        scene = rng.integers(0, n_scenes, size=n_rays).astype(np.int32)
    target = rng.random((n_rays, 3), dtype=np.float32)
    time = None
    if kind == HEXPLANE:
        # times over a little more than the range, so that some rays clamp onto its ends
        span = t_range[1] - t_range[0]
        time = rng.uniform(t_range[0] - 0.1 * span, t_range[1] + 0.1 * span, size=n_rays).astype(np.float32)
    return Inputs(time=time, t_range=tuple(t_range), kind=kind, n_scenes=n_scenes, channels=channels, res=tuple(res), grid=grid,
                  aabb_min=tuple(aabb_min), aabb_max=tuple(aabb_max), mlp_dims=tuple(mlp_dims),
                  weights=ws, biases=bs, origins=np.ascontiguousarray(origins),
                  dirs=np.ascontiguousarray(d), near=nr, far=fr, scene=scene, samples=samples,
                  bg=tuple(bg), target=target)


def upstream_grads(n_rays: int, seed: int):
    """Random upstream gradients for alpha and depth (the MSE loss only feeds rgb)."""
    rng = np.random.default_rng(seed)
    p_alpha = (rng.standard_normal(n_rays) / n_rays).astype(np.float32)
    p_depth = (rng.standard_normal(n_rays) / n_rays).astype(np.float32)
    return p_alpha, p_depth


# ---- Splatter inputs ----------------------------------------------------------------------

@dataclasses.dataclass
class SplatInputs:
    """Host buffers for one call of the Splatter: M pixels (rays + feature vectors) pushed
    into a target hash structure of `channels` channels; optional prior structure and MLP."""
    kind: int
    n_scenes: int
    channels: int                     # channels of the target structure
    res: Tuple[int, int, int]
    aabb_min: Tuple[float, float, float]
    aabb_max: Tuple[float, float, float]
    origins: np.ndarray               # [M][3] float32
    dirs: np.ndarray                  # [M][3] float32, unit length
    near: np.ndarray
    far: np.ndarray
    scene: Optional[np.ndarray]
    samples: int
    feats: np.ndarray                 # [M][n_in] float32 pixel features
    n_freq: int = -1                  # octaves of the direction encoding fed to the MLP, -1: none
    prior: Optional[List[np.ndarray]] = None   # prior structure (same kind and box), float32
    prior_res: Optional[Tuple[int, int, int]] = None
    prior_channels: int = 0
    mlp_dims: Optional[Tuple[int, ...]] = None  # None: naive Splatter (n_in == channels)
    weights: Optional[List[np.ndarray]] = None
    biases: Optional[List[np.ndarray]] = None
    contract_a: float = 0.0
    hash_size: int = 0                # kind HASH: entries per scene of the target table
    prior_hash_size: int = 0          # kind HASH: entries per scene of the prior table

    @property
    def n_rays(self) -> int:
        return int(self.origins.shape[0])

    @property
    def n_in(self) -> int:
        return int(self.feats.shape[1])

    @property
    def n_enc(self) -> int:
        return 0 if self.n_freq < 0 else 3 + 6 * self.n_freq


def make_splat_small(kind: int, *, n_scenes=1, channels=4, res=(5, 4, 6), n_in=None, hidden=None,
                     n_freq=-1, prior_channels=0, prior_res=(4, 5, 3), n_rays=6, samples=7, seed=0,
                     bias_std=0.3, hash_size=0, prior_hash_size=0, **ray_kw) -> SplatInputs:
    """A small random Splatter problem: the rays of `make_small`, random pixel features,
    optionally a random prior structure and a He-normal MLP with hidden widths `hidden`."""
    base = make_small(kind, n_scenes=n_scenes, channels=channels, res=res, mlp_dims=(channels, 4),
                      n_rays=n_rays, samples=samples, seed=seed, hash_size=hash_size or None, **ray_kw)
    rng = np.random.default_rng(seed + 50)
    n_in = channels if n_in is None else n_in
    feats = rng.standard_normal((n_rays, n_in)).astype(np.float32)
    prior = None
    if prior_channels:
        prior = make_grid(kind, n_scenes, prior_res, prior_channels, 0.5, seed + 51, prior_hash_size or None)
    dims = ws = bs = None
    if hidden is not None:
        n_enc = 0 if n_freq < 0 else 3 + 6 * n_freq
        dims = (n_in + prior_channels + n_enc, *hidden, channels)
        ws, bs = make_mlp(dims, seed + 52, bias_std)
    return SplatInputs(kind=kind, n_scenes=n_scenes, channels=channels, res=tuple(res),
                       aabb_min=base.aabb_min, aabb_max=base.aabb_max, origins=base.origins, dirs=base.dirs,
                       near=base.near, far=base.far, scene=base.scene, samples=samples, feats=feats,
                       n_freq=n_freq if hidden is not None else -1, prior=prior,
                       prior_res=tuple(prior_res) if prior_channels else None, prior_channels=prior_channels,
                       mlp_dims=dims, weights=ws, biases=bs, hash_size=int(hash_size),
                       prior_hash_size=int(prior_hash_size) if prior_channels else 0)


@dataclasses.dataclass(frozen=True)
class SplatWorkload:
    """Shapes of a Splatter benchmark: `n_cameras` views of `image`^2 pixels with `n_in`-channel
    features pushed into a `res` structure of `channels` channels, `samples` points per ray."""
    name: str
    kind: int
    channels: int
    res: Tuple[int, int, int]
    n_in: int
    image: int
    n_cameras: int
    samples: int
    hidden: Optional[Tuple[int, ...]] = None   # None: naive Splatter
    prior_channels: int = 0
    n_freq: int = -1
    near: float = 1.0
    far: float = 4.0
    aabb: float = 2.75
    cfg_id: int = 0

    @property
    def rays(self) -> int:
        return self.n_cameras * self.image * self.image

    @property
    def ray_samples(self) -> int:
        return self.rays * self.samples

    @property
    def push_bytes_per_sample(self) -> int:
        """Algorithmic bytes one point adds to the target (corners x (C + 1) x 4)."""
        corners = 8 if self.kind == VOXEL else 12
        return corners * (self.channels + 1) * 4


# The paper's Splatter setting (appendix, "Experimental Details"): 160^3 voxel grid, 32-dimensional
# image features, 160 points per ray, 3-layer MLP of width 64; four views of 128^2 pixels.
SPLAT_WORKLOADS = {
    "splat_naive": SplatWorkload("splat_naive", VOXEL, 32, (160, 160, 160), 32, 128, 4, 160, cfg_id=8),
    # with the MLP of the paper's setting (32-channel features, prior and target; 3 layers of width
    # 64; raw direction), fewer rays: it runs on the generic kernels
    "splat_mlp": SplatWorkload("splat_mlp", VOXEL, 32, (160, 160, 160), 32, 64, 4, 160, hidden=(64, 64),
                               prior_channels=32, n_freq=0, cfg_id=9),
}


def make_splat_inputs(name: str) -> SplatInputs:
    w = SPLAT_WORKLOADS[name]
    cam = Workload(name, w.kind, 1, w.channels, w.res, 0.1, (w.channels, 4), w.image, w.n_cameras, w.samples,
                   near=w.near, far=w.far, aabb=w.aabb)
    origins, dirs, near, far, scene = make_rays(cam)
    rng = np.random.default_rng(_seed(w.cfg_id, 0))
    feats = rng.standard_normal((origins.shape[0], w.n_in), dtype=np.float32)
    prior = dims = ws = bs = None
    if w.prior_channels:
        prior = make_grid(w.kind, 1, w.res, w.prior_channels, 0.1, _seed(w.cfg_id, 1))
    if w.hidden is not None:
        n_enc = 0 if w.n_freq < 0 else 3 + 6 * w.n_freq
        dims = (w.n_in + w.prior_channels + n_enc, *w.hidden, w.channels)
        ws, bs = make_mlp(dims, _seed(w.cfg_id, 2))
    a = w.aabb
    return SplatInputs(kind=w.kind, n_scenes=1, channels=w.channels, res=w.res, aabb_min=(-a, -a, -a),
                       aabb_max=(a, a, a), origins=origins, dirs=dirs, near=near, far=far, scene=scene,
                       samples=w.samples, feats=feats, n_freq=w.n_freq if w.hidden is not None else -1, prior=prior,
                       prior_res=w.res if w.prior_channels else None, prior_channels=w.prior_channels,
                       mlp_dims=dims, weights=ws, biases=bs)
