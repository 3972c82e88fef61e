"""Python face of the CPU oracle (`lp_oracle.c`).  TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py`
may import this package.  It compiles `lp_oracle.c` with gcc (fp64, OpenMP over
rays) into `oracle/liblp_oracle.so` and calls it through ctypes.  Inputs are the
float32 host buffers of `lp_inputs.Inputs`, widened exactly to float64; every
result is float64.  Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lp_oracle.c")
_LIB = os.path.join(_HERE, "liblp_oracle.so")
_MAX_LAYERS = 8
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Grid(C.Structure):
    _fields_ = [("kind", C.c_int32), ("B", C.c_int32), ("C", C.c_int32),
                ("NX", C.c_int32), ("NY", C.c_int32), ("NZ", C.c_int32),
                ("data", C.c_void_p * 3),
                ("aabb_min", C.c_double * 3), ("aabb_max", C.c_double * 3),
                ("contract_a", C.c_double), ("hash_size", C.c_int64),
                ("data_t", C.c_void_p * 3), ("NT", C.c_int32), ("t_min", C.c_double), ("t_max", C.c_double)]


class _Mlp(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.c_int32 * (_MAX_LAYERS + 1)),
                ("W", C.c_void_p * _MAX_LAYERS), ("b", C.c_void_p * _MAX_LAYERS)]


class _Decoder(C.Structure):
    _fields_ = [("opacity", _Mlp), ("color", _Mlp), ("n_freq", C.c_int32), ("n_feat", C.c_int32),
                ("feat_act", C.c_int32)]


class _Rays(C.Structure):
    _fields_ = [("M", C.c_int64), ("S", C.c_int32),
                ("origins", C.c_void_p), ("dirs", C.c_void_p),
                ("near", C.c_void_p), ("far", C.c_void_p), ("scene", C.c_void_p), ("time", C.c_void_p)]


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.lpo_render_fwd.restype = C.c_int
        _lib.lpo_render_bwd.restype = C.c_int
        _lib.lpo_ray_trace.restype = C.c_int
        _lib.lpo_num_threads.restype = C.c_int
        _lib.lpo_render2_fwd.restype = C.c_int
        _lib.lpo_render2_bwd.restype = C.c_int
        _lib.lpo_dir_encode.restype = C.c_int
    return _lib


def hash_slot(ix: int, iy: int, iz: int, hash_size: int) -> int:
    """Entry of lattice corner (ix, iy, iz) in a hash table of `hash_size` entries."""
    lib = _load()
    lib.lpo_hash_slot.restype = C.c_int64
    return int(lib.lpo_hash_slot(C.c_int32(ix), C.c_int32(iy), C.c_int32(iz), C.c_int64(hash_size)))


def num_threads() -> int:
    return int(_load().lpo_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


class Problem:
    """Float64 copies of one `lp_inputs.Inputs` plus the C structs that point at them."""

    def __init__(self, inp):
        self.inp = inp
        self.grid = [_f64(g) for g in inp.grid]
        self.W = [_f64(w) for w in inp.weights]
        self.b = [_f64(b) for b in inp.biases]
        self.origins = _f64(inp.origins)
        self.dirs = _f64(inp.dirs)
        self.near = _f64(inp.near)
        self.far = _f64(inp.far)
        self.scene = None if inp.scene is None else np.ascontiguousarray(inp.scene, dtype=np.int32)
        self.time = None if getattr(inp, "time", None) is None else _f64(inp.time)
        # the library takes bg as float32; widen that value exactly
        self.bg = (C.c_double * len(inp.bg))(*[float(np.float32(v)) for v in inp.bg])

        g = _Grid()
        g.kind, g.B, g.C = inp.kind, inp.n_scenes, inp.channels
        g.NX, g.NY, g.NZ = inp.res
        for p, arr in enumerate(self.grid):
            if p < 3:
                g.data[p] = arr.ctypes.data
            else:
                g.data_t[p - 3] = arr.ctypes.data          # HexPlane: the space-time planes
        if inp.kind == 3:
            g.NT = int(self.grid[3].shape[2])
            g.t_min, g.t_max = float(np.float32(inp.t_range[0])), float(np.float32(inp.t_range[1]))
        for a in range(3):
            g.aabb_min[a] = float(inp.aabb_min[a])
            g.aabb_max[a] = float(inp.aabb_max[a])
        # the library takes the scale as float32; widen that value exactly
        g.contract_a = float(np.float32(getattr(inp, "contract_a", 0.0)))
        g.hash_size = int(self.grid[0].shape[1]) if inp.kind == 2 else 0   # hash table [B][T][C]
        self.c_grid = g

        m = _Mlp()
        m.n_layers = len(self.W)
        for i, d in enumerate(inp.mlp_dims):
            m.dims[i] = int(d)
        for l in range(len(self.W)):
            assert self.W[l].shape == (inp.mlp_dims[l + 1], inp.mlp_dims[l])
            m.W[l] = self.W[l].ctypes.data
            m.b[l] = self.b[l].ctypes.data
        self.c_mlp = m

        self.c_decoder = None
        dec = getattr(inp, "decoder", None)
        if dec is not None:
            self.Ws = [_f64(w) for w in dec.weights_s]
            self.bs = [_f64(b) for b in dec.biases_s]
            self.Wv = [_f64(w) for w in dec.weights_v]
            self.bv = [_f64(b) for b in dec.biases_v]
            d = _Decoder()
            for mm, dims, Ws, bs in ((d.opacity, dec.dims_s, self.Ws, self.bs),
                                     (d.color, dec.dims_v, self.Wv, self.bv)):
                mm.n_layers = len(Ws)
                for i, v in enumerate(dims):
                    mm.dims[i] = int(v)
                for l in range(len(Ws)):
                    assert Ws[l].shape == (dims[l + 1], dims[l])
                    mm.W[l] = Ws[l].ctypes.data
                    mm.b[l] = bs[l].ctypes.data
            d.n_freq, d.n_feat, d.feat_act = int(dec.n_freq), int(dec.n_feat), int(dec.feat_act)
            self.c_decoder = d
            self.bg = (C.c_double * dec.n_feat)(*[float(np.float32(v)) for v in inp.bg])

        r = _Rays()
        r.M, r.S = self.origins.shape[0], int(inp.samples)
        r.origins, r.dirs = self.origins.ctypes.data, self.dirs.ctypes.data
        r.near, r.far = self.near.ctypes.data, self.far.ctypes.data
        r.scene = None if self.scene is None else self.scene.ctypes.data
        r.time = None if self.time is None else self.time.ctypes.data
        self.c_rays = r

    @property
    def n_rays(self) -> int:
        return int(self.origins.shape[0])


def render_fwd(inp):
    """rgb [M][3], alpha [M], depth [M] (float64) by Eq. (1) of the paper."""
    p = inp if isinstance(inp, Problem) else Problem(inp)
    m = p.n_rays
    rgb = np.zeros((m, 3)); alpha = np.zeros(m); depth = np.zeros(m)
    rc = _load().lpo_render_fwd(C.byref(p.c_grid), C.byref(p.c_mlp), C.byref(p.c_rays), p.bg,
                                C.c_void_p(rgb.ctypes.data), C.c_void_p(alpha.ctypes.data),
                                C.c_void_p(depth.ctypes.data))
    if rc != 0:
        raise RuntimeError(f"lpo_render_fwd failed with status {rc}")
    return rgb, alpha, depth


def render_bwd(inp, p_rgb, p_alpha=None, p_depth=None, kink_band: float = 0.0, kink_side: int = 0):
    """Gradients of sum_i (p_rgb.rgb + p_alpha alpha + p_depth depth) w.r.t. the grid
    tensors, weights and biases.  Returns (d_grid list, dW list, db list), float64.
    kink_side = 0 is the definition; +1 / -1 give the upper / lower envelope over the
    one-sided ReLU derivatives of pre-activations within kink_band times the unit's
    rounding-error scale of zero (see lp_oracle.c)."""
    p = inp if isinstance(inp, Problem) else Problem(inp)
    p_rgb = _f64(p_rgb)
    assert p_rgb.shape == (p.n_rays, 3)
    pa = None if p_alpha is None else _f64(p_alpha)
    pd = None if p_depth is None else _f64(p_depth)
    d_grid = [np.zeros_like(g) for g in p.grid]
    dW = [np.zeros_like(w) for w in p.W]
    db = [np.zeros_like(b) for b in p.b]
    dg_arr = (C.c_void_p * 6)(*[d_grid[i].ctypes.data if i < len(d_grid) else None for i in range(6)])
    dW_arr = (C.c_void_p * _MAX_LAYERS)(*[w.ctypes.data for w in dW])
    db_arr = (C.c_void_p * _MAX_LAYERS)(*[b.ctypes.data for b in db])
    rc = _load().lpo_render_bwd(C.byref(p.c_grid), C.byref(p.c_mlp), C.byref(p.c_rays), p.bg,
                                C.c_void_p(p_rgb.ctypes.data),
                                None if pa is None else C.c_void_p(pa.ctypes.data),
                                None if pd is None else C.c_void_p(pd.ctypes.data),
                                dg_arr, dW_arr, db_arr, C.c_double(kink_band), C.c_int(kink_side))
    if rc != 0:
        raise RuntimeError(f"lpo_render_bwd failed with status {rc}")
    return d_grid, dW, db


def ray_trace(inp, ray: int, p_rgb=None, p_alpha: float = 0.0, p_depth: float = 0.0):
    """Per-sample quantities of one ray (dict of float64 arrays): t, x, feat, sigma, col,
    T (S+1 entries, T[0] = 1), w; plus dsigma, dcol when p_rgb (3 floats) is given."""
    p = inp if isinstance(inp, Problem) else Problem(inp)
    s, c = int(p.c_rays.S), int(p.c_grid.C)
    out = dict(t=np.zeros(s), x=np.zeros((s, 3)), feat=np.zeros((s, c)), sigma=np.zeros(s),
               col=np.zeros((s, 3)), T=np.zeros(s + 1), w=np.zeros(s))
    ptr = lambda a: C.c_void_p(a.ctypes.data)
    pr = None
    dsig = dcol = None
    if p_rgb is not None:
        pr = _f64(p_rgb).reshape(3)
        dsig, dcol = np.zeros(s), np.zeros((s, 3))
        out["dsigma"], out["dcol"] = dsig, dcol
    rc = _load().lpo_ray_trace(C.byref(p.c_grid), C.byref(p.c_mlp), C.byref(p.c_rays), p.bg,
                               C.c_int64(ray), None if pr is None else ptr(pr),
                               C.c_double(p_alpha), C.c_double(p_depth),
                               ptr(out["t"]), ptr(out["x"]), ptr(out["feat"]), ptr(out["sigma"]),
                               ptr(out["col"]), ptr(out["T"]), ptr(out["w"]),
                               None if dsig is None else ptr(dsig),
                               None if dcol is None else ptr(dcol))
    if rc != 0:
        raise RuntimeError(f"lpo_ray_trace failed with status {rc}")
    return out


# ---- the paper's two-MLP, view-dependent decoder (Section 3.3, below Eq. (1)) ----------------

def dir_encode(d, n_freq: int) -> np.ndarray:
    """enc(d) of one direction: (d, sin(2^k pi d), cos(2^k pi d) for k < n_freq)."""
    d = _f64(d).reshape(3)
    enc = np.zeros(3 + 6 * n_freq)
    rc = _load().lpo_dir_encode(C.c_void_p(d.ctypes.data), C.c_int(n_freq), C.c_void_p(enc.ctypes.data))
    if rc != 0:
        raise RuntimeError(f"lpo_dir_encode failed with status {rc}")
    return enc


def render2_fwd(inp):
    """Rendered features [M][F], alpha [M], depth [M] with the decoder `inp.decoder`."""
    p = inp if isinstance(inp, Problem) else Problem(inp)
    assert p.c_decoder is not None, "inputs carry no decoder"
    m, f = p.n_rays, int(p.c_decoder.n_feat)
    out = np.zeros((m, f)); alpha = np.zeros(m); depth = np.zeros(m)
    rc = _load().lpo_render2_fwd(C.byref(p.c_grid), C.byref(p.c_decoder), C.byref(p.c_rays), p.bg,
                                 C.c_void_p(out.ctypes.data), C.c_void_p(alpha.ctypes.data),
                                 C.c_void_p(depth.ctypes.data))
    if rc != 0:
        raise RuntimeError(f"lpo_render2_fwd failed with status {rc}")
    return out, alpha, depth


def render2_bwd(inp, p_out, p_alpha=None, p_depth=None, kink_band: float = 0.0, kink_side: int = 0):
    """Gradients with the two-MLP decoder.  Returns (d_grid, dWs, dbs, dWv, dbv): lists of
    float64 arrays for the grid tensors, the opacity MLP and the feature MLP."""
    p = inp if isinstance(inp, Problem) else Problem(inp)
    assert p.c_decoder is not None, "inputs carry no decoder"
    f = int(p.c_decoder.n_feat)
    p_out = _f64(p_out)
    assert p_out.shape == (p.n_rays, f)
    pa = None if p_alpha is None else _f64(p_alpha)
    pd = None if p_depth is None else _f64(p_depth)
    d_grid = [np.zeros_like(g) for g in p.grid]
    dWs = [np.zeros_like(w) for w in p.Ws]; dbs = [np.zeros_like(b) for b in p.bs]
    dWv = [np.zeros_like(w) for w in p.Wv]; dbv = [np.zeros_like(b) for b in p.bv]
    arr = lambda lst: (C.c_void_p * _MAX_LAYERS)(*[a.ctypes.data for a in lst])
    dg_arr = (C.c_void_p * 6)(*[d_grid[i].ctypes.data if i < len(d_grid) else None for i in range(6)])
    rc = _load().lpo_render2_bwd(C.byref(p.c_grid), C.byref(p.c_decoder), C.byref(p.c_rays), p.bg,
                                 C.c_void_p(p_out.ctypes.data),
                                 None if pa is None else C.c_void_p(pa.ctypes.data),
                                 None if pd is None else C.c_void_p(pd.ctypes.data),
                                 dg_arr, arr(dWs), arr(dbs), arr(dWv), arr(dbv),
                                 C.c_double(kink_band), C.c_int(kink_side))
    if rc != 0:
        raise RuntimeError(f"lpo_render2_bwd failed with status {rc}")
    return d_grid, dWs, dbs, dWv, dbv


# ---- Splatter (Section 3.3 and the appendix's normalisation paragraph) -----------------------

class _Splat(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_freq", C.c_int32), ("feats", C.c_void_p),
                ("prior", C.POINTER(_Grid)), ("mlp", C.POINTER(_Mlp))]


class SplatProblem:
    """Float64 copies of one `lp_inputs.SplatInputs` plus the C structs that point at them."""

    def __init__(self, sp):
        self.sp = sp
        self.origins, self.dirs = _f64(sp.origins), _f64(sp.dirs)
        self.near, self.far = _f64(sp.near), _f64(sp.far)
        self.scene = None if sp.scene is None else np.ascontiguousarray(sp.scene, dtype=np.int32)
        self.feats = _f64(sp.feats)

        def grid_struct(res, channels, arrays, hash_size):
            g = _Grid()
            g.kind, g.B, g.C = sp.kind, sp.n_scenes, channels
            g.NX, g.NY, g.NZ = res
            g.hash_size = int(hash_size) if sp.kind == 2 else 0
            for p, arr in enumerate(arrays or []):
                g.data[p] = arr.ctypes.data
            for a in range(3):
                g.aabb_min[a] = float(sp.aabb_min[a])
                g.aabb_max[a] = float(sp.aabb_max[a])
            g.contract_a = float(np.float32(sp.contract_a))
            return g
        self.c_target = grid_struct(sp.res, sp.channels, None, getattr(sp, "hash_size", 0))
        self.prior = None if sp.prior is None else [_f64(g) for g in sp.prior]
        self.c_prior = None if sp.prior is None else grid_struct(sp.prior_res, sp.prior_channels, self.prior,
                                                                 getattr(sp, "prior_hash_size", 0))
        self.W = self.b = None
        self.c_mlp = None
        if sp.mlp_dims is not None:
            self.W = [_f64(w) for w in sp.weights]
            self.b = [_f64(b) for b in sp.biases]
            m = _Mlp()
            m.n_layers = len(self.W)
            for i, d in enumerate(sp.mlp_dims):
                m.dims[i] = int(d)
            for l in range(len(self.W)):
                assert self.W[l].shape == (sp.mlp_dims[l + 1], sp.mlp_dims[l])
                m.W[l] = self.W[l].ctypes.data
                m.b[l] = self.b[l].ctypes.data
            self.c_mlp = m
        r = _Rays()
        r.M, r.S = self.origins.shape[0], int(sp.samples)
        r.origins, r.dirs = self.origins.ctypes.data, self.dirs.ctypes.data
        r.near, r.far = self.near.ctypes.data, self.far.ctypes.data
        r.scene = None if self.scene is None else self.scene.ctypes.data
        self.c_rays = r
        s = _Splat()
        s.n_in, s.n_freq, s.feats = int(sp.n_in), int(sp.n_freq), self.feats.ctypes.data
        s.prior = C.pointer(self.c_prior) if self.c_prior is not None else None
        s.mlp = C.pointer(self.c_mlp) if self.c_mlp is not None else None
        self.c_splat = s

    def shapes(self, channels):
        sp = self.sp
        b, (nx, ny, nz) = sp.n_scenes, sp.res
        if sp.kind == 0:
            return [(b, nx, ny, nz, channels)]
        if sp.kind == 2:
            return [(b, int(sp.hash_size), channels)]
        return [(b, nx, ny, channels), (b, ny, nz, channels), (b, nz, nx, channels)]


def _ptr3(arrs):
    return (C.c_void_p * 3)(*[arrs[i].ctypes.data if i < len(arrs) else None for i in range(3)])


def splat_fwd(sp):
    """Returns (theta list, theta_w list): the normalised target structure and the weight sums."""
    p = sp if isinstance(sp, SplatProblem) else SplatProblem(sp)
    theta = [np.zeros(s) for s in p.shapes(p.sp.channels)]
    theta_w = [np.zeros(s[:-1]) for s in p.shapes(1)]
    lib = _load()
    lib.lpo_splat_fwd.restype = C.c_int
    rc = lib.lpo_splat_fwd(C.byref(p.c_target), C.byref(p.c_rays), C.byref(p.c_splat), _ptr3(theta), _ptr3(theta_w))
    if rc != 0:
        raise RuntimeError(f"lpo_splat_fwd failed with status {rc}")
    return theta, theta_w


def splat_bwd(sp, theta_w, d_out, kink_band: float = 0.0, kink_side: int = 0):
    """Gradients of sum(d_out * out).  Returns (d_feats [M][n_in], d_prior list, dW list, db list)."""
    p = sp if isinstance(sp, SplatProblem) else SplatProblem(sp)
    theta_w = [_f64(a) for a in theta_w]
    d_out = [_f64(a) for a in d_out]
    d_feats = np.zeros_like(p.feats)
    d_prior = [] if p.prior is None else [np.zeros_like(g) for g in p.prior]
    dW = [] if p.W is None else [np.zeros_like(w) for w in p.W]
    db = [] if p.b is None else [np.zeros_like(b) for b in p.b]
    arr = lambda lst: (C.c_void_p * _MAX_LAYERS)(*[a.ctypes.data for a in lst])
    lib = _load()
    lib.lpo_splat_bwd.restype = C.c_int
    rc = lib.lpo_splat_bwd(C.byref(p.c_target), C.byref(p.c_rays), C.byref(p.c_splat), _ptr3(theta_w), _ptr3(d_out),
                           C.c_void_p(d_feats.ctypes.data), _ptr3(d_prior), arr(dW), arr(db),
                           C.c_double(kink_band), C.c_int(kink_side))
    if rc != 0:
        raise RuntimeError(f"lpo_splat_bwd failed with status {rc}")
    return d_feats, d_prior, dW, db
