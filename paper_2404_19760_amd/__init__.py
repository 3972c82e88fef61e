"""Python binding of the MI355X Lightplane Renderer library (`liblightplane.so`).

Argument marshalling only: every step of the Renderer runs in the library's HIP
kernels.  PyTorch supplies device memory (tensors) and streams.  The functions carry
the names of the C entry points declared in `include/lightplane.h`.

There is no CPU fallback: importing this package without a built library, or calling
it without a GPU tensor, raises.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LP_LIB_PATH", os.path.join(_HERE, "liblightplane.so"))

LP_MAX_LAYERS = 8
LP_OK, LP_ERR_INVALID_ARG, LP_ERR_UNSUPPORTED, LP_ERR_HIP, LP_ERR_WORKSPACE = range(5)
LP_GRID_VOXEL, LP_GRID_TRIPLANE, LP_GRID_HASH, LP_GRID_HEXPLANE = 0, 1, 2, 3
LP_MATH_DEFAULT, LP_MATH_GENERIC, LP_MATH_BF16X3 = 0, 1, 2
LP_FEAT_SIGMOID, LP_FEAT_IDENTITY = 0, 1
LP_F32, LP_BF16, LP_F16 = 0, 1, 2


class LightplaneError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lightplane status {status}: {message}")
        self.status = status


class _Grid(C.Structure):
    _fields_ = [("kind", C.c_int32), ("B", C.c_int32), ("C", C.c_int32),
                ("NX", C.c_int32), ("NY", C.c_int32), ("NZ", C.c_int32),
                ("data", C.c_void_p * 3),
                ("aabb_min", C.c_float * 3), ("aabb_max", C.c_float * 3), ("contract_a", C.c_float),
                ("dtype", C.c_int32), ("hash_size", C.c_int64),
                ("data_t", C.c_void_p * 3), ("NT", C.c_int32), ("t_min", C.c_float), ("t_max", C.c_float)]


class _Mlp(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.c_int32 * (LP_MAX_LAYERS + 1)),
                ("W", C.c_void_p * LP_MAX_LAYERS), ("b", C.c_void_p * LP_MAX_LAYERS)]


class _Decoder(C.Structure):
    _fields_ = [("opacity", _Mlp), ("feature", _Mlp), ("n_freq", C.c_int32), ("n_feat", C.c_int32),
                ("feat_act", C.c_int32)]


class _Splat(C.Structure):
    _fields_ = [("n_in", C.c_int32), ("n_freq", C.c_int32), ("feats", C.c_void_p),
                ("prior", C.POINTER(_Grid)), ("mlp", C.POINTER(_Mlp))]


class _Rays(C.Structure):
    _fields_ = [("M", C.c_int64), ("S", C.c_int32),
                ("origins", C.c_void_p), ("dirs", C.c_void_p),
                ("near", C.c_void_p), ("far", C.c_void_p), ("scene", C.c_void_p), ("time", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python paper_2404_19760_amd/build.py` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    lib.lp_last_error.restype = C.c_char_p
    lib.lp_version.restype = C.c_int32
    lib.lp_diag_coexecution.restype = C.c_int
    lib.lp_diag_coexecution.argtypes = [C.POINTER(C.c_float), C.c_void_p]
    lib.lp_diag_atomic_rate.restype = C.c_int
    lib.lp_diag_atomic_rate.argtypes = [C.POINTER(C.c_float), C.c_void_p]
    lib.lp_diag_ws_phases.restype = C.c_int
    lib.lp_diag_ws_phases.argtypes = [C.POINTER(C.c_ulonglong)]
    lib.lp_has_fast_path.restype = C.c_int32
    lib.lp_has_fast_path.argtypes = [C.POINTER(_Grid), C.POINTER(_Mlp)]
    lib.lp_render_fwd.restype = C.c_int
    lib.lp_render_fwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Mlp), C.POINTER(_Rays),
                                  C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_int32, C.c_void_p]
    lib.lp_render_bwd.restype = C.c_int
    lib.lp_render_bwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Mlp), C.POINTER(_Rays),
                                  C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                  C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t, C.c_int32,
                                  C.c_void_p]
    lib.lp_render_bwd_static.restype = C.c_int
    lib.lp_render_bwd_static.argtypes = [C.POINTER(_Grid), C.POINTER(_Mlp), C.POINTER(_Rays),
                                         C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                         C.POINTER(C.c_void_p), C.c_int32, C.c_void_p]
    lib.lp_bwd_workspace_bytes.restype = C.c_int
    lib.lp_bwd_workspace_bytes.argtypes = [C.POINTER(_Grid), C.POINTER(_Mlp), C.POINTER(_Rays),
                                           C.c_int32, C.POINTER(C.c_size_t)]
    lib.lp_dec_has_fast_path.restype = C.c_int32
    lib.lp_dec_has_fast_path.argtypes = [C.POINTER(_Grid), C.POINTER(_Decoder)]
    lib.lp_dec_workspace_bytes.restype = C.c_int
    lib.lp_dec_workspace_bytes.argtypes = [C.POINTER(_Grid), C.POINTER(_Decoder), C.POINTER(_Rays), C.c_int32,
                                           C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.lp_render_dec_fwd.restype = C.c_int
    lib.lp_render_dec_fwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Decoder), C.POINTER(_Rays),
                                      C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
    lib.lp_render_dec_bwd.restype = C.c_int
    lib.lp_render_dec_bwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Decoder), C.POINTER(_Rays),
                                      C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                      C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t,
                                      C.c_int32, C.c_void_p]
    lib.lp_splat_fwd.restype = C.c_int
    lib.lp_splat_fwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Rays), C.POINTER(_Splat), C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p), C.c_void_p]
    lib.lp_splat_has_fast_path.restype = C.c_int32
    lib.lp_splat_has_fast_path.argtypes = [C.POINTER(_Grid), C.POINTER(_Splat)]
    lib.lp_splat_bwd_workspace_bytes.restype = C.c_int
    lib.lp_splat_bwd_workspace_bytes.argtypes = [C.POINTER(_Grid), C.POINTER(_Rays), C.POINTER(_Splat),
                                                 C.POINTER(C.c_size_t)]
    lib.lp_splat_bwd.restype = C.c_int
    lib.lp_splat_bwd.argtypes = [C.POINTER(_Grid), C.POINTER(_Rays), C.POINTER(_Splat), C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t, C.c_void_p]
    return lib


_lib = _load()


def _check(status: int):
    if status != LP_OK:
        raise LightplaneError(status, _lib.lp_last_error().decode())


def _dev_f32(t: Optional[torch.Tensor], name: str, shape=None) -> Optional[int]:
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous float32 tensor on the GPU")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


_GRID_DTYPES = {torch.float32: LP_F32, torch.bfloat16: LP_BF16, torch.float16: LP_F16}


@dataclasses.dataclass
class Grid:
    """Voxel grid [B][NX][NY][NZ][C] (one tensor), triplane (three tensors [B][NX][NY][C],
    [B][NY][NZ][C], [B][NZ][NX][C]) or hash table [B][T][C] (one tensor; res = the virtual lattice
    whose corners are hashed into it) or HexPlane (six tensors: the triplane's three, then the
    space-time planes [B][NZ][NT][C], [B][NX][NT][C], [B][NY][NT][C]; t_range = the times of the first
    and last index of the time axis); float32, bfloat16 or float16 (all tensors alike), on the GPU."""
    kind: int
    data: List[torch.Tensor]
    res: Sequence[int]
    aabb_min: Sequence[float] = (-1.0, -1.0, -1.0)
    aabb_max: Sequence[float] = (1.0, 1.0, 1.0)
    contract_a: float = 0.0
    t_range: Sequence[float] = (0.0, 1.0)

    @property
    def n_scenes(self) -> int:
        return int(self.data[0].shape[0])

    @property
    def channels(self) -> int:
        return int(self.data[0].shape[-1])

    def shapes(self):
        b, c = self.n_scenes, self.channels
        nx, ny, nz = self.res
        if self.kind == LP_GRID_VOXEL:
            return [(b, nx, ny, nz, c)]
        if self.kind == LP_GRID_HASH:
            return [(b, int(self.data[0].shape[1]), c)]
        planes = [(b, nx, ny, c), (b, ny, nz, c), (b, nz, nx, c)]
        if self.kind == LP_GRID_HEXPLANE:
            if len(self.data) != 6:
                raise ValueError("a HexPlane has six tensors")
            nt = int(self.data[3].shape[2])
            planes += [(b, nz, nt, c), (b, nx, nt, c), (b, ny, nt, c)]
        return planes

    def c_struct(self) -> _Grid:
        g = _Grid()
        g.kind, g.B, g.C = self.kind, self.n_scenes, self.channels
        g.NX, g.NY, g.NZ = [int(v) for v in self.res]
        g.hash_size = int(self.data[0].shape[1]) if self.kind == LP_GRID_HASH else 0
        shapes = self.shapes()
        if len(self.data) != len(shapes):
            raise ValueError("wrong number of grid tensors for this kind")
        dt = self.data[0].dtype
        if dt not in _GRID_DTYPES:
            raise ValueError("grid tensors must be float32, bfloat16 or float16")
        g.dtype = _GRID_DTYPES[dt]
        for p, (t, s) in enumerate(zip(self.data, shapes)):
            if not (t.is_cuda and t.dtype == dt and t.is_contiguous() and tuple(t.shape) == tuple(s)):
                raise ValueError(f"grid.data[{p}] must be a contiguous GPU tensor of shape {tuple(s)} and the "
                                 "dtype of grid.data[0]")
            if p < 3:
                g.data[p] = t.data_ptr()
            else:
                g.data_t[p - 3] = t.data_ptr()
        if self.kind == LP_GRID_HEXPLANE:
            g.NT = int(self.data[3].shape[2])
            g.t_min, g.t_max = float(self.t_range[0]), float(self.t_range[1])
        for a in range(3):
            g.aabb_min[a] = float(self.aabb_min[a])
            g.aabb_max[a] = float(self.aabb_max[a])
        g.contract_a = float(self.contract_a)
        return g


@dataclasses.dataclass
class Mlp:
    """weights[l] = [out][in], biases[l] = [out]; float32, on the GPU."""
    weights: List[torch.Tensor]
    biases: List[torch.Tensor]

    @property
    def dims(self):
        return [int(self.weights[0].shape[1])] + [int(w.shape[0]) for w in self.weights]

    def c_struct(self) -> _Mlp:
        if len(self.weights) != len(self.biases) or not 1 <= len(self.weights) <= LP_MAX_LAYERS:
            raise ValueError("MLP needs 1..8 layers with one bias per weight matrix")
        m = _Mlp()
        m.n_layers = len(self.weights)
        dims = self.dims
        for i, d in enumerate(dims):
            m.dims[i] = d
        for l, (w, b) in enumerate(zip(self.weights, self.biases)):
            m.W[l] = _dev_f32(w, f"weights[{l}]", (dims[l + 1], dims[l]))
            m.b[l] = _dev_f32(b, f"biases[{l}]", (dims[l + 1],))
        return m


@dataclasses.dataclass
class Decoder:
    """The two-MLP decoder: opacity MLP (C -> ... -> 1) and feature MLP
    (C + 3 + 6 n_freq -> ... -> n_feat); feat_act LP_FEAT_SIGMOID or LP_FEAT_IDENTITY."""
    opacity: Mlp
    feature: Mlp
    n_freq: int
    n_feat: int
    feat_act: int = 0

    def c_struct(self) -> _Decoder:
        d = _Decoder()
        d.opacity, d.feature = self.opacity.c_struct(), self.feature.c_struct()
        d.n_freq, d.n_feat, d.feat_act = int(self.n_freq), int(self.n_feat), int(self.feat_act)
        return d


@dataclasses.dataclass
class Rays:
    origins: torch.Tensor          # [M][3]
    dirs: torch.Tensor             # [M][3] unit
    near: torch.Tensor             # [M]
    far: torch.Tensor              # [M]
    samples: int                   # S
    scene: Optional[torch.Tensor] = None  # [M] int32
    time: Optional[torch.Tensor] = None   # [M] float32, the time of every ray (read by a HexPlane only)

    @property
    def n_rays(self) -> int:
        return int(self.origins.shape[0])

    def c_struct(self) -> _Rays:
        m = self.n_rays
        r = _Rays()
        r.M, r.S = m, int(self.samples)
        r.origins = _dev_f32(self.origins, "origins", (m, 3))
        r.dirs = _dev_f32(self.dirs, "dirs", (m, 3))
        r.near = _dev_f32(self.near, "near", (m,))
        r.far = _dev_f32(self.far, "far", (m,))
        if self.scene is not None:
            s = self.scene
            if not (s.is_cuda and s.dtype == torch.int32 and s.is_contiguous() and tuple(s.shape) == (m,)):
                raise ValueError("scene must be a contiguous int32 GPU tensor of shape [M]")
            r.scene = s.data_ptr()
        if self.time is not None:
            r.time = _dev_f32(self.time, "time", (m,))
        return r


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _bg(bg) -> C.Array:
    return (C.c_float * 3)(*[float(v) for v in bg])


def lp_version() -> int:
    return int(_lib.lp_version())


def lp_diag_coexecution(stream=None):
    """Nanoseconds per loop iteration of the ten measurements the header describes."""
    out = (C.c_float * 10)()
    _check(_lib.lp_diag_coexecution(out, _stream_ptr(stream)))
    return [float(v) for v in out]


def lp_diag_atomic_rate(stream=None):
    """64-byte lines of fp32 atomic adds per second in the six settings the header describes."""
    out = (C.c_float * 6)()
    _check(_lib.lp_diag_atomic_rate(out, _stream_ptr(stream)))
    return [float(v) for v in out]


def lp_diag_ws_phases():
    """Cycle sums per phase of the two-wave backward (measurement builds only; see the header)."""
    out = (C.c_ulonglong * 32)()
    _check(_lib.lp_diag_ws_phases(out))
    return [int(v) for v in out]


def lp_has_fast_path(grid: Grid, mlp: Mlp) -> bool:
    g, m = grid.c_struct(), mlp.c_struct()
    return bool(_lib.lp_has_fast_path(C.byref(g), C.byref(m)))


def lp_render_fwd(grid: Grid, mlp: Mlp, rays: Rays, bg, rgb: torch.Tensor,
                  alpha: Optional[torch.Tensor], depth: Optional[torch.Tensor],
                  ray_cache: Optional[torch.Tensor], math_mode: int = LP_MATH_DEFAULT,
                  stream=None) -> None:
    """Enqueue the forward on `stream` (default: torch's current stream); outputs are
    caller-allocated GPU tensors rgb [M][3], alpha [M], depth [M], ray_cache [M]."""
    m = rays.n_rays
    g, ml, r = grid.c_struct(), mlp.c_struct(), rays.c_struct()
    _check(_lib.lp_render_fwd(C.byref(g), C.byref(ml), C.byref(r), _bg(bg),
                              _dev_f32(rgb, "rgb", (m, 3)), _dev_f32(alpha, "alpha", (m,)),
                              _dev_f32(depth, "depth", (m,)), _dev_f32(ray_cache, "ray_cache", (m,)),
                              int(math_mode), _stream_ptr(stream)))


def lp_bwd_workspace_bytes(grid: Grid, mlp: Mlp, rays: Rays, math_mode: int = LP_MATH_DEFAULT) -> int:
    g, ml, r = grid.c_struct(), mlp.c_struct(), rays.c_struct()
    n = C.c_size_t(0)
    _check(_lib.lp_bwd_workspace_bytes(C.byref(g), C.byref(ml), C.byref(r), int(math_mode), C.byref(n)))
    return int(n.value)


LP_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def lp_render_bwd_static(grid: Grid, mlp: Mlp, rays: Rays, bg, d_rgb: torch.Tensor,
                         d_alpha: Optional[torch.Tensor], d_depth: Optional[torch.Tensor],
                         ray_cache: torch.Tensor, d_grid: List[torch.Tensor], dW: List[torch.Tensor],
                         db: List[torch.Tensor], math_mode: int = LP_MATH_DEFAULT, stream=None) -> None:
    """lp_render_bwd without a workspace: the library's static device scratch holds the records
    (nothing is allocated; shapes that need more than LP_STATIC_SCRATCH_BYTES are refused)."""
    _render_bwd(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, None, math_mode, stream)


def lp_render_bwd(grid: Grid, mlp: Mlp, rays: Rays, bg, d_rgb: torch.Tensor,
                  d_alpha: Optional[torch.Tensor], d_depth: Optional[torch.Tensor],
                  ray_cache: torch.Tensor, d_grid: List[torch.Tensor], dW: List[torch.Tensor],
                  db: List[torch.Tensor], workspace: torch.Tensor,
                  math_mode: int = LP_MATH_DEFAULT, stream=None) -> None:
    """Enqueue the backward; d_grid / dW / db are ACCUMULATED into (same shapes as the
    grid tensors, weights and biases); `workspace` is a GPU byte tensor of at least
    lp_bwd_workspace_bytes(...) bytes."""
    if workspace is None:
        raise ValueError("workspace must be a contiguous GPU tensor")
    _render_bwd(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, workspace, math_mode, stream)


def _render_bwd(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, workspace, math_mode, stream):
    m = rays.n_rays
    g, ml, r = grid.c_struct(), mlp.c_struct(), rays.c_struct()
    shapes = grid.shapes()
    if len(d_grid) != len(shapes):
        raise ValueError("d_grid needs one tensor per grid tensor")
    dg = (C.c_void_p * 6)(*[_dev_f32(d_grid[p], f"d_grid[{p}]", shapes[p]) if p < len(shapes) else None
                            for p in range(6)])
    dims = mlp.dims
    if len(dW) != len(mlp.weights) or len(db) != len(mlp.weights):
        raise ValueError("dW / db need one tensor per layer")
    dWp = (C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(w, f"dW[{l}]", (dims[l + 1], dims[l])) for l, w in enumerate(dW)])
    dbp = (C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(b, f"db[{l}]", (dims[l + 1],)) for l, b in enumerate(db)])
    common = (C.byref(g), C.byref(ml), C.byref(r), _bg(bg),
              _dev_f32(d_rgb, "d_rgb", (m, 3)), _dev_f32(d_alpha, "d_alpha", (m,)),
              _dev_f32(d_depth, "d_depth", (m,)), _dev_f32(ray_cache, "ray_cache", (m,)), dg, dWp, dbp)
    if workspace is None:
        _check(_lib.lp_render_bwd_static(*common, int(math_mode), _stream_ptr(stream)))
        return
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous GPU tensor")
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(_lib.lp_render_bwd(*common, C.c_void_p(workspace.data_ptr()), C.c_size_t(ws_bytes),
                              int(math_mode), _stream_ptr(stream)))


def lp_dec_has_fast_path(grid: Grid, dec: Decoder) -> bool:
    g, d = grid.c_struct(), dec.c_struct()
    return bool(_lib.lp_dec_has_fast_path(C.byref(g), C.byref(d)))


def lp_dec_workspace_bytes(grid: Grid, dec: Decoder, rays: Rays, math_mode: int = LP_MATH_DEFAULT):
    """(forward bytes, backward bytes) of workspace for the two-MLP decoder calls."""
    g, d, r = grid.c_struct(), dec.c_struct(), rays.c_struct()
    nf, nb = C.c_size_t(0), C.c_size_t(0)
    _check(_lib.lp_dec_workspace_bytes(C.byref(g), C.byref(d), C.byref(r), int(math_mode), C.byref(nf), C.byref(nb)))
    return int(nf.value), int(nb.value)


def _workspace(workspace: torch.Tensor):
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous GPU tensor")
    return C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel() * workspace.element_size())


def lp_render_dec_fwd(grid: Grid, dec: Decoder, rays: Rays, bg, out: torch.Tensor,
                      alpha: Optional[torch.Tensor], depth: Optional[torch.Tensor],
                      ray_cache: Optional[torch.Tensor], workspace: torch.Tensor,
                      math_mode: int = LP_MATH_DEFAULT, stream=None) -> None:
    """Forward with the two-MLP decoder; out [M][n_feat]; bg has n_feat entries."""
    m, f = rays.n_rays, int(dec.n_feat)
    g, d, r = grid.c_struct(), dec.c_struct(), rays.c_struct()
    wp, wn = _workspace(workspace)
    _check(_lib.lp_render_dec_fwd(C.byref(g), C.byref(d), C.byref(r), (C.c_float * f)(*[float(v) for v in bg]),
                                  _dev_f32(out, "out", (m, f)), _dev_f32(alpha, "alpha", (m,)),
                                  _dev_f32(depth, "depth", (m,)), _dev_f32(ray_cache, "ray_cache", (m,)),
                                  wp, wn, int(math_mode), _stream_ptr(stream)))


def lp_render_dec_bwd(grid: Grid, dec: Decoder, rays: Rays, bg, d_out: torch.Tensor,
                      d_alpha: Optional[torch.Tensor], d_depth: Optional[torch.Tensor],
                      ray_cache: torch.Tensor, d_grid: List[torch.Tensor],
                      dW_opacity: List[torch.Tensor], db_opacity: List[torch.Tensor],
                      dW_feature: List[torch.Tensor], db_feature: List[torch.Tensor],
                      workspace: torch.Tensor, math_mode: int = LP_MATH_DEFAULT, stream=None) -> None:
    """Backward with the two-MLP decoder; all gradient tensors are ACCUMULATED into."""
    m, f = rays.n_rays, int(dec.n_feat)
    g, d, r = grid.c_struct(), dec.c_struct(), rays.c_struct()
    shapes = grid.shapes()
    if len(d_grid) != len(shapes):
        raise ValueError("d_grid needs one tensor per grid tensor")
    dg = (C.c_void_p * 6)(*[_dev_f32(d_grid[p], f"d_grid[{p}]", shapes[p]) if p < len(shapes) else None
                            for p in range(6)])

    def lists(mlp, dW, db, name):
        dims = mlp.dims
        if len(dW) != len(mlp.weights) or len(db) != len(mlp.weights):
            raise ValueError(f"dW_{name} / db_{name} need one tensor per layer")
        return ((C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(w, f"dW_{name}[{l}]", (dims[l + 1], dims[l]))
                                               for l, w in enumerate(dW)]),
                (C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(b, f"db_{name}[{l}]", (dims[l + 1],))
                                               for l, b in enumerate(db)]))
    dWs, dbs = lists(dec.opacity, dW_opacity, db_opacity, "opacity")
    dWv, dbv = lists(dec.feature, dW_feature, db_feature, "feature")
    wp, wn = _workspace(workspace)
    _check(_lib.lp_render_dec_bwd(C.byref(g), C.byref(d), C.byref(r), (C.c_float * f)(*[float(v) for v in bg]),
                                  _dev_f32(d_out, "d_out", (m, f)), _dev_f32(d_alpha, "d_alpha", (m,)),
                                  _dev_f32(d_depth, "d_depth", (m,)), _dev_f32(ray_cache, "ray_cache", (m,)),
                                  dg, dWs, dbs, dWv, dbv, wp, wn, int(math_mode), _stream_ptr(stream)))


@dataclasses.dataclass
class Splat:
    """Arguments of the Splatter besides target and rays: pixel features [M][n_in], optional
    prior structure (a Grid of the target's kind) and MLP, octaves of the direction encoding."""
    feats: torch.Tensor
    prior: Optional[Grid] = None
    mlp: Optional[Mlp] = None
    n_freq: int = -1

    def c_struct(self):
        """Returns (struct, keep-alive objects)."""
        s = _Splat()
        m, n_in = int(self.feats.shape[0]), int(self.feats.shape[1])
        s.n_in, s.n_freq = n_in, int(self.n_freq)
        s.feats = _dev_f32(self.feats, "feats", (m, n_in))
        keep = []
        if self.prior is not None:
            g = self.prior.c_struct()
            keep.append(g)
            s.prior = C.pointer(g)
        if self.mlp is not None:
            ml = self.mlp.c_struct()
            keep.append(ml)
            s.mlp = C.pointer(ml)
        return s, keep


def target_struct(kind: int, n_scenes: int, channels: int, res, aabb_min=(-1.0, -1.0, -1.0),
                  aabb_max=(1.0, 1.0, 1.0), contract_a: float = 0.0, hash_size: int = 0) -> _Grid:
    """lp_grid describing the structure a Splatter call builds (no data pointers; hash_size: the
    entries per scene of a hash-table target)."""
    g = _Grid()
    g.hash_size = int(hash_size) if int(kind) == LP_GRID_HASH else 0
    g.kind, g.B, g.C = int(kind), int(n_scenes), int(channels)
    g.NX, g.NY, g.NZ = [int(v) for v in res]
    for a in range(3):
        g.aabb_min[a] = float(aabb_min[a])
        g.aabb_max[a] = float(aabb_max[a])
    g.contract_a = float(contract_a)
    return g


def _target_shapes(t: _Grid, channels: Optional[int]):
    b, nx, ny, nz = t.B, t.NX, t.NY, t.NZ
    c = () if channels is None else (channels,)
    if t.kind == LP_GRID_VOXEL:
        return [(b, nx, ny, nz) + c]
    if t.kind == LP_GRID_HASH:
        return [(b, int(t.hash_size)) + c]
    return [(b, nx, ny) + c, (b, ny, nz) + c, (b, nz, nx) + c]


def _ptr3(tensors, shapes, name):
    if len(tensors) != len(shapes):
        raise ValueError(f"{name} needs {len(shapes)} tensors")
    return (C.c_void_p * 3)(*[_dev_f32(tensors[p], f"{name}[{p}]", shapes[p]) if p < len(shapes) else None
                              for p in range(3)])


def lp_splat_fwd(target: _Grid, rays: Rays, splat: Splat, theta: List[torch.Tensor],
                 theta_w: List[torch.Tensor], stream=None) -> None:
    """Enqueue the Splatter forward: theta (shapes of the target's tensors) and theta_w (same
    without the channel axis) are written."""
    r = rays.c_struct()
    s, keep = splat.c_struct()
    _check(_lib.lp_splat_fwd(C.byref(target), C.byref(r), C.byref(s),
                             _ptr3(theta, _target_shapes(target, target.C), "theta"),
                             _ptr3(theta_w, _target_shapes(target, None), "theta_w"), _stream_ptr(stream)))
    del keep


def lp_splat_has_fast_path(target: _Grid, splat: Splat) -> bool:
    s, keep = splat.c_struct()
    fast = bool(_lib.lp_splat_has_fast_path(C.byref(target), C.byref(s)))
    del keep
    return fast


def lp_splat_bwd_workspace_bytes(target: _Grid, rays: Rays, splat: Splat) -> int:
    r = rays.c_struct()
    s, keep = splat.c_struct()
    n = C.c_size_t(0)
    _check(_lib.lp_splat_bwd_workspace_bytes(C.byref(target), C.byref(r), C.byref(s), C.byref(n)))
    del keep
    return int(n.value)


def lp_splat_bwd(target: _Grid, rays: Rays, splat: Splat, theta_w: List[torch.Tensor],
                 d_theta: List[torch.Tensor], d_feats: torch.Tensor, d_prior: Optional[List[torch.Tensor]],
                 dW: Optional[List[torch.Tensor]], db: Optional[List[torch.Tensor]], workspace: torch.Tensor,
                 stream=None) -> None:
    """Enqueue the Splatter backward: d_feats is written; d_prior, dW, db are accumulated into."""
    r = rays.c_struct()
    s, keep = splat.c_struct()
    m, n_in = int(splat.feats.shape[0]), int(splat.feats.shape[1])
    dp = (C.c_void_p * 3)()
    if splat.prior is not None:
        dp = _ptr3(d_prior, splat.prior.shapes(), "d_prior")
    dWp, dbp = (C.c_void_p * LP_MAX_LAYERS)(), (C.c_void_p * LP_MAX_LAYERS)()
    if splat.mlp is not None:
        dims = splat.mlp.dims
        dWp = (C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(w, f"dW[{l}]", (dims[l + 1], dims[l])) for l, w in enumerate(dW)])
        dbp = (C.c_void_p * LP_MAX_LAYERS)(*[_dev_f32(b, f"db[{l}]", (dims[l + 1],)) for l, b in enumerate(db)])
    wp, wn = _workspace(workspace)
    _check(_lib.lp_splat_bwd(C.byref(target), C.byref(r), C.byref(s),
                             _ptr3(theta_w, _target_shapes(target, None), "theta_w"),
                             _ptr3(d_theta, _target_shapes(target, target.C), "d_theta"),
                             _dev_f32(d_feats, "d_feats", (m, n_in)), dp, dWp, dbp, wp, wn, _stream_ptr(stream)))
    del keep


# ---------------------------------------------------------------------------------------
# Conveniences on top of the entry points: move host buffers to the GPU, allocate outputs.

def to_device(inp, device="cuda:0"):
    """Upload host buffers (any object with the fields of `lp_inputs.Inputs`) and return
    (Grid, Mlp, Rays, bg) on `device`."""
    dev = torch.device(device)
    up = lambda a: torch.from_numpy(a).to(dev)
    grid = Grid(kind=int(inp.kind), data=[up(g) for g in inp.grid], res=tuple(inp.res),
                aabb_min=tuple(inp.aabb_min), aabb_max=tuple(inp.aabb_max),
                contract_a=float(getattr(inp, "contract_a", 0.0)), t_range=tuple(getattr(inp, "t_range", (0.0, 1.0))))
    mlp = Mlp(weights=[up(w) for w in inp.weights], biases=[up(b) for b in inp.biases])
    rays = Rays(origins=up(inp.origins), dirs=up(inp.dirs), near=up(inp.near), far=up(inp.far),
                samples=int(inp.samples), scene=None if inp.scene is None else up(inp.scene),
                time=None if getattr(inp, "time", None) is None else up(inp.time))
    return grid, mlp, rays, tuple(float(v) for v in inp.bg)


def decoder_to_device(dec, device="cuda:0") -> Decoder:
    """Upload a host decoder (fields of `lp_inputs.Decoder`)."""
    dev = torch.device(device)
    up = lambda a: torch.from_numpy(a).to(dev)
    return Decoder(opacity=Mlp([up(w) for w in dec.weights_s], [up(b) for b in dec.biases_s]),
                   feature=Mlp([up(w) for w in dec.weights_v], [up(b) for b in dec.biases_v]),
                   n_freq=int(dec.n_freq), n_feat=int(dec.n_feat), feat_act=int(dec.feat_act))


def render_dec_fwd(grid: Grid, dec: Decoder, rays: Rays, bg, math_mode: int = LP_MATH_DEFAULT):
    """Allocate outputs and workspace and run lp_render_dec_fwd.  Returns (out, alpha, depth, ray_cache)."""
    dev = rays.origins.device
    m = rays.n_rays
    out = torch.empty((m, dec.n_feat), dtype=torch.float32, device=dev)
    alpha = torch.empty((m,), dtype=torch.float32, device=dev)
    depth = torch.empty((m,), dtype=torch.float32, device=dev)
    cache = torch.empty((m,), dtype=torch.float32, device=dev)
    ws = torch.empty(lp_dec_workspace_bytes(grid, dec, rays, math_mode)[0], dtype=torch.uint8, device=dev)
    lp_render_dec_fwd(grid, dec, rays, bg, out, alpha, depth, cache, ws, math_mode)
    return out, alpha, depth, cache


def render_dec_bwd(grid: Grid, dec: Decoder, rays: Rays, bg, d_out, ray_cache, d_alpha=None, d_depth=None,
                   math_mode: int = LP_MATH_DEFAULT):
    """Allocate zeroed gradient buffers and a workspace and run lp_render_dec_bwd.
    Returns (d_grid, dW_opacity, db_opacity, dW_feature, db_feature)."""
    dev = rays.origins.device
    d_grid = [torch.zeros_like(t, dtype=torch.float32) for t in grid.data]   # gradients are float32 whatever the storage
    z = lambda lst: [torch.zeros_like(t) for t in lst]
    dWs, dbs, dWv, dbv = z(dec.opacity.weights), z(dec.opacity.biases), z(dec.feature.weights), z(dec.feature.biases)
    ws = torch.empty(lp_dec_workspace_bytes(grid, dec, rays, math_mode)[1], dtype=torch.uint8, device=dev)
    lp_render_dec_bwd(grid, dec, rays, bg, d_out, d_alpha, d_depth, ray_cache, d_grid, dWs, dbs, dWv, dbv, ws,
                      math_mode)
    return d_grid, dWs, dbs, dWv, dbv


def render_fwd(grid: Grid, mlp: Mlp, rays: Rays, bg, math_mode: int = LP_MATH_DEFAULT):
    """Allocate outputs and run lp_render_fwd.  Returns (rgb, alpha, depth, ray_cache)."""
    dev = rays.origins.device
    m = rays.n_rays
    rgb = torch.empty((m, 3), dtype=torch.float32, device=dev)
    alpha = torch.empty((m,), dtype=torch.float32, device=dev)
    depth = torch.empty((m,), dtype=torch.float32, device=dev)
    cache = torch.empty((m,), dtype=torch.float32, device=dev)
    lp_render_fwd(grid, mlp, rays, bg, rgb, alpha, depth, cache, math_mode)
    return rgb, alpha, depth, cache


def render_bwd(grid: Grid, mlp: Mlp, rays: Rays, bg, d_rgb, ray_cache, d_alpha=None, d_depth=None,
               math_mode: int = LP_MATH_DEFAULT, workspace: Optional[torch.Tensor] = None):
    """Allocate zeroed gradient buffers (and a workspace) and run lp_render_bwd.
    Returns (d_grid list, dW list, db list)."""
    dev = rays.origins.device
    d_grid = [torch.zeros_like(t, dtype=torch.float32) for t in grid.data]   # gradients are float32 whatever the storage
    dW = [torch.zeros_like(w) for w in mlp.weights]
    db = [torch.zeros_like(b) for b in mlp.biases]
    if workspace is None:
        workspace = torch.empty(lp_bwd_workspace_bytes(grid, mlp, rays, math_mode), dtype=torch.uint8, device=dev)
    lp_render_bwd(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, ray_cache, d_grid, dW, db, workspace, math_mode)
    return d_grid, dW, db


def splat_to_device(sp, device="cuda:0"):
    """Upload host buffers with the fields of `lp_inputs.SplatInputs`.  Returns (target, Rays, Splat)."""
    dev = torch.device(device)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    target = target_struct(sp.kind, sp.n_scenes, sp.channels, sp.res, sp.aabb_min, sp.aabb_max, sp.contract_a,
                           getattr(sp, "hash_size", 0))
    rays = Rays(origins=up(sp.origins), dirs=up(sp.dirs), near=up(sp.near), far=up(sp.far),
                samples=int(sp.samples), scene=None if sp.scene is None else up(sp.scene))
    prior = None
    if sp.prior is not None:
        prior = Grid(kind=int(sp.kind), data=[up(g) for g in sp.prior], res=tuple(sp.prior_res),
                     aabb_min=tuple(sp.aabb_min), aabb_max=tuple(sp.aabb_max), contract_a=float(sp.contract_a))
    mlp = None if sp.mlp_dims is None else Mlp([up(w) for w in sp.weights], [up(b) for b in sp.biases])
    return target, rays, Splat(feats=up(sp.feats), prior=prior, mlp=mlp, n_freq=int(sp.n_freq))


def splat_fwd(target: _Grid, rays: Rays, splat: Splat):
    """Allocate outputs and run lp_splat_fwd.  Returns (theta list, theta_w list)."""
    dev = rays.origins.device
    theta = [torch.empty(s, dtype=torch.float32, device=dev) for s in _target_shapes(target, target.C)]
    theta_w = [torch.empty(s, dtype=torch.float32, device=dev) for s in _target_shapes(target, None)]
    lp_splat_fwd(target, rays, splat, theta, theta_w)
    return theta, theta_w


def splat_bwd(target: _Grid, rays: Rays, splat: Splat, theta_w, d_theta):
    """Allocate gradient buffers and workspace and run lp_splat_bwd.
    Returns (d_feats, d_prior list, dW list, db list)."""
    dev = rays.origins.device
    d_feats = torch.empty_like(splat.feats)
    d_prior = [] if splat.prior is None else [torch.zeros_like(t) for t in splat.prior.data]
    dW = [] if splat.mlp is None else [torch.zeros_like(w) for w in splat.mlp.weights]
    db = [] if splat.mlp is None else [torch.zeros_like(b) for b in splat.mlp.biases]
    ws = torch.empty(lp_splat_bwd_workspace_bytes(target, rays, splat), dtype=torch.uint8, device=dev)
    lp_splat_bwd(target, rays, splat, theta_w, d_theta, d_feats, d_prior, dW, db, ws)
    return d_feats, d_prior, dW, db
