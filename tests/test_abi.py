"""The C-ABI library loads and exports every function include/*.h declares; argument
errors are reported as statuses before anything touches a GPU.  CPU only."""
import ctypes as C
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2404_19760_amd", "liblightplane.so")


def declared_functions():
    names = []
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        src = open(h).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(lp_[a-z_0-9]+)\s*\(", src)
    return sorted(set(names))


def test_header_declares_the_entry_points():
    names = declared_functions()
    for required in ("lp_render_fwd", "lp_render_bwd", "lp_bwd_workspace_bytes", "lp_last_error"):
        assert required in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build the library first: python -m paper_2404_19760_amd.build"
    lib = C.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported"


def test_invalid_arguments_are_statuses_not_crashes():
    import paper_2404_19760_amd as lp
    lib = lp._lib
    assert lp.lp_version() >= 1000
    st = lib.lp_render_fwd(None, None, None, None, None, None, None, None, 0, None)
    assert st == lp.LP_ERR_INVALID_ARG
    assert b"NULL" in lib.lp_last_error()
    g = lp._Grid(); m = lp._Mlp(); r = lp._Rays()
    g.kind, g.B, g.C, g.NX, g.NY, g.NZ = 0, 1, 4, 1, 8, 8      # NX < 2
    g.data[0] = 4096
    for a in range(3):
        g.aabb_min[a], g.aabb_max[a] = -1.0, 1.0
    bg = (C.c_float * 3)(1, 1, 1)
    st = lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), bg, None, None, None, None, 0, None)
    assert st == lp.LP_ERR_INVALID_ARG and b"resolution" in lib.lp_last_error()
    g.NX = 8
    m.n_layers = 1; m.dims[0] = 4; m.dims[1] = 3                # last layer must have 4 outputs
    m.W[0] = 4096; m.b[0] = 4096
    r.M, r.S = 0, 4
    st = lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), bg, None, None, None, None, 0, None)
    assert st == lp.LP_ERR_INVALID_ARG and b"4 outputs" in lib.lp_last_error()
    m.dims[1] = 4
    r.S = 0
    st = lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), bg, None, None, None, None, 0, None)
    assert st == lp.LP_ERR_INVALID_ARG and b"rays->S" in lib.lp_last_error()
    r.S = 4
    st = lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), bg, None, None, None, None, 99, None)
    assert st == lp.LP_ERR_INVALID_ARG and b"math_mode" in lib.lp_last_error()
    # M == 0 with valid shapes is a successful no-op and needs no GPU
    st = lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), bg, None, None, None, None, 0, None)
    assert st == lp.LP_OK


def test_fast_path_queries_are_host_logic():
    """Which shapes the matrix-core / wavefront-per-ray kernels cover is decided on the host from
    the argument structs alone (the device pointers are only checked for NULL and alignment)."""
    import paper_2404_19760_amd as lp
    lib = lp._lib

    def grid(kind, channels, res=(8, 8, 8), contract=0.0, dtype=None, hash_size=0, n_time=0):
        g = lp._Grid()
        g.kind, g.B, g.C = kind, 1, channels
        g.NX, g.NY, g.NZ = res
        for p in range(3):
            g.data[p] = 4096
            g.data_t[p] = 4096 if n_time else None
            g.aabb_min[p], g.aabb_max[p] = -1.0, 1.0
        g.contract_a = contract
        g.dtype = lp.LP_F32 if dtype is None else dtype
        g.hash_size = hash_size
        g.NT, g.t_min, g.t_max = n_time, 0.0, 1.0
        return g

    def mlp(*dims):
        m = lp._Mlp()
        m.n_layers = len(dims) - 1
        for i, d in enumerate(dims):
            m.dims[i] = d
        for l in range(m.n_layers):
            m.W[l] = 4096
            m.b[l] = 4096
        return m

    render = lambda g, m: lib.lp_has_fast_path(C.byref(g), C.byref(m))
    assert render(grid(0, 16), mlp(16, 64, 64, 4)) == 1
    assert render(grid(1, 32), mlp(32, 64, 4)) == 1
    assert render(grid(0, 16, contract=1.0), mlp(16, 32, 4)) == 1
    assert render(grid(0, 16, contract=1.0, dtype=lp.LP_BF16), mlp(16, 64, 64, 4)) == 1   # reduced-precision storage too
    assert render(grid(1, 32, dtype=lp.LP_F16), mlp(32, 64, 4)) == 1
    assert render(grid(0, 24), mlp(24, 64, 4)) == 0          # 16 or 32 channels
    assert render(grid(0, 16), mlp(16, 48, 4)) == 0          # hidden width 32 or 64
    assert render(grid(0, 16), mlp(16, 64, 32, 4)) == 0      # equal hidden widths
    assert render(grid(0, 16), mlp(16, 64, 64, 64, 4)) == 0  # at most two hidden layers
    # hash tables: a size that is a power of two; HexPlanes: 16 or 32 channels
    assert render(grid(lp.LP_GRID_HASH, 16, hash_size=1 << 14), mlp(16, 64, 64, 4)) == 1
    assert render(grid(lp.LP_GRID_HASH, 32, hash_size=4096, contract=1.0, dtype=lp.LP_BF16), mlp(32, 32, 4)) == 1
    assert render(grid(lp.LP_GRID_HASH, 16, hash_size=1), mlp(16, 32, 4)) == 1
    assert render(grid(lp.LP_GRID_HASH, 16, hash_size=12289), mlp(16, 64, 64, 4)) == 0
    assert render(grid(lp.LP_GRID_HASH, 8, hash_size=4096), mlp(8, 64, 4)) == 0
    assert render(grid(lp.LP_GRID_HASH, 16, hash_size=0), mlp(16, 64, 4)) == 0       # invalid: no fast path either
    assert render(grid(lp.LP_GRID_HEXPLANE, 16, n_time=5), mlp(16, 64, 64, 4)) == 1
    assert render(grid(lp.LP_GRID_HEXPLANE, 32, n_time=2, contract=1.0, dtype=lp.LP_F16), mlp(32, 32, 4)) == 1
    assert render(grid(lp.LP_GRID_HEXPLANE, 8, n_time=5), mlp(8, 64, 4)) == 0
    assert render(grid(lp.LP_GRID_HEXPLANE, 16, n_time=1), mlp(16, 64, 4)) == 0      # invalid: a time axis has two entries at least

    def decoder(g, dims_s, dims_v, n_freq, n_feat=3, feat_act=0):
        d = lp._Decoder()
        d.opacity, d.feature = mlp(*dims_s), mlp(*dims_v)
        d.n_freq, d.n_feat, d.feat_act = n_freq, n_feat, feat_act
        return lib.lp_dec_has_fast_path(C.byref(g), C.byref(d))

    assert decoder(grid(0, 16), (16, 32, 32, 1), (31, 32, 32, 3), 2) == 1     # merged into one 64-wide MLP
    assert decoder(grid(1, 32), (32, 64, 64, 1), (47, 64, 64, 3), 2) == 1     # the paper's size: two chains
    assert decoder(grid(0, 16, contract=1.0), (16, 64, 64, 1), (19, 64, 64, 3), 0) == 1
    assert decoder(grid(0, 32), (32, 64, 64, 1), (59, 64, 64, 3), 4) == 1     # any number of octaves
    assert decoder(grid(0, 16, dtype=lp.LP_BF16), (16, 32, 32, 1), (31, 32, 32, 3), 2) == 1   # grids in bf16 / fp16 too
    assert decoder(grid(0, 32, contract=1.0, dtype=lp.LP_F16), (32, 64, 64, 1), (47, 64, 64, 3), 2) == 1
    assert decoder(grid(0, 32), (32, 64, 64, 1), (47, 64, 64, 3), 2, feat_act=1) == 1   # identity features too
    assert decoder(grid(0, 16), (16, 32, 32, 1), (31, 32, 32, 3), 2, feat_act=1) == 1
    assert decoder(grid(0, 16), (16, 16, 16, 1), (37, 48, 48, 3), 3) == 0     # merged: at most 16 direction inputs
    assert decoder(grid(0, 32), (32, 64, 1), (47, 64, 64, 3), 2) == 0         # two chains: both 3-layer
    assert decoder(grid(0, 32), (32, 64, 64, 1), (47, 64, 64, 4), 2, n_feat=4) == 0
    assert decoder(grid(0, 24), (24, 64, 64, 1), (39, 64, 64, 3), 2) == 0
    # hash tables and HexPlanes: the merged decoder (16 channels + direction inputs), not the two chains
    assert decoder(grid(lp.LP_GRID_HASH, 16, hash_size=4096), (16, 32, 32, 1), (31, 32, 32, 3), 2) == 1
    assert decoder(grid(lp.LP_GRID_HEXPLANE, 16, n_time=4), (16, 32, 32, 1), (31, 32, 32, 3), 2) == 1
    assert decoder(grid(lp.LP_GRID_HASH, 32, hash_size=4096), (32, 64, 64, 1), (47, 64, 64, 3), 2) == 0
    assert decoder(grid(lp.LP_GRID_HEXPLANE, 32, n_time=4), (32, 64, 64, 1), (47, 64, 64, 3), 2) == 0

    def splat(target, n_in, n_freq=-1, prior=None, m=None):
        s = lp._Splat()
        s.n_in, s.n_freq, s.feats = n_in, n_freq, 4096
        s.prior = C.pointer(prior) if prior is not None else None
        s.mlp = C.pointer(m) if m is not None else None
        return lib.lp_splat_has_fast_path(C.byref(target), C.byref(s))

    assert splat(grid(0, 32), 32) == 1                                                   # naive, 32 channels
    assert splat(grid(1, 16), 16) == 1
    assert splat(grid(0, 8), 8) == 0
    assert splat(grid(lp.LP_GRID_HASH, 32, hash_size=4096), 32) == 1                     # naive, a table of a power-of-two size
    assert splat(grid(lp.LP_GRID_HASH, 32, hash_size=4097), 32) == 0
    assert splat(grid(lp.LP_GRID_HASH, 32, hash_size=4096), 32, 0, grid(lp.LP_GRID_HASH, 32, hash_size=4096), mlp(67, 64, 64, 32)) == 0   # with an MLP: generic
    assert splat(grid(lp.LP_GRID_HEXPLANE, 32, n_time=4), 32) == 0
    assert splat(grid(0, 32), 32, 0, grid(0, 32, (5, 6, 7)), mlp(67, 64, 64, 32)) == 1   # the paper's MLP
    assert splat(grid(1, 16), 20, 1, grid(1, 16), mlp(45, 64, 16)) == 1
    assert splat(grid(0, 32), 32, 0, grid(0, 32), mlp(67, 64, 60, 32)) == 0              # hidden width 64 only
    assert splat(grid(0, 32), 32, 0, grid(0, 16), mlp(51, 64, 32)) == 0                  # prior and target alike
    assert splat(grid(0, 32), 46, 0, grid(0, 32), mlp(81, 64, 32)) == 0                  # at most 48 per-ray inputs
    assert splat(grid(0, 32, contract=1.0), 32, 0, grid(0, 32, contract=1.0), mlp(67, 64, 32)) == 1
    assert splat(grid(0, 32, contract=1.0), 32, 0, grid(0, 32), mlp(67, 64, 32)) == 0      # prior without the target's contraction
    assert splat(grid(0, 32), 32, 0, None, mlp(35, 64, 32)) == 0                         # needs a prior
    assert splat(grid(0, 32), 30, 0, grid(0, 32), mlp(67, 64, 32)) == 0                  # inconsistent widths


def test_product_path_does_not_reach_the_oracle():
    """Nothing under the package names, imports or links the oracle."""
    pkg = os.path.join(ROOT, "paper_2404_19760_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
