"""GPU parity of the HexPlane structure (Section 3.2 names HexPlane among the structures h; the
reading -- six planes in three complementary pairs, the reads of a pair multiplied, the three
products added, a time per ray -- is pinned on the CPU in test_oracle_hexplane.py).  The generic
and -- for 16 or 32 channels -- the matrix-core kernels serve it: forward outputs and the gradients of
all six planes and of the MLP against the CPU oracle, with several scenes, contract coordinates, times
beyond both ends of the range, planes stored in reduced precision, no times given, the two-MLP
decoder; and the calls that must refuse it."""
import ctypes as C
import dataclasses

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HEXPLANE

from parity import check_case, check_case_dec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


@pytest.mark.parametrize("n_time", [2, 7])
@pytest.mark.parametrize("contract", [0.0, 1.3])
def test_hexplane_renderer(lp, oracle, n_time, contract):
    kw = dict(origin_radius=0.8, near=(0.0, 0.3), far=(4.0, 9.0)) if contract else {}
    inp = lp_inputs.make_small(HEXPLANE, n_scenes=2, channels=8, res=(24, 19, 21), mlp_dims=(8, 16, 12, 4), n_rays=203,
                               samples=70, seed=181 + n_time, grid_std=0.4, n_time=n_time, t_range=(-0.5, 1.5), **kw)
    inp = dataclasses.replace(inp, contract_a=contract)
    assert (inp.time < -0.5).any() and (inp.time > 1.5).any()      # times clamp at both ends
    grid, mlp, _, _ = lp.to_device(inp)
    assert len(grid.data) == 6 and not lp.lp_has_fast_path(grid, mlp)
    worst = check_case(lp, oracle, inp, lp.LP_MATH_DEFAULT, label=f"hexplane NT={n_time} contract={contract}")
    assert all(f"d_grid{p}" in worst for p in range(6))
    print(worst, flush=True)


MATRIX_CORE_CASES = [
    # channels, MLP, time resolution, contract, stored as, times given
    (16, (16, 64, 64, 4), 4, 0.0, None, True),
    (16, (16, 32, 4), 2, 1.3, None, True),
    (16, (16, 64, 4), 5, 0.0, "bfloat16", True),
    (16, (16, 32, 32, 4), 3, 0.0, None, False),
    (32, (32, 64, 64, 4), 4, 1.3, None, True),
    (32, (32, 32, 4), 6, 0.0, "float16", True),
    (32, (32, 64, 4), 3, 0.0, None, True),
]


@pytest.mark.parametrize("channels,dims,n_time,contract,stored,timed", MATRIX_CORE_CASES)
def test_hexplane_on_the_matrix_cores(lp, oracle, channels, dims, n_time, contract, stored, timed):
    """Both arithmetic modes on the shapes the matrix-core kernels cover (16 or 32 channels): several
    scenes, more samples than two 32-sample backward steps with a ragged tail, more rays than one wave
    per workgroup, times beyond both ends of the range."""
    import torch
    kw = dict(origin_radius=0.8, near=(0.0, 0.3), far=(4.0, 9.0)) if contract else {}
    inp = lp_inputs.make_small(HEXPLANE, n_scenes=2, channels=channels, res=(24, 19, 21), mlp_dims=dims, n_rays=157,
                               samples=83, seed=223 + channels + len(dims) + n_time, grid_std=0.3, n_time=n_time,
                               t_range=(-0.5, 1.5), **kw)
    inp = dataclasses.replace(inp, contract_a=contract, time=inp.time if timed else None)
    dtype = None
    if stored:
        dtype = getattr(torch, stored)
        kept = [torch.from_numpy(g).to(dtype) for g in inp.grid]
        inp = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in kept])
    grid, mlp, _, _ = lp.to_device(inp)
    assert lp.lp_has_fast_path(grid, mlp)
    for mode in (lp.LP_MATH_GENERIC, lp.LP_MATH_BF16X3):
        print(check_case(lp, oracle, inp, mode, label=f"hexplane {channels}ch {dims} NT={n_time} mode={mode}",
                         max_strict_fail=0.05, grid_dtype=dtype), flush=True)   # (the space-time planes have few
        # hundred to few thousand elements: the share of elements that need the kink envelope is a noisy figure there)


def test_hexplane_stored_in_bf16_and_without_times(lp, oracle):
    import torch
    inp = lp_inputs.make_small(HEXPLANE, channels=8, res=(24, 19, 21), mlp_dims=(8, 16, 4), n_rays=203, samples=70,
                               seed=193, grid_std=0.4, n_time=5)
    stored = [torch.from_numpy(g).to(torch.bfloat16) for g in inp.grid]
    widened = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored])
    print(check_case(lp, oracle, widened, lp.LP_MATH_DEFAULT, label="hexplane bf16", grid_dtype=torch.bfloat16), flush=True)
    print(check_case(lp, oracle, dataclasses.replace(inp, time=None), lp.LP_MATH_DEFAULT, label="hexplane no times"), flush=True)


def test_hexplane_under_the_two_mlp_decoder(lp, oracle):
    inp = lp_inputs.make_small(HEXPLANE, n_scenes=2, channels=6, res=(16, 14, 15), mlp_dims=(6, 4), n_rays=131, samples=37,
                               seed=197, grid_std=0.4, n_time=3)
    dec = lp_inputs.make_decoder(6, (8,), (9, 7), 1, 3, 198, 0.2, 0)
    rng = np.random.default_rng(199)
    inp = dataclasses.replace(inp, decoder=dec, bg=tuple(rng.random(3).astype(np.float32).tolist()),
                              target=rng.random((inp.n_rays, 3), dtype=np.float32))
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_DEFAULT, label="hexplane decoder"), flush=True)


def test_hexplane_arguments(lp):
    inp = lp_inputs.make_small(HEXPLANE, channels=4, res=(6, 5, 7), mlp_dims=(4, 8, 4), n_rays=9, samples=5, seed=211,
                               n_time=3, t_range=(1.0, 2.0))
    grid, mlp, rays, bg = lp.to_device(inp)
    g, m, r = grid.c_struct(), mlp.c_struct(), rays.c_struct()
    assert g.kind == lp.LP_GRID_HEXPLANE and g.NT == 3 and (g.t_min, g.t_max) == (1.0, 2.0)

    def fwd(gs):
        return lp._lib.lp_render_fwd(C.byref(gs), C.byref(m), C.byref(r), (C.c_float * 3)(*bg), None, None, None, None, 0, None)

    bad = grid.c_struct(); bad.NT = 1
    assert fwd(bad) == lp.LP_ERR_INVALID_ARG and b"NT" in lp._lib.lp_last_error()
    bad = grid.c_struct(); bad.t_max = bad.t_min
    assert fwd(bad) == lp.LP_ERR_INVALID_ARG and b"t_max" in lp._lib.lp_last_error()
    bad = grid.c_struct(); bad.data_t[1] = None
    assert fwd(bad) == lp.LP_ERR_INVALID_ARG and b"data_t" in lp._lib.lp_last_error()
