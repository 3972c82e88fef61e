"""GPU parity of the hash-table structure (Section 3.2 names hash tables among the structures h; the
reading -- the spatial hash of Teschner et al. 2003 with Instant-NGP's primes, trilinear over a
virtual lattice -- is pinned on the CPU in test_oracle_hash.py).  The generic kernels serve it:
forward outputs and every gradient tensor against the CPU oracle, with tables small enough that most
lattice corners collide and large enough that few do, several scenes, contract coordinates, a table
stored in bf16, the two-MLP decoder; and the calls that must refuse it."""
import dataclasses

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HASH

from parity import check_case, check_case_dec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


@pytest.mark.parametrize("hash_size", [1, 37, 4096, 250007])
@pytest.mark.parametrize("contract", [0.0, 1.3])
def test_hash_table_renderer(lp, oracle, hash_size, contract):
    kw = dict(origin_radius=0.8, near=(0.0, 0.3), far=(4.0, 9.0)) if contract else {}
    inp = lp_inputs.make_small(HASH, n_scenes=2, channels=8, res=(24, 19, 21), mlp_dims=(8, 16, 12, 4), n_rays=203,
                               samples=70, seed=151 + hash_size % 7, grid_std=0.4, hash_size=hash_size, **kw)
    inp = dataclasses.replace(inp, contract_a=contract)
    grid, mlp, _, _ = lp.to_device(inp)
    assert not lp.lp_has_fast_path(grid, mlp)        # generic kernels
    # (a table of a few entries collects the kink decisions of every sample in each of them)
    print(check_case(lp, oracle, inp, lp.LP_MATH_DEFAULT, label=f"hash T={hash_size} contract={contract}",
                     max_strict_fail=0.25 if hash_size < 100 else 0.02), flush=True)


def test_hash_table_with_matrix_core_shapes_runs_on_the_generic_kernels(lp, oracle):
    """16 channels and a 16-64-64-4 MLP would be a matrix-core shape for a voxel grid; a hash table of
    the same shape is served by the generic kernels, and asking for the matrix-core mode is refused."""
    inp = lp_inputs.make_small(HASH, channels=16, res=(20, 20, 20), mlp_dims=(16, 64, 64, 4), n_rays=150, samples=48,
                               seed=157, grid_std=0.3, hash_size=8191)
    grid, mlp, rays, bg = lp.to_device(inp)
    assert not lp.lp_has_fast_path(grid, mlp)
    print(check_case(lp, oracle, inp, lp.LP_MATH_DEFAULT, label="hash 16ch"), flush=True)
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_fwd(grid, mlp, rays, bg, lp.LP_MATH_BF16X3)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED


def test_hash_table_stored_in_bf16(lp, oracle):
    import torch
    inp = lp_inputs.make_small(HASH, channels=8, res=(24, 19, 21), mlp_dims=(8, 16, 4), n_rays=203, samples=70,
                               seed=163, grid_std=0.4, hash_size=4096)
    stored = [torch.from_numpy(g).to(torch.bfloat16) for g in inp.grid]
    widened = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored])
    print(check_case(lp, oracle, widened, lp.LP_MATH_DEFAULT, label="hash bf16", grid_dtype=torch.bfloat16), flush=True)


def test_hash_table_under_the_two_mlp_decoder(lp, oracle):
    inp = lp_inputs.make_small(HASH, n_scenes=2, channels=6, res=(16, 14, 15), mlp_dims=(6, 4), n_rays=131, samples=37,
                               seed=167, grid_std=0.4, hash_size=2048)
    dec = lp_inputs.make_decoder(6, (8,), (9, 7), 1, 3, 168, 0.2, 0)
    rng = np.random.default_rng(169)
    inp = dataclasses.replace(inp, decoder=dec, bg=tuple(rng.random(3).astype(np.float32).tolist()),
                              target=rng.random((inp.n_rays, 3), dtype=np.float32))
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_DEFAULT, label="hash decoder"), flush=True)


def test_hash_table_arguments(lp):
    import ctypes as C
    inp = lp_inputs.make_small(HASH, channels=4, res=(6, 5, 7), mlp_dims=(4, 8, 4), n_rays=9, samples=5, seed=173,
                               hash_size=64)
    grid, mlp, rays, bg = lp.to_device(inp)
    g, m, r = grid.c_struct(), mlp.c_struct(), rays.c_struct()
    assert g.kind == lp.LP_GRID_HASH and g.hash_size == 64
    g.hash_size = 0
    st = lp._lib.lp_render_fwd(C.byref(g), C.byref(m), C.byref(r), (C.c_float * 3)(*bg), None, None, None, None, 0, None)
    assert st == lp.LP_ERR_INVALID_ARG and b"hash_size" in lp._lib.lp_last_error()
