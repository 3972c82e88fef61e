"""The backward entry point that allocates nothing (lp_render_bwd_static): same results as
lp_render_bwd, on two calls in a row that share the library's static device scratch, the second
with a smaller input; and the refusal of a shape whose records do not fit."""
import numpy as np
import pytest
import torch

import lp_inputs
from lp_inputs import TRIPLANE, VOXEL

from parity import BWD_RTOL, close

pytestmark = pytest.mark.gpu


def _both(lp, inp, mode):
    grid, mlp, rays, bg = lp.to_device(inp)
    rgb, alpha, depth, cache = lp.render_fwd(grid, mlp, rays, bg, mode)
    rng = np.random.default_rng(3)
    m = inp.n_rays
    up = lambda a: torch.from_numpy(a.astype(np.float32)).to("cuda:0")
    d_rgb, d_alpha, d_depth = up(rng.standard_normal((m, 3)) / m), up(rng.standard_normal(m) / m), up(rng.standard_normal(m) / m)
    ref = lp.render_bwd(grid, mlp, rays, bg, d_rgb, cache, d_alpha, d_depth, mode)
    d_grid = [torch.zeros_like(t, dtype=torch.float32) for t in grid.data]
    dW = [torch.zeros_like(w) for w in mlp.weights]
    db = [torch.zeros_like(b) for b in mlp.biases]
    # no allocation request reaches torch's allocator during the call (frees of earlier tensors by
    # the garbage collector do not count: this is the number of allocation events)
    events = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    before = events()
    lp.lp_render_bwd_static(grid, mlp, rays, bg, d_rgb, d_alpha, d_depth, cache, d_grid, dW, db, mode)
    torch.cuda.synchronize()
    assert events() == before
    return ref, (d_grid, dW, db)


def _compare(ref, got, label):
    for name, a, b in zip(("d_grid", "dW", "db"), ref, got):
        for l, (x, y) in enumerate(zip(a, b)):
            x, y = x.cpu().numpy(), y.cpu().numpy()
            if name == "d_grid":   # summed with atomics: equal up to summation order
                close(y, x, BWD_RTOL * 1e-2, f"{label} {name}[{l}]")
            else:                  # the records are added in a fixed order: bit for bit
                assert np.array_equal(x, y), f"{label} {name}[{l}] differs from lp_render_bwd"


@pytest.mark.parametrize("kind,channels,dims,mode_name", [
    (VOXEL, 16, (16, 64, 64, 4), "LP_MATH_BF16X3"), (TRIPLANE, 32, (32, 64, 64, 4), "LP_MATH_BF16X3"),
    (VOXEL, 5, (5, 7, 9, 4), "LP_MATH_GENERIC")])
def test_static_scratch_backward_matches_the_workspace_backward(lp, kind, channels, dims, mode_name):
    mode = getattr(lp, mode_name)
    big = lp_inputs.make_small(kind, channels=channels, res=(12, 10, 11), mlp_dims=dims, n_rays=2500, samples=70,
                               seed=141, n_scenes=2, grid_std=0.3, aabb_min=(-1.5,) * 3, aabb_max=(1.5,) * 3)
    small = lp_inputs.make_small(kind, channels=channels, res=(7, 6, 5), mlp_dims=dims, n_rays=37, samples=33,
                                 seed=142, grid_std=0.3)
    for label, inp in (("first call", big), ("second, smaller call", small)):
        ref, got = _both(lp, inp, mode)
        _compare(ref, got, f"{label} kind={kind}")


def test_static_scratch_refuses_what_does_not_fit(lp):
    """An MLP whose per-block records exceed the static scratch is refused with a clear message."""
    inp = lp_inputs.make_small(VOXEL, channels=24, res=(6, 5, 7), mlp_dims=(24, 96, 96, 4), n_rays=9, samples=5, seed=143)
    grid, mlp, rays, bg = lp.to_device(inp)
    need = lp.lp_bwd_workspace_bytes(grid, mlp, rays, lp.LP_MATH_GENERIC)
    assert need > lp.LP_STATIC_SCRATCH_BYTES
    _, _, _, cache = lp.render_fwd(grid, mlp, rays, bg, lp.LP_MATH_GENERIC)
    d_rgb = torch.zeros((9, 3), device="cuda:0")
    d_grid = [torch.zeros_like(t) for t in grid.data]
    dW = [torch.zeros_like(w) for w in mlp.weights]
    db = [torch.zeros_like(b) for b in mlp.biases]
    with pytest.raises(lp.LightplaneError) as e:
        lp.lp_render_bwd_static(grid, mlp, rays, bg, d_rgb, None, None, cache, d_grid, dW, db, lp.LP_MATH_GENERIC)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED and "LP_STATIC_SCRATCH_BYTES" in str(e.value)
    assert all(float(t.abs().max()) == 0.0 for t in d_grid + dW + db)
