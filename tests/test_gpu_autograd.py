"""The torch.autograd wrapper hands the library's gradients to PyTorch unchanged, and a few optimiser
steps on a synthetic fitting problem reduce the loss (a training loop through the C ABI)."""
import numpy as np
import pytest

import lp_inputs
from lp_inputs import TRIPLANE, VOXEL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,channels,dims", [(VOXEL, 16, (16, 64, 64, 4)), (TRIPLANE, 5, (5, 7, 4))])
def test_autograd_gradients_are_the_librarys(lp, kind, channels, dims):
    import torch
    from paper_2404_19760_amd import autograd as lpa
    inp = lp_inputs.make_small(kind, n_scenes=2, channels=channels, res=(12, 10, 11), mlp_dims=dims, n_rays=150,
                               samples=48, seed=301, grid_std=0.3)
    grid, mlp, rays, bg = lp.to_device(inp)
    for t in grid.data + mlp.weights + mlp.biases:
        t.requires_grad_(True)
    rgb, alpha, depth = lpa.render(grid, mlp, rays, bg)
    target = torch.from_numpy(inp.target).to(rgb.device)
    rng = np.random.default_rng(5)
    pa = torch.from_numpy(rng.standard_normal(inp.n_rays).astype(np.float32)).to(rgb.device)
    pd = torch.from_numpy(rng.standard_normal(inp.n_rays).astype(np.float32)).to(rgb.device)
    loss = ((rgb - target) ** 2).mean() + (pa * alpha).mean() + (pd * depth).mean()
    loss.backward()
    # the same upstream gradients through the plain binding
    d_rgb = (2.0 * (rgb.detach() - target) / rgb.numel()).contiguous()
    with torch.no_grad():
        out = lp.render_fwd(grid, mlp, rays, bg)
        ref = lp.render_bwd(grid, mlp, rays, bg, d_rgb, out[3], d_alpha=pa / inp.n_rays, d_depth=pd / inp.n_rays)
    got = [t.grad for t in grid.data], [t.grad for t in mlp.weights], [t.grad for t in mlp.biases]
    for a_list, b_list in zip(got, ref):
        for a, b in zip(a_list, b_list):
            # (atomic adds: equal up to the order of the sums)
            assert float((a.double() - b.double()).norm() / b.double().norm().clamp_min(1e-30)) < 1e-5


def test_a_few_optimiser_steps_reduce_the_loss(lp):
    import torch
    from paper_2404_19760_amd import autograd as lpa
    inp = lp_inputs.make_small(VOXEL, channels=16, res=(16, 16, 16), mlp_dims=(16, 32, 4), n_rays=600, samples=40,
                               seed=303, grid_std=0.1, bias_std=0.0)
    grid, mlp, rays, bg = lp.to_device(inp)
    params = grid.data + mlp.weights + mlp.biases
    for t in params:
        t.requires_grad_(True)
    target = torch.from_numpy(inp.target).to(rays.origins.device)
    opt = torch.optim.Adam(params, lr=3e-2)
    losses = []
    for _ in range(25):
        opt.zero_grad()
        rgb, _, _ = lpa.render(grid, mlp, rays, bg)
        loss = ((rgb - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.7 * losses[0], losses
