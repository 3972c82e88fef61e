"""torch.autograd wrapper around the Renderer's two entry points, for callers that train with
PyTorch optimisers: the forward keeps one scalar per ray (Section 3.4: the backward recomputes the
rest), the backward calls lp_render_bwd.  Argument marshalling only: every step of the path runs in the
library's kernels.  No gradient flows to the rays (the library produces none)."""
from typing import List, Optional, Sequence

import torch

from . import (LP_MATH_DEFAULT, Grid, Mlp, Rays, lp_bwd_workspace_bytes, lp_render_bwd, lp_render_fwd)


class _Render(torch.autograd.Function):
    @staticmethod
    def forward(ctx, spec, n_grid: int, n_layers: int, *tensors):
        kind, res, aabb_min, aabb_max, contract_a, t_range, rays, bg, math_mode = spec
        data = [t.detach() for t in tensors[:n_grid]]
        weights = [t.detach() for t in tensors[n_grid:n_grid + n_layers]]
        biases = [t.detach() for t in tensors[n_grid + n_layers:]]
        grid = Grid(kind=kind, data=data, res=res, aabb_min=aabb_min, aabb_max=aabb_max, contract_a=contract_a,
                    t_range=t_range)
        mlp = Mlp(weights=weights, biases=biases)
        m, dev = rays.n_rays, rays.origins.device
        rgb = torch.empty((m, 3), dtype=torch.float32, device=dev)
        alpha = torch.empty((m,), dtype=torch.float32, device=dev)
        depth = torch.empty((m,), dtype=torch.float32, device=dev)
        cache = torch.empty((m,), dtype=torch.float32, device=dev)
        lp_render_fwd(grid, mlp, rays, bg, rgb, alpha, depth, cache, math_mode)
        ctx.lp = (grid, mlp, rays, bg, math_mode, cache)
        ctx.mark_non_differentiable(cache)
        return rgb, alpha, depth

    @staticmethod
    def backward(ctx, d_rgb, d_alpha, d_depth):
        grid, mlp, rays, bg, math_mode, cache = ctx.lp
        dev = rays.origins.device
        d_grid = [torch.zeros_like(t, dtype=torch.float32) for t in grid.data]
        dW = [torch.zeros_like(w) for w in mlp.weights]
        db = [torch.zeros_like(b) for b in mlp.biases]
        ws = torch.empty(lp_bwd_workspace_bytes(grid, mlp, rays, math_mode), dtype=torch.uint8, device=dev)
        as_f32 = lambda t: None if t is None else t.contiguous().float()
        lp_render_bwd(grid, mlp, rays, bg, as_f32(d_rgb), as_f32(d_alpha), as_f32(d_depth), cache, d_grid, dW, db, ws,
                      math_mode)
        # gradients of structures stored in reduced precision come back in that type
        d_grid = [g.to(t.dtype) for g, t in zip(d_grid, grid.data)]
        return (None, None, None, *d_grid, *dW, *db)


def render(grid: Grid, mlp: Mlp, rays: Rays, bg: Sequence[float], math_mode: int = LP_MATH_DEFAULT):
    """Differentiable Renderer: returns (rgb [M][3], alpha [M], depth [M]); gradients flow to
    grid.data, mlp.weights and mlp.biases (tensors with requires_grad)."""
    spec = (grid.kind, tuple(grid.res), tuple(grid.aabb_min), tuple(grid.aabb_max), float(grid.contract_a),
            tuple(grid.t_range), rays, tuple(float(v) for v in bg), int(math_mode))
    return _Render.apply(spec, len(grid.data), len(mlp.weights), *grid.data, *mlp.weights, *mlp.biases)
