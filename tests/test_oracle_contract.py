"""Pins of the oracle's contract coordinates (appendix "Experimental Details", equation CC)
against what the paper and the mathematics fix: hand-worked values, the stated foreground
range, the limit at infinity, the reduction to the standard contraction at a = 1, a pure
re-parametrisation, and finite differences of the full gradient."""
import dataclasses
import os

import numpy as np
import pytest

import lp_inputs
import oracle
from lp_inputs import TRIPLANE, VOXEL

from test_oracle_pins import _feat_of_points, _loss64

HERE = os.path.dirname(os.path.abspath(__file__))


def _axis_probe(kind, a_scale, axis):
    """A problem whose channel 0 is exactly the (contracted) coordinate along `axis`: the grid
    holds the affine field y_axis over the cube [-1, 1]^3, which interpolation reproduces."""
    res = (5, 4, 6)
    inp = lp_inputs.make_small(kind, res=res, channels=1, mlp_dims=(1, 4))
    ax = [np.linspace(-1.0, 1.0, n) for n in res]
    if kind == VOXEL:
        g = np.zeros(res + (1,))
        shape = [1, 1, 1, 1]
        shape[axis] = res[axis]
        g[...] = ax[axis].reshape(shape)
        grids = [g[None]]
    else:
        # planes (x,y), (y,z), (z,x): put the coordinate on the first plane that has the axis
        pairs = [(0, 1), (1, 2), (2, 0)]
        grids = []
        used = False
        for (pa, pb) in pairs:
            g = np.zeros((res[pa], res[pb], 1))
            if not used and axis in (pa, pb):
                if axis == pa:
                    g[...] = ax[axis].reshape(-1, 1, 1)
                else:
                    g[...] = ax[axis].reshape(1, -1, 1)
                used = True
            grids.append(g[None])
    return dataclasses.replace(inp, grid=[np.ascontiguousarray(x) for x in grids], contract_a=a_scale)


def _cc(kind, a_scale, xs, axis=0):
    """CC(x) as the oracle applies it, read back through an affine grid."""
    inp = _axis_probe(kind, a_scale, axis)
    pts = np.zeros((len(xs), 3))
    pts[:, axis] = xs
    # the other axes sit somewhere harmless but different
    pts[:, (axis + 1) % 3] = 0.3
    pts[:, (axis + 2) % 3] = -7.0
    return _feat_of_points(inp, pts)[:, 0]


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_contract_matches_hand_worked_values(kind):
    rows = np.loadtxt(os.path.join(HERE, "golden", "contract_values.txt"))
    for a_scale in np.unique(rows[:, 0]):
        sel = rows[rows[:, 0] == a_scale]
        for axis in range(3):
            got = _cc(kind, float(a_scale), sel[:, 1], axis)
            np.testing.assert_allclose(got, sel[:, 2], rtol=0, atol=1e-12)


def test_contract_properties():
    """Odd, strictly increasing, continuous at |x| = 1, foreground [-1, 1] -> [-a/2, a/2],
    limit +-1 at infinity (the unbounded scene lands inside the [-1, 1] cube)."""
    for a_scale in (0.5, 1.0, 1.7):
        xs = np.array([-1e9, -50.0, -3.0, -1.0 - 1e-6, -1.0, -0.999999, -0.2, 0.0, 0.2, 0.999999, 1.0,
                       1.0 + 1e-6, 3.0, 50.0, 1e9]).astype(np.float32).astype(np.float64)
        y = _cc(VOXEL, a_scale, xs)
        np.testing.assert_allclose(y, -y[::-1], atol=1e-15)
        assert np.all(np.diff(y) > 0)
        assert abs(y[np.argmin(abs(xs - 1.0))] - 0.5 * np.float32(a_scale)) < 1e-12
        assert abs(y[-4] - y[-5]) < 2e-6 and abs(y[-6] - y[-5]) < 2e-6      # continuity at 1
        assert np.all(np.abs(y) < 1.0) and 1.0 - y[-1] < 2e-9


def test_contract_at_scale_one_is_the_standard_contraction():
    """a = 1 "becomes the normal contract coordinates": half of (2 - 1/|x|) sign(x) outside
    the unit interval, half of x inside (the factor 0.5 maps the radius-2 ball to the cube)."""
    xs = np.array([-30.0, -2.5, -1.25, -0.75, 0.1, 1.5, 4.0, 100.0])
    std = np.where(np.abs(xs) <= 1.0, xs, (2.0 - 1.0 / np.abs(xs)) * np.sign(xs))
    np.testing.assert_allclose(_cc(TRIPLANE, 1.0, xs, axis=1), 0.5 * std, atol=1e-13)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_contract_is_a_rescaling_inside_the_unit_cube(kind):
    """Rays that stay inside |x| <= 1 on every axis only see 0.5 a x: the render and all its
    gradients equal those of the uncontracted renderer with the box widened by 2 / a."""
    a_scale = 1.5
    inp = lp_inputs.make_small(kind, res=(6, 5, 7), channels=4, mlp_dims=(4, 8, 4), n_rays=9, samples=11,
                               seed=41, origin_radius=0.7, near=(0.0, 0.1), far=(0.2, 0.28))
    span = np.abs(inp.origins.astype(np.float64)[:, None, :]
                  + np.linspace(0, 0.3, 5)[None, :, None] * inp.dirs.astype(np.float64)[:, None, :])
    assert span.max() < 1.0
    con = dataclasses.replace(inp, contract_a=a_scale)
    s = 2.0 / a_scale
    wide = dataclasses.replace(inp, aabb_min=(-s, -s, -s), aabb_max=(s, s, s))
    for x, y in zip(oracle.render_fwd(con), oracle.render_fwd(wide)):
        np.testing.assert_allclose(x, y, rtol=1e-10, atol=1e-13)
    rng = np.random.default_rng(1)
    p, pa, pd = rng.standard_normal((9, 3)), rng.standard_normal(9), rng.standard_normal(9)
    gc, gw = oracle.render_bwd(con, p, pa, pd), oracle.render_bwd(wide, p, pa, pd)
    for x, y in zip(gc[0] + gc[1] + gc[2], gw[0] + gw[1] + gw[2]):
        np.testing.assert_allclose(x, y, rtol=1e-9, atol=1e-12)


def test_contract_axes_are_independent():
    """One axis far outside, the others inside: each coordinate is contracted on its own."""
    pts_x = np.array([5.0, -0.4, 40.0])
    got = [_cc(VOXEL, 1.0, pts_x[[k]], axis=k)[0] for k in range(3)]
    np.testing.assert_allclose(got, [0.9, -0.2, 0.9875], atol=1e-13)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_contract_gradients_match_finite_differences(kind):
    """The scatter uses the same contracted positions as the gather: central differences of
    the loss with respect to every grid entry, rays reaching far outside the unit cube."""
    inp = lp_inputs.make_small(kind, res=(3, 4, 3), channels=2, mlp_dims=(2, 4, 4), n_rays=4, samples=6,
                               seed=53, grid_std=0.8, origin_radius=3.0, near=(0.2, 0.5), far=(5.0, 7.0))
    inp = dataclasses.replace(inp, contract_a=1.25, grid=[g.astype(np.float64) for g in inp.grid])
    rng = np.random.default_rng(5)
    p, pa, pd = rng.standard_normal((4, 3)), rng.standard_normal(4), rng.standard_normal(4)
    dg, _, _ = oracle.render_bwd(inp, p, pa, pd)
    h, checked = 1e-6, 0
    for arr, grad in zip(inp.grid, dg):
        flat, gflat = arr.reshape(-1), grad.reshape(-1)
        for k in range(flat.size):
            old = flat[k]
            flat[k] = old + h
            lp_ = _loss64(inp, p, pa, pd)
            flat[k] = old - h
            lm = _loss64(inp, p, pa, pd)
            flat[k] = old
            l0 = _loss64(inp, p, pa, pd)
            if abs(lp_ - 2 * l0 + lm) > 1e-9 * max(1.0, abs(l0)):
                continue
            assert gflat[k] == pytest.approx((lp_ - lm) / (2 * h), rel=2e-6, abs=2e-9)
            checked += 1
    assert checked > 30
