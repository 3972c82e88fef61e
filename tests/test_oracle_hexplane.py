"""Pins of the oracle's HexPlane structure (Section 3.2 names HexPlane among the structures h and
defines none; the reading is Cao & Johnson 2023's six planes in three complementary pairs, (x,y)
with (z,t), (y,z) with (x,t), (z,x) with (y,t): the two bilinear reads of a pair are multiplied
channel by channel and the three products added).  CPU only.

* one point worked by hand (tests/golden/hexplane_point.txt);
* the feature of every sample against scipy's RegularGridInterpolator on the six planes (which
  plane reads which two coordinates, in which order; the clamp of positions and times);
* space-time planes of ones make it the triplane: outputs and plane gradients equal the triplane's
  (ties the spatial half to the path the other pin files cover), and the space-time planes then
  receive the gradient of a sum-of-products by the product rule;
* central differences on entries of all six planes; no time given = every ray at the first time.
"""
import dataclasses
import os

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HEXPLANE, TRIPLANE

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hexplane_point.txt")


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _problem(seed, contract=0.0, n_scenes=1, res=(5, 4, 6), n_time=4, t_range=(0.5, 2.0)):
    kw = dict(origin_radius=0.8, near=(0.0, 0.3), far=(4.0, 9.0)) if contract else {}
    inp = lp_inputs.make_small(HEXPLANE, n_scenes=n_scenes, channels=3, res=res, mlp_dims=(3, 6, 5, 4), n_rays=40,
                               samples=23, seed=seed, n_time=n_time, t_range=t_range, **kw)
    return dataclasses.replace(inp, contract_a=contract)


def test_the_point_worked_by_hand(oracle):
    rows = [tuple(float(v) for v in l.split()) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    (x, y, z, t, want), = rows
    planes = [[[1, 2], [3, 4]], [[0.5, 1.5], [2.5, 3.5]], [[2, 0], [1, 3]],
              [[1, 3], [5, 7]], [[2, 4], [6, 8]], [[1, 0], [0, 1]]]
    grid = [np.asarray(p, dtype=np.float32).reshape(1, 2, 2, 1) for p in planes]
    W = [np.ones((4, 1), dtype=np.float32)]
    b = [np.zeros(4, dtype=np.float32)]
    # one sample at distance 0.75 along +z from (x, y, 0)
    inp = lp_inputs.Inputs(kind=HEXPLANE, n_scenes=1, channels=1, res=(2, 2, 2), grid=grid, aabb_min=(0.0, 0.0, 0.0),
                           aabb_max=(1.0, 1.0, 1.0), mlp_dims=(1, 4), weights=W, biases=b,
                           origins=np.array([[x, y, 0.0]], dtype=np.float32), dirs=np.array([[0.0, 0.0, 1.0]], dtype=np.float32),
                           near=np.array([0.5], dtype=np.float32), far=np.array([1.0], dtype=np.float32), scene=None, samples=1,
                           bg=(0.0, 0.0, 0.0), time=np.array([t], dtype=np.float32), t_range=(0.0, 1.0))
    tr = oracle.ray_trace(inp, 0)
    assert tr["x"][0].tolist() == [x, y, z]
    assert tr["feat"][0, 0] == pytest.approx(want, rel=1e-14)


@pytest.mark.parametrize("contract", [0.0, 1.3])
def test_features_match_interpolators_on_the_six_planes(oracle, contract):
    from scipy.interpolate import RegularGridInterpolator as RGI
    inp = _problem(seed=31, contract=contract, n_scenes=2)
    N = inp.res
    nt = inp.n_time
    lo, hi = np.asarray(inp.aabb_min, dtype=np.float64), np.asarray(inp.aabb_max, dtype=np.float64)
    t0, t1 = float(np.float32(inp.t_range[0])), float(np.float32(inp.t_range[1]))
    axes = [np.linspace(lo[a], hi[a], N[a]) for a in range(3)]
    taxis = np.linspace(t0, t1, nt)
    a_c = float(np.float32(contract))

    def cc(x):
        if not contract:
            return x
        m = np.maximum(np.abs(x), 1.0)
        return np.where(np.abs(x) <= 1.0, 0.5 * a_c * x, np.sign(x) * 0.5 * ((2.0 - a_c) * (1.0 - 1.0 / m) + a_c))

    clamped_times = 0
    below, above = np.flatnonzero(inp.time < t0), np.flatnonzero(inp.time > t1)
    assert below.size and above.size     # the recipe draws times beyond both ends of the range
    for ray in (0, 7, int(below[0]), int(above[0])):
        tr = oracle.ray_trace(inp, ray)
        b = 0 if inp.scene is None else int(inp.scene[ray])
        pos = np.clip(cc(tr["x"]), lo, hi)                                   # [S][3]
        t_ray = float(inp.time[ray])
        clamped_times += t_ray < t0 or t_ray > t1
        t = np.full(pos.shape[0], min(max(t_ray, t0), t1))
        want = np.zeros_like(tr["feat"])
        for p in range(3):
            a, bb, c = p, (p + 1) % 3, (p + 2) % 3
            for k in range(inp.channels):
                s = RGI((axes[a], axes[bb]), inp.grid[p][b, :, :, k].astype(np.float64))(pos[:, [a, bb]])
                u = RGI((axes[c], taxis), inp.grid[3 + p][b, :, :, k].astype(np.float64))(np.stack([pos[:, c], t], 1))
                want[:, k] += s * u
        np.testing.assert_allclose(tr["feat"], want, rtol=1e-11, atol=1e-13)
    assert clamped_times >= 2


def test_unit_space_time_planes_make_it_the_triplane(oracle):
    inp = _problem(seed=37, n_scenes=2)
    ones = dataclasses.replace(inp, grid=inp.grid[:3] + [np.ones_like(g) for g in inp.grid[3:]])
    tri = dataclasses.replace(inp, kind=TRIPLANE, grid=inp.grid[:3], time=None)
    for a, b in zip(oracle.render_fwd(ones), oracle.render_fwd(tri)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    rng = np.random.default_rng(5)
    p_rgb, p_alpha, p_depth = rng.standard_normal((inp.n_rays, 3)), rng.standard_normal(inp.n_rays), rng.standard_normal(inp.n_rays)
    gh = oracle.render_bwd(ones, p_rgb, p_alpha, p_depth)
    gt = oracle.render_bwd(tri, p_rgb, p_alpha, p_depth)
    for p in range(3):
        np.testing.assert_allclose(gh[0][p], gt[0][p], rtol=1e-12, atol=1e-15)
        assert np.abs(gh[0][3 + p]).max() > 0
    for l in range(len(inp.weights)):
        np.testing.assert_allclose(gh[1][l], gt[1][l], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(gh[2][l], gt[2][l], rtol=1e-12, atol=1e-15)
    # and the other way round: unit spatial planes leave a "triplane" over (z,t), (x,t), (y,t), whose
    # gradient is the spatial planes' gradient of the mirrored problem summed over the spatial read's
    # weights -- checked through the sum over each space-time plane's entries at one time index pair:
    # with every plane constant (spatial s, space-time u) the feature is 3 s u at every point, so
    # d/ds and d/du of any loss are u and s times the same number
    const = dataclasses.replace(inp, grid=[np.full_like(g, 0.7) for g in inp.grid[:3]] + [np.full_like(g, 1.9) for g in inp.grid[3:]])
    g = oracle.render_bwd(const, p_rgb)[0]
    ds = sum(float(x.sum()) for x in g[:3])      # = dL/dfeat_total * u summed over pairs
    du = sum(float(x.sum()) for x in g[3:])      # = dL/dfeat_total * s summed over pairs
    s_val, u_val = float(np.float32(0.7)), float(np.float32(1.9))    # (the planes hold float32 values)
    assert ds * s_val == pytest.approx(du * u_val, rel=1e-10) and abs(ds) > 0


def test_gradients_by_central_differences(oracle):
    inp = _problem(seed=41, res=(3, 4, 3), n_time=3)
    rng = np.random.default_rng(6)
    p_rgb = rng.standard_normal((inp.n_rays, 3))
    g = oracle.render_bwd(inp, p_rgb)[0]
    loss = lambda i: float((oracle.render_fwd(i)[0] * p_rgb).sum())
    h = 1e-4
    checked = 0
    for p in range(6):
        flat = np.argsort(-np.abs(g[p]).reshape(-1))[:3]          # the entries that matter most
        for f in flat:
            idx = np.unravel_index(int(f), g[p].shape)
            up = [a.copy() for a in inp.grid]; dn = [a.copy() for a in inp.grid]
            up[p][idx] += np.float32(h); dn[p][idx] -= np.float32(h)
            step = float(up[p][idx]) - float(dn[p][idx])
            fd = (loss(dataclasses.replace(inp, grid=up)) - loss(dataclasses.replace(inp, grid=dn))) / step
            assert abs(fd - g[p][idx]) <= 2e-5 * max(1.0, abs(fd)), (p, idx, fd, g[p][idx])
            checked += 1
    assert checked == 18


def test_time_is_clamped_and_defaults_to_the_first_time(oracle):
    inp = _problem(seed=43)
    t0, t1 = inp.t_range
    early = dataclasses.replace(inp, time=np.full(inp.n_rays, t0 - 3.0, dtype=np.float32))
    first = dataclasses.replace(inp, time=np.full(inp.n_rays, t0, dtype=np.float32))
    none = dataclasses.replace(inp, time=None)
    late = dataclasses.replace(inp, time=np.full(inp.n_rays, t1 + 5.0, dtype=np.float32))
    last = dataclasses.replace(inp, time=np.full(inp.n_rays, t1, dtype=np.float32))
    a, b, c = oracle.render_fwd(early)[0], oracle.render_fwd(first)[0], oracle.render_fwd(none)[0]
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(b, c)
    np.testing.assert_array_equal(oracle.render_fwd(late)[0], oracle.render_fwd(last)[0])
    assert np.abs(oracle.render_fwd(last)[0] - b).max() > 1e-3      # time matters


@pytest.mark.parametrize("decoder", [False, True])
def test_kink_envelope_brackets_the_definition(oracle, decoder):
    """The feature gradient's envelope reaches the planes through products with signed plane reads: the
    upper side must still lie above the definition, the lower side below it, on all six planes (a
    wide band, so that many units fall inside it), and a vanishing band must collapse onto it."""
    inp = _problem(seed=47, n_scenes=2)
    assert min(float(g.min()) for g in inp.grid[:3]) < 0        # negative reads occur
    rng = np.random.default_rng(8)
    if decoder:
        dec = lp_inputs.make_decoder(3, (5,), (6, 4), 1, 3, 48, 0.2, 0)
        inp = dataclasses.replace(inp, decoder=dec)
        p = rng.standard_normal((inp.n_rays, 3))
        run = lambda band, side: oracle.render2_bwd(inp, p, kink_band=band, kink_side=side)[0]
    else:
        p = rng.standard_normal((inp.n_rays, 3))
        run = lambda band, side: oracle.render_bwd(inp, p, kink_band=band, kink_side=side)[0]
    base, lo, hi = run(0.0, 0), run(5e-2, -1), run(5e-2, +1)
    wide = 0
    for q in range(6):
        tol = 1e-12 * np.abs(base[q]).max()
        assert (lo[q] <= base[q] + tol).all() and (base[q] <= hi[q] + tol).all(), q
        wide += int(((hi[q] - lo[q]) > 1e-6 * np.abs(base[q]).max()).sum())
    assert wide > 0
    for q, (a, b) in enumerate(zip(run(1e-15, +1), run(1e-15, -1))):
        # (the scatter adds with atomics from several threads: equal up to the order of the sums)
        np.testing.assert_allclose(a, base[q], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(b, base[q], rtol=1e-12, atol=1e-15)
