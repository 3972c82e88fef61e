"""Pins of the oracle's hash-table structure (Section 3.2 names hash tables among the structures h
and defines none; the reading is the single-resolution spatial hash of Teschner et al. 2003 with
Instant-NGP's primes).  CPU only.

* the slot of a lattice corner against values worked out with arbitrary-precision integers
  (tests/golden/hash_slots.txt);
* a render through a hash table against a render through the VOXEL grid whose cell (ix, iy, iz)
  holds the table entry of that corner -- outputs equal, and the table's gradient equal to the voxel
  grid's gradient summed over the corners that share an entry -- which ties gather and scatter
  (collisions included) to the voxel path that the other pin files cover;
* a table with one entry is a constant field; central differences on table entries.
"""
import dataclasses
import os

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HASH, VOXEL

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hash_slots.txt")


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def test_slots_match_the_worked_values(oracle):
    rows = [tuple(int(v) for v in l.split()) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for ix, iy, iz, T, want in rows:
        assert oracle.hash_slot(ix, iy, iz, T) == want, (ix, iy, iz, T)


def _slots(oracle, res, T):
    nx, ny, nz = res
    s = np.empty(res, dtype=np.int64)
    for ix in range(nx):
        for iy in range(ny):
            for iz in range(nz):
                s[ix, iy, iz] = oracle.hash_slot(ix, iy, iz, T)
    return s


def _problem(T, seed, contract=0.0, n_scenes=1, res=(5, 4, 6)):
    kw = dict(origin_radius=0.8, near=(0.0, 0.3), far=(4.0, 9.0)) if contract else {}
    inp = lp_inputs.make_small(HASH, n_scenes=n_scenes, channels=3, res=res, mlp_dims=(3, 6, 5, 4), n_rays=40,
                               samples=23, seed=seed, hash_size=T, **kw)
    return dataclasses.replace(inp, contract_a=contract)


@pytest.mark.parametrize("T", [1, 7, 64, 1000003])     # everything collides ... nothing collides
@pytest.mark.parametrize("contract", [0.0, 1.3])
def test_equals_the_voxel_grid_of_the_hashed_entries(oracle, T, contract):
    inp = _problem(T, seed=5 + T, contract=contract, n_scenes=2)
    slots = _slots(oracle, inp.res, T)
    if T == 1000003:
        assert len(np.unique(slots)) == slots.size        # no collision on this lattice
    if T == 7:
        assert len(np.unique(slots)) < slots.size
    table = inp.grid[0]                                     # [B][T][C]
    voxel = np.ascontiguousarray(table[:, slots.reshape(-1), :].reshape(inp.n_scenes, *inp.res, inp.channels))
    as_voxel = dataclasses.replace(inp, kind=VOXEL, grid=[voxel])

    out_h = oracle.render_fwd(inp)
    out_v = oracle.render_fwd(as_voxel)
    for a, b in zip(out_h, out_v):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)

    rng = np.random.default_rng(3)
    p_rgb = rng.standard_normal((inp.n_rays, 3))
    p_alpha = rng.standard_normal(inp.n_rays)
    p_depth = rng.standard_normal(inp.n_rays)
    gh = oracle.render_bwd(inp, p_rgb, p_alpha, p_depth)
    gv = oracle.render_bwd(as_voxel, p_rgb, p_alpha, p_depth)
    d_table = gh[0][0]
    d_voxel = gv[0][0].reshape(inp.n_scenes, -1, inp.channels)
    want = np.zeros_like(d_table)
    for b in range(inp.n_scenes):
        np.add.at(want[b], slots.reshape(-1), d_voxel[b])    # corners that share an entry add
    np.testing.assert_allclose(d_table, want, rtol=1e-12, atol=1e-14)
    assert np.abs(d_table).max() > 0
    for l in range(len(inp.weights)):
        np.testing.assert_allclose(gh[1][l], gv[1][l], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(gh[2][l], gv[2][l], rtol=1e-12, atol=1e-14)


def test_single_entry_table_is_a_constant_field(oracle):
    """T = 1: every corner reads the same vector, so the feature of every sample is that vector (the
    trilinear weights sum to one) and the render equals the closed form for a constant medium."""
    inp = _problem(1, seed=11)
    rgb, alpha, depth = oracle.render_fwd(inp)[:3]
    v = inp.grid[0][0, 0].astype(np.float64)
    x = v
    for l, (W, b) in enumerate(zip(inp.weights, inp.biases)):
        x = W.astype(np.float64) @ x + b.astype(np.float64)
        if l + 1 < len(inp.weights):
            x = np.maximum(x, 0.0)
    sigma = np.log1p(np.exp(x[0]))
    col = 1.0 / (1.0 + np.exp(-x[1:4]))
    length = inp.far.astype(np.float64) - inp.near.astype(np.float64)
    T_end = np.exp(-sigma * length)
    np.testing.assert_allclose(alpha, 1.0 - T_end, rtol=1e-12)
    want = (1.0 - T_end)[:, None] * col[None, :] + T_end[:, None] * np.asarray(inp.bg, dtype=np.float32).astype(np.float64)[None, :]   # (the background is a float32 input)
    np.testing.assert_allclose(rgb, want, rtol=1e-12)


def test_table_gradient_by_central_differences(oracle):
    inp = _problem(13, seed=17)
    rng = np.random.default_rng(4)
    p_rgb = rng.standard_normal((inp.n_rays, 3))
    g = oracle.render_bwd(inp, p_rgb)[0][0]
    loss = lambda i: float((oracle.render_fwd(i)[0] * p_rgb).sum())
    h = 1e-4
    for (t, c) in [(0, 0), (5, 2), (12, 1), (7, 0)]:
        up = [a.copy() for a in inp.grid]; dn = [a.copy() for a in inp.grid]
        up[0][0, t, c] += np.float32(h); dn[0][0, t, c] -= np.float32(h)
        step = float(up[0][0, t, c]) - float(dn[0][0, t, c])
        fd = (loss(dataclasses.replace(inp, grid=up)) - loss(dataclasses.replace(inp, grid=dn))) / step
        assert abs(fd - g[0, t, c]) <= 1e-5 * max(1.0, abs(fd)), (t, c, fd, g[0, t, c])


# ---- the Splatter into a hash table (Section 3.3: the Splatter writes the hash structure; colliding
# corners share an entry, whose feature is the weighted mean over everything pushed into it)

def _splat(T, seed, hidden=None, prior_T=0, n_freq=-1):
    return lp_inputs.make_splat_small(HASH, n_scenes=2, channels=3, res=(5, 4, 6), n_rays=40, samples=11, seed=seed,
                                      hash_size=T, hidden=hidden, n_freq=n_freq, n_in=3 if hidden is None else 4,
                                      prior_channels=2 if prior_T else 0, prior_res=(4, 5, 3), prior_hash_size=prior_T)


@pytest.mark.parametrize("T", [1, 7, 64, 1000003])
def test_splat_into_a_table_pools_the_voxel_splat_over_colliding_corners(oracle, T):
    sp = _splat(T, seed=61 + T % 5)
    as_voxel = dataclasses.replace(sp, kind=VOXEL, hash_size=0)
    th, tw = oracle.splat_fwd(sp)
    tv, wv = oracle.splat_fwd(as_voxel)
    slots = _slots(oracle, sp.res, T).reshape(-1)
    for b in range(sp.n_scenes):
        w = np.zeros(T)
        s = np.zeros((T, sp.channels))
        np.add.at(w, slots, wv[0][b].reshape(-1))
        np.add.at(s, slots, (tv[0][b] * wv[0][b][..., None]).reshape(-1, sp.channels))   # un-normalised sums
        np.testing.assert_allclose(tw[0][b], w, rtol=1e-12, atol=1e-15)
        want = np.divide(s, w[:, None], out=np.zeros_like(s), where=w[:, None] > 0)
        np.testing.assert_allclose(th[0][b], want, rtol=1e-11, atol=1e-14)
    assert np.isclose(tw[0].sum(), sp.n_rays * sp.samples)         # the weights of a point sum to one


def test_splat_into_a_table_gradients_by_central_differences(oracle):
    """Naive Splatter: pixel features; with MLP and a prior table: features, prior entries, weights."""
    rng = np.random.default_rng(9)
    for sp in (_splat(13, seed=67), _splat(29, seed=71, hidden=(6,), prior_T=11, n_freq=0)):
        th, tw = oracle.splat_fwd(sp)
        G = [rng.standard_normal(t.shape) for t in th]
        d_feats, d_prior, dW, db = oracle.splat_bwd(sp, tw, G)
        loss = lambda s: float(sum((a * g).sum() for a, g in zip(oracle.splat_fwd(s)[0], G)))
        h = 1e-4

        def fd(field, idx, which=None):
            up, dn = [np.array(a, copy=True) for a in (getattr(sp, field) if which is None else getattr(sp, field)[which],) * 2]
            up[idx] += np.float32(h); dn[idx] -= np.float32(h)
            step = float(up[idx]) - float(dn[idx])
            def put(a):
                if which is None:
                    return dataclasses.replace(sp, **{field: a})
                lst = list(getattr(sp, field)); lst[which] = a
                return dataclasses.replace(sp, **{field: lst})
            return (loss(put(up)) - loss(put(dn))) / step

        for idx in [(0, 0), (17, 2), (39, 1)]:
            v = fd("feats", idx)
            assert abs(v - d_feats[idx]) <= 2e-5 * max(1.0, abs(v)), ("feats", idx, v, d_feats[idx])
        if sp.mlp_dims is not None:
            flat = np.argsort(-np.abs(d_prior[0]).reshape(-1))[:3]
            for f in flat:
                idx = np.unravel_index(int(f), d_prior[0].shape)
                v = fd("prior", idx, 0)
                assert abs(v - d_prior[0][idx]) <= 2e-5 * max(1.0, abs(v)), ("prior", idx, v, d_prior[0][idx])
            for l in range(len(dW)):
                idx = np.unravel_index(int(np.argmax(np.abs(dW[l]))), dW[l].shape)
                v = fd("weights", idx, l)
                assert abs(v - dW[l][idx]) <= 2e-5 * max(1.0, abs(v)), ("W", l, idx, v, dW[l][idx])
