"""Pins of the oracle's Splatter (Section 3.3 "Splatter", appendix "Normalization Process"):
a hand-worked single point, partition of unity, constant features, adjointness with the
Renderer's (separately pinned) interpolation read, a dense-matrix restatement in torch with
autograd for every gradient, finite differences, and the kink envelope."""
import dataclasses

import numpy as np
import pytest

import lp_inputs
import oracle
from lp_inputs import TRIPLANE, VOXEL

from test_oracle_pins import _feat_of_points


def _single_ray(kind, point, feats, res=(3, 3, 3)):
    p = np.asarray(point, np.float32)
    d = np.array([[1.0, 0.0, 0.0]], np.float32)
    return lp_inputs.SplatInputs(kind=kind, n_scenes=1, channels=len(feats), res=res, aabb_min=(-1.0, -1.0, -1.0),
                                 aabb_max=(1.0, 1.0, 1.0), origins=p[None] - d, dirs=d,
                                 near=np.array([0.5], np.float32), far=np.array([1.5], np.float32), scene=None,
                                 samples=1, feats=np.asarray(feats, np.float32)[None])


def test_single_point_hand_worked():
    """Point (0.25, -0.5, 0.5) in a 3^3 grid over [-1,1]^3: index (1.25, 0.5, 1.5), cell (1,0,1),
    fractions (1/4, 1/2, 1/2).  Weights 3/16 on the four corners with x index 1 and 1/16 on those
    with x index 2 (Section 3.3: "normalized inverse distance ... eight voxel vertices").
    A single point leaves its own feature on every corner it touched."""
    sp = _single_ray(VOXEL, (0.25, -0.5, 0.5), (2.0, -3.0))
    theta, theta_w = oracle.splat_fwd(sp)
    w = np.zeros((3, 3, 3))
    w[1, 0:2, 1:3] = 3.0 / 16.0
    w[2, 0:2, 1:3] = 1.0 / 16.0
    np.testing.assert_allclose(theta_w[0][0], w, atol=1e-15)
    expect = np.zeros((3, 3, 3, 2))
    expect[w > 0] = (2.0, -3.0)
    np.testing.assert_allclose(theta[0][0], expect, atol=1e-14)
    # triplane: plane (x,y) gets the bilinear weights of (1.25, 0.5), plane (y,z) of (0.5, 1.5), ...
    sp = _single_ray(TRIPLANE, (0.25, -0.5, 0.5), (2.0, -3.0))
    theta, theta_w = oracle.splat_fwd(sp)
    wxy = np.zeros((3, 3)); wxy[1, 0:2] = 0.375; wxy[2, 0:2] = 0.125
    wyz = np.zeros((3, 3)); wyz[0:2, 1:3] = 0.25
    wzx = np.zeros((3, 3)); wzx[1:3, 1] = 0.375; wzx[1:3, 2] = 0.125
    for got, want in zip(theta_w, (wxy, wyz, wzx)):
        np.testing.assert_allclose(got[0], want, atol=1e-15)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_weights_are_a_partition_of_unity_and_constant_features_survive(kind):
    sp = lp_inputs.make_splat_small(kind, channels=3, res=(9, 8, 10), n_rays=40, samples=9, seed=4, n_scenes=2)
    sp.feats[...] = np.array([0.5, -1.25, 3.0], np.float32)
    theta, theta_w = oracle.splat_fwd(sp)
    for t, w in zip(theta, theta_w):
        assert w.sum() == pytest.approx(40 * 9, rel=1e-12)
        hit = w > 0
        np.testing.assert_allclose(t[hit], np.broadcast_to([0.5, -1.25, 3.0], t[hit].shape), rtol=1e-12)
        assert np.all(t[~hit] == 0.0)
        assert hit.any() and (kind == TRIPLANE or (~hit).any())


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_splat_is_the_transpose_of_the_renderers_read(kind):
    """sum_cells theta_unnormalised * G  ==  sum_ij v_i . h_G(x_ij): pushing with the weights the
    Renderer reads with (the read is pinned against scipy / torch in test_oracle_pins.py)."""
    rng = np.random.default_rng(8)
    sp = lp_inputs.make_splat_small(kind, channels=3, res=(5, 4, 6), n_rays=12, samples=7, seed=6)
    theta, theta_w = oracle.splat_fwd(sp)
    G = [rng.standard_normal(t.shape) for t in theta]
    lhs = sum(float((t * w[..., None] * g).sum()) for t, w, g in zip(theta, theta_w, G))
    # the same points, read from the structure G by the renderer oracle
    S = sp.samples
    delta = (sp.far.astype(np.float64) - sp.near) / S
    t = sp.near.astype(np.float64)[:, None] + (np.arange(S) + 0.5)[None] * delta[:, None]
    x = sp.origins.astype(np.float64)[:, None] + t[..., None] * sp.dirs.astype(np.float64)[:, None]
    ren = lp_inputs.make_small(kind, channels=3, res=(5, 4, 6), mlp_dims=(3, 4))
    ren = dataclasses.replace(ren, grid=G, aabb_min=sp.aabb_min, aabb_max=sp.aabb_max)
    # _feat_of_points rounds its points to float32, the splatter's points are fp64 combinations of
    # float32 rays: compare at the points the probe really uses
    pts32 = x.reshape(-1, 3).astype(np.float32)
    sp32 = dataclasses.replace(sp, origins=pts32 - np.array([1, 0, 0], np.float32), dirs=np.tile(np.array([[1.0, 0, 0]], np.float32), (len(pts32), 1)),
                               near=np.full(len(pts32), 0.5, np.float32), far=np.full(len(pts32), 1.5, np.float32),
                               samples=1, feats=np.repeat(sp.feats, S, axis=0))
    theta, theta_w = oracle.splat_fwd(sp32)
    lhs = sum(float((t * w[..., None] * g).sum()) for t, w, g in zip(theta, theta_w, G))
    read = _feat_of_points(ren, (sp32.origins.astype(np.float64) + np.array([1.0, 0, 0])))
    rhs = float((np.repeat(sp.feats.astype(np.float64), S, axis=0) * read).sum())
    assert lhs == pytest.approx(rhs, rel=1e-11)


def _interp_matrix(sp, res, points):
    """Dense [n_points, n_cells(+planes)] interpolation matrices of structure `res`, built by
    reading one-hot grids with torch's grid_sample (align_corners, border)."""
    import torch
    amin = torch.tensor(sp.aabb_min, dtype=torch.float64); amax = torch.tensor(sp.aabb_max, dtype=torch.float64)
    xn = (torch.from_numpy(points) - amin) / (amax - amin) * 2 - 1
    nx, ny, nz = res
    mats = []
    if sp.kind == VOXEL:
        n = nx * ny * nz
        basis = torch.eye(n, dtype=torch.float64).reshape(1, n, nx, ny, nz)
        a = torch.nn.functional.grid_sample(basis, xn[:, [2, 1, 0]][None, None, None], mode="bilinear",
                                            padding_mode="border", align_corners=True)[0, :, 0, 0].T
        mats.append(a)
    else:
        for (a_, b_), (na, nb) in zip([(0, 1), (1, 2), (2, 0)], [(nx, ny), (ny, nz), (nz, nx)]):
            n = na * nb
            basis = torch.eye(n, dtype=torch.float64).reshape(1, n, na, nb)
            a = torch.nn.functional.grid_sample(basis, xn[:, [b_, a_]][None, None], mode="bilinear",
                                                padding_mode="border", align_corners=True)[0, :, 0].T
            mats.append(a)
    return mats


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("with_mlp", [False, True])
def test_matches_dense_torch_restatement(kind, with_mlp):
    """theta = A^T vt, theta_w = A^T 1, out = theta / theta_w with A the dense interpolation
    matrix; the MLP and the prior read in torch; every gradient by torch autograd."""
    import torch
    kw = dict(hidden=(6, 5), n_freq=1, prior_channels=2, n_in=3) if with_mlp else {}
    sp = lp_inputs.make_splat_small(kind, channels=4, res=(4, 3, 5), n_rays=9, samples=6, seed=17, **kw)
    M, S, C = sp.n_rays, sp.samples, sp.channels
    theta, theta_w = oracle.splat_fwd(sp)
    rng = np.random.default_rng(3)
    G = [rng.standard_normal(t.shape) for t in theta]
    d_feats, d_prior, dW, db = oracle.splat_bwd(sp, theta_w, G)

    delta = (sp.far.astype(np.float64) - sp.near) / S
    t = sp.near.astype(np.float64)[:, None] + (np.arange(S) + 0.5)[None] * delta[:, None]
    x = (sp.origins.astype(np.float64)[:, None] + t[..., None] * sp.dirs.astype(np.float64)[:, None]).reshape(-1, 3)
    A = _interp_matrix(sp, sp.res, x)
    feats = torch.from_numpy(sp.feats.astype(np.float64)).requires_grad_()
    vt = feats[:, None, :].expand(M, S, -1).reshape(M * S, -1)
    leaves = [feats]
    if with_mlp:
        tp = [torch.from_numpy(g.astype(np.float64)).requires_grad_() for g in sp.prior]
        P = _interp_matrix(sp, sp.prior_res, x)
        prior_feat = sum(p @ g[0].reshape(-1, sp.prior_channels) for p, g in zip(P, tp))
        d = torch.from_numpy(sp.dirs.astype(np.float64))
        enc = torch.cat([d] + [fn((2.0 ** k) * np.pi * d) for k in range(sp.n_freq) for fn in (torch.sin, torch.cos)], 1)
        h = torch.cat([vt, prior_feat, enc[:, None, :].expand(M, S, -1).reshape(M * S, -1)], dim=1)
        tW = [torch.from_numpy(w.astype(np.float64)).requires_grad_() for w in sp.weights]
        tb = [torch.from_numpy(b.astype(np.float64)).requires_grad_() for b in sp.biases]
        for l in range(len(tW)):
            h = torch.nn.functional.linear(h, tW[l], tb[l])
            if l + 1 < len(tW):
                h = torch.relu(h)
        vt = h
        leaves += tp + tW + tb
    L = 0.0
    for a, th, tw, g in zip(A, theta, theta_w, G):
        acc = a.T @ vt                                   # [cells, C]
        wsum = a.sum(0)                                  # [cells]
        out = torch.where(wsum[:, None] > 0, acc / wsum.clamp_min(1e-300)[:, None], torch.zeros_like(acc))
        np.testing.assert_allclose(th[0].reshape(-1, C), out.detach().numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(tw[0].reshape(-1), wsum.numpy(), rtol=1e-11, atol=1e-14)
        L = L + (out * torch.from_numpy(g[0].reshape(-1, C))).sum()
    L.backward()
    mine = [d_feats] + (d_prior + dW + db if with_mlp else [])
    for a, b in zip(mine, leaves):
        np.testing.assert_allclose(a, b.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_gradients_match_finite_differences():
    sp = lp_inputs.make_splat_small(TRIPLANE, channels=2, res=(3, 4, 3), n_in=2, hidden=(4,), n_freq=0,
                                    prior_channels=2, prior_res=(3, 3, 4), n_rays=5, samples=4, seed=29, n_scenes=2)
    sp.feats = sp.feats.astype(np.float64)
    sp.prior = [g.astype(np.float64) for g in sp.prior]
    sp.weights = [w.astype(np.float64) for w in sp.weights]
    sp.biases = [b.astype(np.float64) for b in sp.biases]
    rng = np.random.default_rng(2)
    theta, theta_w = oracle.splat_fwd(sp)
    G = [rng.standard_normal(t.shape) for t in theta]

    def loss():
        th, _ = oracle.splat_fwd(sp)
        return float(sum((a * g).sum() for a, g in zip(th, G)))
    d_feats, d_prior, dW, db = oracle.splat_bwd(sp, theta_w, G)
    h, checked = 1e-6, 0
    for arrs, grads in (([sp.feats], [d_feats]), (sp.prior, d_prior), (sp.weights, dW), (sp.biases, db)):
        for arr, grad in zip(arrs, grads):
            flat, gflat = arr.reshape(-1), grad.reshape(-1)
            for k in range(flat.size):
                old = flat[k]
                flat[k] = old + h; lp_ = loss()
                flat[k] = old - h; lm = loss()
                flat[k] = old; l0 = loss()
                if abs(lp_ - 2 * l0 + lm) > 1e-9 * max(1.0, abs(l0)):
                    continue
                assert gflat[k] == pytest.approx((lp_ - lm) / (2 * h), rel=2e-6, abs=2e-9), k
                checked += 1
    assert checked > 100


def test_kink_envelope_brackets_the_definition():
    sp = lp_inputs.make_splat_small(VOXEL, channels=4, n_in=3, hidden=(16, 16), n_freq=0, prior_channels=3,
                                    n_rays=30, samples=12, seed=37, bias_std=0.0)
    theta, theta_w = oracle.splat_fwd(sp)
    G = [np.random.default_rng(1).standard_normal(t.shape) for t in theta]
    base = oracle.splat_bwd(sp, theta_w, G)
    lo = oracle.splat_bwd(sp, theta_w, G, kink_band=5e-2, kink_side=-1)
    hi = oracle.splat_bwd(sp, theta_w, G, kink_band=5e-2, kink_side=+1)
    flat = lambda r: [r[0]] + r[1] + r[2] + r[3]
    differs = 0
    for b, l, h in zip(flat(base), flat(lo), flat(hi)):
        tol = 1e-12 * max(1.0, np.abs(b).max())
        assert np.all(l <= b + tol) and np.all(b <= h + tol)
        differs += int(np.any(h - l > 1e-9))
    assert differs > 0
