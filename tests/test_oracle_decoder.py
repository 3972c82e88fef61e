"""Pins of the oracle's two-MLP, view-dependent decoder (Section 3.3, text below Eq. (1)):
hand-worked encoding values, closed forms with a constant feature, reduction to the
single-MLP renderer (pinned in test_oracle_pins.py), torch autograd as a third opinion,
finite differences, and the kink envelope bracketing the definition."""
import dataclasses
import os

import numpy as np
import pytest

import lp_inputs
import oracle
from lp_inputs import TRIPLANE, VOXEL

HERE = os.path.dirname(os.path.abspath(__file__))


def _problem(kind, *, channels=4, hidden_s=(6,), hidden_v=(7, 5), n_freq=1, n_feat=3, feat_act=0, seed=0,
             n_rays=7, samples=6, n_scenes=1, bias_std=0.3, **kw):
    inp = lp_inputs.make_small(kind, channels=channels, mlp_dims=(channels, 4), n_rays=n_rays, samples=samples,
                               seed=seed, n_scenes=n_scenes, **kw)
    dec = lp_inputs.make_decoder(channels, hidden_s, hidden_v, n_freq, n_feat, seed + 100, bias_std, feat_act)
    rng = np.random.default_rng(seed + 7)
    return dataclasses.replace(inp, decoder=dec, bg=tuple(rng.random(n_feat).astype(np.float32).tolist()),
                               target=rng.random((n_rays, n_feat), dtype=np.float32))


def test_direction_encoding_matches_hand_worked_values():
    gold = np.loadtxt(os.path.join(HERE, "golden", "dir_encoding.txt"))
    np.testing.assert_allclose(oracle.dir_encode([0.5, 0.0, -0.5], 2), gold, atol=1e-15)
    # L = 0 is the raw direction; more octaves only append
    np.testing.assert_array_equal(oracle.dir_encode([0.3, -0.2, 0.9], 0), [0.3, -0.2, 0.9])
    np.testing.assert_array_equal(oracle.dir_encode([0.3, -0.2, 0.9], 3)[:9], oracle.dir_encode([0.3, -0.2, 0.9], 1))


@pytest.mark.parametrize("feat_act", [0, 1])
def test_constant_feature_closed_form(feat_act):
    """A feature MLP that is one linear layer with zero weights returns act(b) everywhere:
    out = (1 - T_S) act(b) + T_S bg, whatever the opacity MLP does."""
    inp = _problem(VOXEL, hidden_v=(), n_feat=5, feat_act=feat_act, seed=3)
    dec = inp.decoder
    dec.weights_v[0][...] = 0.0
    dec.biases_v[0][...] = np.array([0.3, -1.2, 2.0, 0.0, -0.4], np.float32)
    out, alpha, _ = oracle.render2_fwd(inp)
    b = dec.biases_v[0].astype(np.float64)
    f = 1.0 / (1.0 + np.exp(-b)) if feat_act == 0 else b
    bg = np.asarray(inp.bg, np.float32).astype(np.float64)
    np.testing.assert_allclose(out, alpha[:, None] * f + (1.0 - alpha[:, None]) * bg, rtol=1e-12, atol=1e-14)
    assert 0.05 < alpha.min() and alpha.max() < 0.999


def _combined_single_mlp(dec, channels):
    """Block-diagonal single MLP C -> ... -> 4 equal to a decoder whose feature MLP ignores the
    direction (its direction columns must be zero); a shallower MLP is carried through the
    extra layers by identity blocks, exact behind a ReLU."""
    Ls, Lv = len(dec.weights_s), len(dec.weights_v)
    L = max(Ls, Lv)

    def padded(ws, bs, n):   # hidden layers, identity layers, output layer
        hid = [(w.astype(np.float64), b.astype(np.float64)) for w, b in zip(ws[:-1], bs[:-1])]
        width = hid[-1][0].shape[0]
        hid += [(np.eye(width), np.zeros(width))] * (n - len(ws))
        return hid + [(ws[-1].astype(np.float64), bs[-1].astype(np.float64))]
    S = padded(dec.weights_s, dec.biases_s, L)
    V = padded([dec.weights_v[0][:, :channels]] + dec.weights_v[1:], dec.biases_v, L)
    Ws, bs = [], []
    for l in range(L):
        (ws, b1), (wv, b2) = S[l], V[l]
        if l == 0:
            W = np.concatenate([ws, wv], axis=0)
        else:
            W = np.zeros((ws.shape[0] + wv.shape[0], ws.shape[1] + wv.shape[1]))
            W[:ws.shape[0], :ws.shape[1]] = ws
            W[ws.shape[0]:, ws.shape[1]:] = wv
        Ws.append(W)
        bs.append(np.concatenate([b1, b2]))
    return Ws, bs


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("hidden_s,hidden_v", [((6,), (5,)), ((6,), (7, 5)), ((4, 3), (5,))])
def test_reduces_to_the_single_mlp_renderer(kind, hidden_s, hidden_v):
    """With the direction columns of the feature MLP zeroed and three sigmoid features, the
    decoder is the single-MLP decoder with block-diagonal weights: same images, and the
    gradients of the blocks agree."""
    inp = _problem(kind, hidden_s=hidden_s, hidden_v=hidden_v, n_freq=1, n_feat=3, seed=11, n_scenes=2)
    dec, C = inp.decoder, inp.channels
    dec.weights_v[0][:, C:] = 0.0
    Ws, bs = _combined_single_mlp(dec, C)
    dims = (C,) + tuple(w.shape[0] for w in Ws)
    single = dataclasses.replace(inp, decoder=None, mlp_dims=dims, weights=Ws, biases=bs)
    out2, a2, d2 = oracle.render2_fwd(inp)
    out1, a1, d1 = oracle.render_fwd(single)
    np.testing.assert_allclose(out2, out1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(a2, a1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(d2, d1, rtol=1e-12, atol=1e-14)
    rng = np.random.default_rng(2)
    M = inp.n_rays
    p, pa, pd = rng.standard_normal((M, 3)), rng.standard_normal(M), rng.standard_normal(M)
    dg2, dWs, dbs, dWv, dbv = oracle.render2_bwd(inp, p, pa, pd)
    dg1, dW1, db1 = oracle.render_bwd(single, p, pa, pd)
    for x, y in zip(dg2, dg1):
        np.testing.assert_allclose(x, y, rtol=1e-10, atol=1e-13)
    hs = dec.dims_s[1]
    # first layer: rows of the opacity block, then rows of the feature block (feature columns)
    np.testing.assert_allclose(dWs[0], dW1[0][:hs], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dWv[0][:, :C], dW1[0][hs:], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dbs[0], db1[0][:hs], rtol=1e-10, atol=1e-13)
    # output layers: row 0 / rows 1..3 of the last combined layer
    ws_last = dec.weights_s[-1].shape[1]
    np.testing.assert_allclose(dWs[-1], dW1[-1][:1, :ws_last], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dWv[-1], dW1[-1][1:, ws_last:], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dbv[-1], db1[-1][1:], rtol=1e-10, atol=1e-13)


def _torch_features(inp, tg):
    """Interpolated features [M,S,C] with torch's grid_sample (align_corners, border)."""
    import torch
    M, S = inp.n_rays, inp.samples
    o = torch.from_numpy(inp.origins.astype(np.float64)); d = torch.from_numpy(inp.dirs.astype(np.float64))
    nr = torch.from_numpy(inp.near.astype(np.float64)); fr = torch.from_numpy(inp.far.astype(np.float64))
    delta = (fr - nr) / S
    t = nr[:, None] + (torch.arange(S, dtype=torch.float64)[None] + 0.5) * delta[:, None]
    x = o[:, None, :] + t[..., None] * d[:, None, :]
    amin = torch.tensor(inp.aabb_min, dtype=torch.float64); amax = torch.tensor(inp.aabb_max, dtype=torch.float64)
    xn = (x - amin) / (amax - amin) * 2 - 1
    scene = torch.zeros(M, dtype=torch.int64) if inp.scene is None else torch.from_numpy(inp.scene.astype(np.int64))
    feat = torch.zeros(M, S, inp.channels, dtype=torch.float64)
    for b in range(inp.n_scenes):
        sel = (scene == b).nonzero()[:, 0]
        if sel.numel() == 0:
            continue
        q = xn[sel]
        if inp.kind == VOXEL:
            vol = tg[0][b].permute(3, 0, 1, 2)[None]
            f = torch.nn.functional.grid_sample(vol, q[..., [2, 1, 0]][None, None], mode="bilinear",
                                                padding_mode="border", align_corners=True)[0, :, 0]
        else:
            f = 0
            for pl, (a, c) in enumerate([(0, 1), (1, 2), (2, 0)]):
                img = tg[pl][b].permute(2, 0, 1)[None]
                f = f + torch.nn.functional.grid_sample(img, q[..., [c, a]][None], mode="bilinear",
                                                        padding_mode="border", align_corners=True)[0]
        feat = feat.index_put((sel,), f.permute(1, 2, 0))
    return feat, t, delta, d


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("feat_act", [0, 1])
def test_matches_torch_autograd(kind, feat_act):
    """The naive autograd renderer with two torch MLPs, differentiated by torch."""
    import torch
    inp = _problem(kind, channels=4, hidden_s=(8, 6), hidden_v=(9,), n_freq=2, n_feat=5, feat_act=feat_act,
                   seed=23, n_rays=11, samples=8, n_scenes=2, res=(6, 5, 7), grid_std=0.7)
    dec = inp.decoder
    M, S, F = inp.n_rays, inp.samples, dec.n_feat
    rng = np.random.default_rng(9)
    p, pa, pd = rng.standard_normal((M, F)), rng.standard_normal(M), rng.standard_normal(M)
    out, alpha, depth = oracle.render2_fwd(inp)
    grads = oracle.render2_bwd(inp, p, pa, pd)

    tg = [torch.from_numpy(g.astype(np.float64)).requires_grad_() for g in inp.grid]
    par = lambda lst: [torch.from_numpy(a.astype(np.float64)).requires_grad_() for a in lst]
    tWs, tbs, tWv, tbv = par(dec.weights_s), par(dec.biases_s), par(dec.weights_v), par(dec.biases_v)
    feat, t, delta, d = _torch_features(inp, tg)
    enc = [d] + [fn((2.0 ** k) * np.pi * d) for k in range(dec.n_freq) for fn in (torch.sin, torch.cos)]
    enc = torch.cat(enc, dim=1)[:, None, :].expand(M, S, -1)

    def mlp(h, Ws, bs):
        for l in range(len(Ws)):
            h = torch.nn.functional.linear(h, Ws[l], bs[l])
            if l + 1 < len(Ws):
                h = torch.relu(h)
        return h
    sigma = torch.nn.functional.softplus(mlp(feat, tWs, tbs)[..., 0], threshold=1e9)
    fv = mlp(torch.cat([feat, enc], dim=-1), tWv, tbv)
    fv = torch.sigmoid(fv) if feat_act == 0 else fv
    T = torch.exp(-torch.cumsum(sigma * delta[:, None], dim=1))
    Tprev = torch.cat([torch.ones(M, 1, dtype=torch.float64), T[:, :-1]], dim=1)
    w = Tprev - T
    bg = torch.tensor(np.asarray(inp.bg, dtype=np.float32).astype(np.float64))
    t_out = (w[..., None] * fv).sum(1) + T[:, -1:] * bg
    t_alpha, t_depth = 1 - T[:, -1], (w * t).sum(1)
    np.testing.assert_allclose(out, t_out.detach().numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(alpha, t_alpha.detach().numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(depth, t_depth.detach().numpy(), rtol=1e-11)
    L = (t_out * torch.from_numpy(p)).sum() + (t_alpha * torch.from_numpy(pa)).sum() + (t_depth * torch.from_numpy(pd)).sum()
    L.backward()
    mine = grads[0] + grads[1] + grads[2] + grads[3] + grads[4]
    for a, b in zip(mine, tg + tWs + tbs + tWv + tbv):
        np.testing.assert_allclose(a, b.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_gradients_match_finite_differences():
    inp = _problem(TRIPLANE, channels=3, hidden_s=(4,), hidden_v=(5,), n_freq=1, n_feat=2, seed=31, n_rays=4,
                   samples=5, res=(3, 4, 3), grid_std=0.8)
    dec = inp.decoder
    inp.grid = [g.astype(np.float64) for g in inp.grid]
    for lst in (dec.weights_s, dec.biases_s, dec.weights_v, dec.biases_v):
        for i in range(len(lst)):
            lst[i] = lst[i].astype(np.float64)
    rng = np.random.default_rng(3)
    p, pa, pd = rng.standard_normal((4, 2)), rng.standard_normal(4), rng.standard_normal(4)

    def loss():
        out, alpha, depth = oracle.render2_fwd(inp)
        return float((out * p).sum() + (alpha * pa).sum() + (depth * pd).sum())
    dg, dWs, dbs, dWv, dbv = oracle.render2_bwd(inp, p, pa, pd)
    h, checked = 1e-6, 0
    for arrs, grads in ((inp.grid, dg), (dec.weights_s, dWs), (dec.biases_s, dbs), (dec.weights_v, dWv),
                        (dec.biases_v, dbv)):
        for arr, grad in zip(arrs, grads):
            flat, gflat = arr.reshape(-1), grad.reshape(-1)
            for k in range(flat.size):
                old = flat[k]
                flat[k] = old + h; lp_ = loss()
                flat[k] = old - h; lm = loss()
                flat[k] = old; l0 = loss()
                if abs(lp_ - 2 * l0 + lm) > 1e-9 * max(1.0, abs(l0)):
                    continue      # a ReLU kink inside the stencil
                assert gflat[k] == pytest.approx((lp_ - lm) / (2 * h), rel=2e-6, abs=2e-9), k
                checked += 1
    assert checked > 150


def test_view_direction_reaches_the_features():
    """Same origin and samples seen along d and along -d from the far end: opacity (alpha)
    depends on position only, the rendered feature also on the direction."""
    inp = _problem(VOXEL, n_rays=6, samples=9, seed=41, near=(0.2, 0.2001), far=(3.0, 3.0001))
    inp.near[...] = 0.2
    inp.far[...] = 3.0
    flipped = dataclasses.replace(
        inp, origins=np.ascontiguousarray(inp.origins + np.float32(3.2) * inp.dirs), dirs=np.ascontiguousarray(-inp.dirs))
    out_a, alpha_a, _ = oracle.render2_fwd(inp)
    out_b, alpha_b, _ = oracle.render2_fwd(flipped)
    np.testing.assert_allclose(alpha_a, alpha_b, rtol=1e-5)     # same points (up to float32 origins)
    assert np.abs(out_a - out_b).max() > 1e-3


def test_kink_envelope_brackets_the_definition():
    inp = _problem(VOXEL, channels=4, hidden_s=(16,), hidden_v=(16, 16), n_rays=40, samples=20, seed=51,
                   bias_std=0.0)
    rng = np.random.default_rng(1)
    p = rng.standard_normal((40, 3))
    base = oracle.render2_bwd(inp, p)
    lo = oracle.render2_bwd(inp, p, kink_band=5e-2, kink_side=-1)
    hi = oracle.render2_bwd(inp, p, kink_band=5e-2, kink_side=+1)
    differs = 0
    for B, L, H in zip(base, lo, hi):
        for b, l, h in zip(B, L, H):
            tol = 1e-12 * max(1.0, np.abs(b).max())
            assert np.all(l <= b + tol) and np.all(b <= h + tol)
            differs += int(np.any(h - l > 1e-9))
    assert differs > 0     # the (wide) band did catch some units
