"""Helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded host buffers and compare element by element."""
from __future__ import annotations

import numpy as np

FWD_RTOL = 1e-4   # forward outputs, fp32 relative tolerance
BWD_RTOL = 1e-3   # gradients


def close(gpu: np.ndarray, ref: np.ndarray, rtol: float, what: str, extra=None):
    """Per tensor, elementwise |gpu - ref| <= rtol |ref| + rtol rms(ref) (+ extra, an elementwise
    absolute allowance for results that are ill-conditioned by construction)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), f"{what}: non-finite values from the GPU"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(gpu - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    if extra is not None:
        bound = bound + extra
    if not (err <= bound).all():
        k = int(np.argmax(err - bound))
        raise AssertionError(
            f"{what}: {int((err > bound).sum())} of {ref.size} elements out of tolerance {rtol:g}; "
            f"worst at flat index {k}: gpu={gpu.reshape(-1)[k]!r} ref={ref.reshape(-1)[k]!r} "
            f"rms(ref)={rms:g} max|err|/max|ref|={err.max() / max(np.abs(ref).max(), 1e-300):g}")
    return float(err.max() / max(rms, 1e-300))


# Kink band, as a multiple of each hidden unit's rounding-error scale |b| + sum_k |W_k x_k|.
# The kernels form sample positions and interpolation fractions in fp64, so what is left on a
# pre-activation is the contraction error and what the layer below passes on.  For the
# split-bf16 matrix-core path each product w x is off by at most 3 * 2^-18 |w x| (hi+lo
# representation of either factor, dropped lo*lo term), i.e. 1.1e-5 of the scale in the worst
# case; a second hidden layer inherits about as much again through its inputs.  The band is
# that worst case, not a multiple of a typical error: split errors of the weights are fixed per
# weight and neighbouring samples are nearly equal, so the errors are far from independent.
KINK_BAND = 2e-5

# The envelope is a worst case: every banded sample adds its whole contribution to upper - lower
# (relative L2 widths of 4e-3 ... 6e-2 on the configurations, see test_oracle_envelope.py),
# while a kernel flips only the few units whose rounding error really crosses zero.  So the
# whole-tensor error around the definition's gradient may use at most this much of the width.
WIDTH_CAP = 1e-3
# Splatter: points of a ray that are clamped to one border position of the prior structure share
# every MLP input (pixel feature and direction are per ray), so their pre-activations coincide and
# flip TOGETHER; there the flips do not average out and the cap is the width itself.
WIDTH_CAP_SPLAT_BORDER = None
# Share of a gradient tensor's elements that may miss the plain tolerance around the definition's
# gradient (they must still lie inside the envelope).  Observed on the GPU: at most 1 %.
MAX_STRICT_FAIL = 0.02


class GradErr(tuple):
    """(max distance to the envelope / rms, share of elements outside the plain tolerance,
    relative L2 error around the definition's gradient, relative L2 width of the envelope)."""
    env = property(lambda s: s[0])
    strict_fail = property(lambda s: s[1])
    l2 = property(lambda s: s[2])
    width = property(lambda s: s[3])


def close_envelope(gpu, ref, lo, hi, rtol: float, what: str, width_cap=WIDTH_CAP):
    """Gradient check.  Where a hidden pre-activation lies within rounding of the ReLU kink,
    either one-sided derivative is a correct answer; `lo`/`hi` are the elementwise envelope
    of the oracle's gradients over those choices (lo == hi == ref for elements no such sample
    touches).  EVERY element must lie within tolerance of the envelope; the fraction of
    elements outside the strict tolerance around `ref` itself is returned for the caller to
    bound.  Returns a GradErr."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), f"{what}: non-finite values from the GPU"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bound = rtol * np.abs(ref) + rtol * rms
    err = np.maximum(np.maximum(lo - gpu, gpu - hi), 0.0)
    if not (err <= bound).all():
        k = int(np.argmax(err - bound))
        raise AssertionError(
            f"{what}: {int((err > bound).sum())} of {ref.size} elements out of tolerance {rtol:g}; "
            f"worst at flat index {k}: gpu={gpu.reshape(-1)[k]!r} ref={ref.reshape(-1)[k]!r} "
            f"envelope=[{lo.reshape(-1)[k]!r}, {hi.reshape(-1)[k]!r}] rms(ref)={rms:g}")
    strict_fail = float((np.abs(gpu - ref) > bound).mean()) if ref.size else 0.0
    # whole-tensor checks.  The part of the difference that no choice at a kink explains (the
    # distance to the envelope) is bounded like an ordinary error.  Around the definition's own
    # gradient the bound grows by the width of the envelope, capped (see WIDTH_CAP).
    norm = max(float(np.linalg.norm(ref)), 1e-300)
    l2_env = float(np.linalg.norm(err)) / norm
    assert l2_env <= 3.0 * rtol, f"{what}: relative L2 distance to the kink envelope {l2_env:g} exceeds {3.0 * rtol:g}"
    l2 = float(np.linalg.norm(gpu - ref)) / norm
    width = float(np.linalg.norm(hi - lo)) / norm
    allowed = width if width_cap is None else min(width, width_cap)
    assert l2 <= 3.0 * rtol + allowed, \
        f"{what}: relative L2 error {l2:g} exceeds {3.0 * rtol:g} + {allowed:g} (envelope width {width:g})"
    return GradErr((float(err.max() / max(rms, 1e-300)), strict_fail, l2, width))


# Which tensors the strict share is asserted for.  Grid gradients (and the Splatter's per-pixel and
# prior gradients): an element sums the few samples that touch it, so a flipped unit spoils few
# elements.  Weight and bias gradients are different: a unit whose sign decision differs from the
# fp64 one (|z| below the kernel's rounding error, probability p per unit and sample) changes a
# whole row of dW by that sample's contribution, and because a row is a sum with random signs over
# ALL samples, the row's relative error is about sqrt(p / P(unit active)) whatever the number of
# samples: 2e-3 ... 4e-3 for the split-bf16 contractions (p ~ 1e-5), i.e. right at the plain
# tolerance, for a third of the elements or none.  For those tensors the envelope (every element)
# and the whole-tensor L2 bound are asserted, and the share is reported.
STRICT_SHARE_TENSORS = ("d_grid", "d_prior", "d_feats")


def assert_strict_share(worst: dict, label: str, max_strict_fail: float):
    """Besides lying inside the envelope, all but a small share of the elements of a grid-like
    gradient tensor must meet the plain tolerance around the definition's gradient."""
    for k, v in worst.items():
        if isinstance(v, GradErr) and k.startswith(STRICT_SHARE_TENSORS):
            assert v.strict_fail <= max_strict_fail, (
                f"{label} {k}: {v.strict_fail:.2%} of the elements miss the plain tolerance "
                f"(allowed {max_strict_fail:.2%}; relative L2 error {v.l2:.2e}, envelope width {v.width:.2e})")


def summary(worst: dict) -> str:
    """One line for logs: worst forward error / rms, and over the gradient tensors the worst
    distance to the envelope / rms, relative L2 error around the definition's gradient, and
    share of elements outside the plain tolerance."""
    fwd = max((v for v in worst.values() if not isinstance(v, GradErr)), default=0.0)
    g = [v for v in worst.values() if isinstance(v, GradErr)]
    if not g:
        return f"forward err/rms {fwd:.1e}"
    grid = [v for k, v in worst.items() if isinstance(v, GradErr) and k.startswith(STRICT_SHARE_TENSORS)]
    par = [v for k, v in worst.items() if isinstance(v, GradErr) and not k.startswith(STRICT_SHARE_TENSORS)]
    share = lambda vs: f"{max((v.strict_fail for v in vs), default=0.0):.2%}"
    return (f"forward err/rms {fwd:.1e}; gradients: outside envelope/rms {max(v.env for v in g):.1e}, "
            f"L2 error vs definition {max(v.l2 for v in g):.1e}, strict-miss share grid {share(grid)} / "
            f"parameters {share(par)} (envelope width up to {max(v.width for v in g):.1e})")


def mse_upstream(rgb64: np.ndarray, target: np.ndarray, scene=None, n_scenes: int = 1) -> np.ndarray:
    """d(loss)/d(rgb) of the mean-squared error to `target` (mean over the rays of a scene
    and the 3 channels, summed over scenes), as float32 — the value both sides receive."""
    m = rgb64.shape[0]
    if scene is None or n_scenes == 1:
        per = np.full(m, m, dtype=np.float64)
    else:
        counts = np.bincount(scene, minlength=n_scenes).astype(np.float64)
        per = counts[scene]
    return (2.0 * (rgb64 - target.astype(np.float64)) / (3.0 * per[:, None])).astype(np.float32)


def run_gpu(lp, inp, p_rgb, p_alpha=None, p_depth=None, math_mode=0, device="cuda:0", grid_dtype=None):
    """Forward + backward on the GPU through the C ABI; everything returned as numpy.
    grid_dtype: torch dtype the grid is STORED in on the GPU (gradients stay float32)."""
    import torch
    grid, mlp, rays, bg = lp.to_device(inp, device)
    if grid_dtype is not None:
        grid.data = [t.to(grid_dtype) for t in grid.data]
    rgb, alpha, depth, cache = lp.render_fwd(grid, mlp, rays, bg, math_mode)
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    d_grid, dW, db = lp.render_bwd(grid, mlp, rays, bg, up(p_rgb), cache, up(p_alpha), up(p_depth), math_mode)
    torch.cuda.synchronize()
    cpu = lambda t: t.cpu().numpy()
    return dict(rgb=cpu(rgb), alpha=cpu(alpha), depth=cpu(depth), cache=cpu(cache),
                d_grid=[cpu(t) for t in d_grid], dW=[cpu(t) for t in dW], db=[cpu(t) for t in db])


def check_case(lp, oracle, inp, math_mode=0, aux_grads=True, seed=0, label="", max_strict_fail=MAX_STRICT_FAIL, grid_dtype=None):
    """Full parity of one problem: forward outputs and every gradient tensor."""
    import lp_inputs
    prob = oracle.Problem(inp)
    o_rgb, o_alpha, o_depth = oracle.render_fwd(prob)
    p_rgb = mse_upstream(o_rgb, inp.target, inp.scene, inp.n_scenes)
    p_alpha = p_depth = None
    if aux_grads:
        p_alpha, p_depth = lp_inputs.upstream_grads(inp.n_rays, 77 + seed)
    o_dg, o_dW, o_db = oracle.render_bwd(prob, p_rgb, p_alpha, p_depth)
    c = KINK_BAND
    upper = oracle.render_bwd(prob, p_rgb, p_alpha, p_depth, kink_band=c, kink_side=+1)
    lower = oracle.render_bwd(prob, p_rgb, p_alpha, p_depth, kink_band=c, kink_side=-1)
    env = lambda i, j: (lower[i][j], upper[i][j])
    g = run_gpu(lp, inp, p_rgb, p_alpha, p_depth, math_mode, grid_dtype=grid_dtype)
    worst = {}
    worst["rgb"] = close(g["rgb"], o_rgb, FWD_RTOL, f"{label} rgb")
    worst["alpha"] = close(g["alpha"], o_alpha, FWD_RTOL, f"{label} alpha")
    worst["depth"] = close(g["depth"], o_depth, FWD_RTOL, f"{label} depth")
    for p, (a, b) in enumerate(zip(g["d_grid"], o_dg)):
        worst[f"d_grid{p}"] = close_envelope(a, b, *env(0, p), BWD_RTOL, f"{label} d_grid[{p}]")
    for l, (a, b) in enumerate(zip(g["dW"], o_dW)):
        worst[f"dW{l}"] = close_envelope(a, b, *env(1, l), BWD_RTOL, f"{label} dW[{l}]")
    for l, (a, b) in enumerate(zip(g["db"], o_db)):
        worst[f"db{l}"] = close_envelope(a, b, *env(2, l), BWD_RTOL, f"{label} db[{l}]")
    assert_strict_share(worst, label, max_strict_fail)
    return worst


# ---- the two-MLP, view-dependent decoder ----------------------------------------------------

def run_gpu_dec(lp, inp, p_out, p_alpha=None, p_depth=None, math_mode=0, device="cuda:0", grid_dtype=None):
    """Forward + backward with `inp.decoder` through the C ABI; everything returned as numpy.
    grid_dtype: torch dtype the grid is STORED in on the GPU (gradients stay float32)."""
    import torch
    grid, _, rays, bg = lp.to_device(inp, device)
    if grid_dtype is not None:
        grid.data = [t.to(grid_dtype) for t in grid.data]
    dec = lp.decoder_to_device(inp.decoder, device)
    out, alpha, depth, cache = lp.render_dec_fwd(grid, dec, rays, bg, math_mode)
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    d_grid, dWs, dbs, dWv, dbv = lp.render_dec_bwd(grid, dec, rays, bg, up(p_out), cache, up(p_alpha), up(p_depth),
                                                   math_mode)
    torch.cuda.synchronize()
    cpu = lambda t: t.cpu().numpy()
    lst = lambda ts: [cpu(t) for t in ts]
    return dict(out=cpu(out), alpha=cpu(alpha), depth=cpu(depth), d_grid=lst(d_grid), dWs=lst(dWs), dbs=lst(dbs),
                dWv=lst(dWv), dbv=lst(dbv))


def check_case_dec(lp, oracle, inp, math_mode=0, aux_grads=True, seed=0, label="", max_strict_fail=MAX_STRICT_FAIL,
                   grid_dtype=None):
    """Full parity of one problem with the two-MLP decoder: outputs and every gradient tensor."""
    import lp_inputs
    prob = oracle.Problem(inp)
    o_out, o_alpha, o_depth = oracle.render2_fwd(prob)
    f = o_out.shape[1]
    p_out = mse_upstream(o_out, inp.target, inp.scene, inp.n_scenes) * np.float32(3.0 / f)
    p_alpha = p_depth = None
    if aux_grads:
        p_alpha, p_depth = lp_inputs.upstream_grads(inp.n_rays, 77 + seed)
    ref = oracle.render2_bwd(prob, p_out, p_alpha, p_depth)
    upper = oracle.render2_bwd(prob, p_out, p_alpha, p_depth, kink_band=KINK_BAND, kink_side=+1)
    lower = oracle.render2_bwd(prob, p_out, p_alpha, p_depth, kink_band=KINK_BAND, kink_side=-1)
    g = run_gpu_dec(lp, inp, p_out, p_alpha, p_depth, math_mode, grid_dtype=grid_dtype)
    worst = {"out": close(g["out"], o_out, FWD_RTOL, f"{label} out"),
             "alpha": close(g["alpha"], o_alpha, FWD_RTOL, f"{label} alpha"),
             "depth": close(g["depth"], o_depth, FWD_RTOL, f"{label} depth")}
    for i, name in enumerate(("d_grid", "dWs", "dbs", "dWv", "dbv")):
        for j, a in enumerate(g[name]):
            worst[f"{name}{j}"] = close_envelope(a, ref[i][j], lower[i][j], upper[i][j], BWD_RTOL,
                                                 f"{label} {name}[{j}]")
    assert_strict_share(worst, label, max_strict_fail)
    return worst


# ---- Splatter ---------------------------------------------------------------------------------

def check_case_splat(lp, oracle, sp, seed=0, label="", max_strict_fail=MAX_STRICT_FAIL, width_cap=WIDTH_CAP):
    """Splatter parity: normalised structure, weight sums and every gradient against the oracle."""
    import torch
    prob = oracle.SplatProblem(sp)
    o_theta, o_w = oracle.splat_fwd(prob)
    rng = np.random.default_rng(900 + seed)
    G = [(rng.standard_normal(t.shape) / max(1, t.size) ** 0.5).astype(np.float32) for t in o_theta]
    ref = oracle.splat_bwd(prob, o_w, G)
    upper = oracle.splat_bwd(prob, o_w, G, kink_band=KINK_BAND, kink_side=+1)
    lower = oracle.splat_bwd(prob, o_w, G, kink_band=KINK_BAND, kink_side=-1)
    target, rays, splat = lp.splat_to_device(sp)
    theta, theta_w = lp.splat_fwd(target, rays, splat)
    # the backward takes the oracle's weight sums rounded to float32?  No: the library's own, as a caller would
    d_feats, d_prior, dW, db = lp.splat_bwd(target, rays, splat, theta_w, [torch.from_numpy(g).to("cuda:0") for g in G])
    torch.cuda.synchronize()
    cpu = lambda t: t.cpu().numpy()
    worst = {}
    for p in range(len(o_theta)):
        g_w, g_t = cpu(theta_w[p]), cpu(theta[p])
        worst[f"theta_w{p}"] = close(g_w, o_w[p], FWD_RTOL, f"{label} theta_w[{p}]")
        # the sums the kernel accumulates, then the normalised result: both at the plain tolerance
        # (the corner weights keep their relative accuracy however small they are: f and 1 - f are
        # both rounded from the fp64 index)
        worst[f"sum{p}"] = close(g_t.astype(np.float64) * g_w[..., None], o_theta[p] * o_w[p][..., None], FWD_RTOL,
                                 f"{label} theta[{p}] * theta_w[{p}]")
        worst[f"theta{p}"] = close(g_t, o_theta[p], FWD_RTOL, f"{label} theta[{p}]")
    flat = lambda r: [("d_feats", r[0])] + [(f"d_prior{i}", a) for i, a in enumerate(r[1])] \
        + [(f"dW{i}", a) for i, a in enumerate(r[2])] + [(f"db{i}", a) for i, a in enumerate(r[3])]
    gpu = [d_feats] + list(d_prior) + list(dW) + list(db)
    for (name, r), (_, lo), (_, hi), g in zip(flat(ref), flat(lower), flat(upper), gpu):
        worst[name] = close_envelope(cpu(g), r, lo, hi, BWD_RTOL, f"{label} {name}", width_cap=width_cap)
    assert_strict_share(worst, label, max_strict_fail)
    return worst
