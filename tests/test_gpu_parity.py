"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs, element by element.  Tolerances: forward 1e-4, gradients 1e-3
(fp32 relative, per tensor: |gpu - ref| <= rtol |ref| + rtol rms(ref))."""
import dataclasses

import numpy as np
import pytest

import lp_inputs
from lp_inputs import TRIPLANE, VOXEL

from parity import BWD_RTOL, FWD_RTOL, check_case, close, mse_upstream, run_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _modes(lp, inp):
    """Math modes to test for a problem: the generic kernels always, the matrix-core
    kernels when they cover the shape."""
    import torch
    grid, mlp, _, _ = lp.to_device(dataclasses.replace(inp, origins=inp.origins[:1], dirs=inp.dirs[:1],
                                                       near=inp.near[:1], far=inp.far[:1],
                                                       scene=None if inp.scene is None else inp.scene[:1]))
    modes = [lp.LP_MATH_GENERIC]
    if lp.lp_has_fast_path(grid, mlp):
        modes.append(lp.LP_MATH_BF16X3)
    return modes


# ------------------------------------------------------------------ small problems, odd sizes

@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_small_odd_shapes_generic(lp, oracle, kind):
    """Channel count, widths, ray count and sample count that fit no tile: generic kernels."""
    inp = lp_inputs.make_small(kind, channels=5, res=(6, 5, 7), mlp_dims=(5, 7, 9, 4), n_rays=131,
                               samples=37, seed=41, n_scenes=3)
    print(check_case(lp, oracle, inp, lp.LP_MATH_GENERIC, label=f"small kind={kind}"), flush=True)


def test_wide_mlp_on_the_generic_kernels(lp, oracle):
    """An MLP whose parameters no longer fit twice into LDS: the generic backward accumulates the
    weight gradients in its workspace records; one that does not fit at all is refused."""
    inp = lp_inputs.make_small(VOXEL, channels=24, res=(6, 5, 7), mlp_dims=(24, 96, 96, 4), n_rays=90, samples=21,
                               seed=45, grid_std=0.3)
    print(check_case(lp, oracle, inp, lp.LP_MATH_GENERIC, label="wide generic"), flush=True)
    # wider still: the activation columns only fit for a partial wavefront of 8 rays, fewer lanes than the
    # grid has channels (the gradient scatter across lanes then takes several channels per lane)
    inp = lp_inputs.make_small(VOXEL, channels=24, res=(6, 5, 7), mlp_dims=(24, 160, 160, 4), n_rays=43, samples=11,
                               seed=46, grid_std=0.3)
    print(check_case(lp, oracle, inp, lp.LP_MATH_GENERIC, label="wider generic"), flush=True)
    huge = lp_inputs.make_small(VOXEL, channels=8, mlp_dims=(8, 256, 256, 4), n_rays=8)
    grid, mlp, rays, bg = lp.to_device(huge)
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_fwd(grid, mlp, rays, bg, lp.LP_MATH_GENERIC)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_clamped_samples_outside_the_box(lp, oracle, kind):
    """Box [-0.4, 0.4]^3 is much smaller than the ray span: most samples clamp to the border."""
    inp = lp_inputs.make_small(kind, channels=16, res=(9, 8, 10), mlp_dims=(16, 32, 4), n_rays=70,
                               samples=65, seed=43, aabb_min=(-0.4, -0.4, -0.4), aabb_max=(0.4, 0.4, 0.4))
    for mode in _modes(lp, inp):
        print(mode, check_case(lp, oracle, inp, mode, label=f"clamp kind={kind} mode={mode}"), flush=True)


@pytest.mark.parametrize("kind,channels,dims", [
    (VOXEL, 16, (16, 64, 64, 4)), (VOXEL, 32, (32, 64, 4)),
    (TRIPLANE, 16, (16, 32, 4)), (TRIPLANE, 32, (32, 64, 64, 4)), (TRIPLANE, 32, (32, 32, 32, 4)),
])
@pytest.mark.parametrize("samples", [1, 64, 150])
def test_config_shapes_ragged(lp, oracle, kind, channels, dims, samples):
    """The MLP / grid shapes of the five configurations on small grids, with ray counts and
    sample counts that leave ragged tails (several tiles plus a partial one)."""
    inp = lp_inputs.make_small(kind, channels=channels, res=(12, 10, 11), mlp_dims=dims, n_rays=203,
                               samples=samples, seed=47 + samples, n_scenes=2, grid_std=0.3,
                               aabb_min=(-1.5, -1.5, -1.5), aabb_max=(1.5, 1.5, 1.5))
    for mode in _modes(lp, inp):
        print(mode, check_case(lp, oracle, inp, mode, label=f"kind={kind} dims={dims} S={samples} mode={mode}"),
              flush=True)


def test_one_wave_backward_of_the_two_wave_shape():
    """The shape whose backward runs as a pair of waves per ray (voxel grid, 16 channels, MLP
    16-64-64-4) also has the one-wave kernel; LP_BWD_ONE_WAVE=1 selects it when the library is loaded,
    hence the child process.  Same parity bar."""
    import os, subprocess, sys
    env = dict(os.environ, LP_BWD_ONE_WAVE="1")
    test = os.path.abspath(__file__) + "::test_config_shapes_ragged[150-0-16-dims0]"
    res = subprocess.run([sys.executable, "-m", "pytest", test, "-m", "gpu", "-x", "-q", "--timeout", "200",
                          "--timeout-method", "thread", "-p", "no:cacheprovider"],
                         env=env, capture_output=True, text=True, timeout=400)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    assert "1 passed" in res.stdout


# ------------------------------------------------------------------ contract coordinates

@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("a_scale", [1.0, 1.6])
def test_contract_coordinates(lp, oracle, kind, a_scale):
    """Rays that start inside the unit cube and run far beyond it (the contraction's two
    branches and the seam between them), generic and matrix-core kernels."""
    small = lp_inputs.make_small(kind, channels=5, res=(6, 5, 7), mlp_dims=(5, 7, 4), n_rays=67, samples=41,
                                 seed=61, origin_radius=0.8, near=(0.0, 0.3), far=(6.0, 30.0))
    small = dataclasses.replace(small, contract_a=a_scale)
    print(check_case(lp, oracle, small, lp.LP_MATH_GENERIC, label=f"contract small kind={kind}"), flush=True)
    inp = lp_inputs.make_small(kind, channels=16 if kind == VOXEL else 32, res=(14, 12, 13),
                               mlp_dims=(16, 64, 64, 4) if kind == VOXEL else (32, 64, 4), n_rays=150,
                               samples=100, seed=62, grid_std=0.3, origin_radius=1.4, near=(0.0, 0.3),
                               far=(6.0, 30.0))
    inp = dataclasses.replace(inp, contract_a=a_scale)
    for mode in _modes(lp, inp):
        print(mode, check_case(lp, oracle, inp, mode, label=f"contract kind={kind} a={a_scale} mode={mode}"),
              flush=True)


def test_contract_workload_on_a_ray_subset(lp, oracle):
    """The paper's experimental Renderer shape (160^3 x 32, width-64 MLP, 384 points per ray,
    contract coordinates), a strided subset of its rays."""
    inp = lp_inputs.make_inputs("contract")
    sub = inp.subset(lp_inputs.strided_ray_subset(inp.n_rays, 1024, offset=5))
    for mode in _modes(lp, sub)[-1:]:
        print(mode, check_case(lp, oracle, sub, mode, label=f"contract subset mode={mode}", max_strict_fail=0.03),
              flush=True)



# ------------------------------------------------------------------ reduced-precision grid storage

@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("dtype", ["bfloat16", "float16"])
def test_reduced_precision_grid_storage(lp, oracle, kind, dtype):
    """Grid stored in bf16 / fp16 (half the bytes per sample), gradients in fp32.  The stored
    values are exactly representable, so the oracle simply receives them widened: same tolerances."""
    import torch
    tdt = getattr(torch, dtype)
    for channels, dims in ((5, (5, 7, 4)), (16, (16, 32, 4)), (16, (16, 64, 64, 4)), (32, (32, 64, 64, 4))):
        inp = lp_inputs.make_small(kind, channels=channels, res=(9, 8, 10), mlp_dims=dims, n_rays=400, samples=70,
                                   seed=59, n_scenes=2, grid_std=0.4)
        stored = [torch.from_numpy(g).to(tdt) for g in inp.grid]
        widened = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored])
        # (two hidden layers of 64 on this 9x8x10 grid: every texel collects the kink decisions of many
        # samples; 2.04 % of the texels were seen outside the plain tolerance, all inside the envelope)
        share = 0.04 if dims == (16, 64, 64, 4) else 0.02
        for mode in _modes(lp, widened):
            print(mode, check_case(lp, oracle, widened, mode, label=f"{dtype} kind={kind} C={channels} mode={mode}",
                                   grid_dtype=tdt, max_strict_fail=share), flush=True)
    # with contract coordinates (rays from inside the unit cube to far beyond it)
    inp = lp_inputs.make_small(kind, channels=32, res=(14, 12, 13), mlp_dims=(32, 64, 64, 4), n_rays=150, samples=100,
                               seed=60, grid_std=0.3, origin_radius=1.4, near=(0.0, 0.3), far=(6.0, 30.0))
    stored = [torch.from_numpy(g).to(tdt) for g in inp.grid]
    widened = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored], contract_a=1.3)
    assert len(_modes(lp, widened)) == 2
    for mode in _modes(lp, widened):
        print(mode, check_case(lp, oracle, widened, mode, label=f"{dtype} contract kind={kind} mode={mode}",
                               grid_dtype=tdt), flush=True)
    # the shape whose backward runs as two waves per ray (voxel grids), with the contraction
    inp = lp_inputs.make_small(kind, channels=16, res=(14, 12, 13), mlp_dims=(16, 64, 64, 4), n_rays=150, samples=100,
                               seed=63, grid_std=0.3, origin_radius=1.4, near=(0.0, 0.3), far=(6.0, 30.0))
    stored = [torch.from_numpy(g).to(tdt) for g in inp.grid]
    widened = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored], contract_a=1.3)
    for mode in _modes(lp, widened):
        print(mode, check_case(lp, oracle, widened, mode, label=f"{dtype} contract 16ch kind={kind} mode={mode}",
                               grid_dtype=tdt), flush=True)

# ------------------------------------------------------------------ the five configurations

def test_config_tiny_full(lp, oracle):
    inp = lp_inputs.make_inputs("tiny")
    for mode in _modes(lp, inp):
        print(mode, check_case(lp, oracle, inp, mode, label=f"tiny mode={mode}", max_strict_fail=0.03), flush=True)


def test_config_single_scene_full(lp, oracle):
    inp = lp_inputs.make_inputs("single_scene")
    for mode in _modes(lp, inp)[-1:]:
        print(mode, check_case(lp, oracle, inp, mode, aux_grads=False, label=f"single_scene mode={mode}", max_strict_fail=0.03),
              flush=True)


@pytest.mark.parametrize("name,n_keep", [("voxel", 1536), ("batched", 1024), ("large", 768)])
def test_config_large_on_ray_subsets(lp, oracle, name, n_keep):
    """Configurations 3-5: the full grid and MLP, a deterministic strided subset of the rays
    run as its own ray set on both sides (rays are independent; gradients are sums over rays)."""
    inp = lp_inputs.make_inputs(name)
    sub = inp.subset(lp_inputs.strided_ray_subset(inp.n_rays, n_keep, offset=3))
    for mode in _modes(lp, sub)[-1:]:
        print(mode, check_case(lp, oracle, sub, mode, label=f"{name} subset mode={mode}", max_strict_fail=0.03), flush=True)


# ------------------------------------------------------------------ edge cases

def test_zero_rays_is_a_noop(lp):
    import torch
    inp = lp_inputs.make_small(VOXEL, channels=16, mlp_dims=(16, 32, 4))
    grid, mlp, rays, bg = lp.to_device(inp.subset(np.arange(0)))
    rgb, alpha, depth, cache = lp.render_fwd(grid, mlp, rays, bg)
    d_rgb = torch.zeros((0, 3), device="cuda:0")
    d_grid, dW, db = lp.render_bwd(grid, mlp, rays, bg, d_rgb, cache)
    torch.cuda.synchronize()
    assert rgb.shape == (0, 3) and all(float(t.abs().sum()) == 0.0 for t in d_grid + dW + db)


def test_optional_outputs_may_be_null(lp):
    """alpha, depth and the ray cache are optional outputs of the forward, in both kernel families."""
    import torch
    inp = lp_inputs.make_small(VOXEL, channels=16, mlp_dims=(16, 32, 4), n_rays=77, samples=40, seed=5)
    grid, mlp, rays, bg = lp.to_device(inp)
    for mode in (lp.LP_MATH_GENERIC, lp.LP_MATH_BF16X3):
        full = lp.render_fwd(grid, mlp, rays, bg, mode)
        rgb = torch.empty_like(full[0])
        lp.lp_render_fwd(grid, mlp, rays, bg, rgb, None, None, None, mode)
        torch.cuda.synchronize()
        assert torch.equal(rgb, full[0])


def test_zero_density_renders_background_exactly(lp):
    import torch
    inp = lp_inputs.make_small(VOXEL, channels=16, mlp_dims=(16, 32, 4), n_rays=100, samples=70)
    inp.weights[-1][0, :] = 0.0
    inp.biases[-1][0] = -200.0
    for mode in _modes(lp, inp):
        grid, mlp, rays, bg = lp.to_device(inp)
        rgb, alpha, depth, _ = lp.render_fwd(grid, mlp, rays, bg, mode)
        torch.cuda.synchronize()
        assert float(alpha.abs().max()) == 0.0 and float(depth.abs().max()) == 0.0
        assert torch.equal(rgb, torch.tensor(bg, device="cuda:0").expand_as(rgb))


def test_errors_through_the_abi(lp):
    import torch
    inp = lp_inputs.make_small(VOXEL, channels=16, mlp_dims=(16, 32, 4), n_rays=10)
    grid, mlp, rays, bg = lp.to_device(inp)
    rgb, alpha, depth, cache = lp.render_fwd(grid, mlp, rays, bg)
    d_rgb = torch.zeros_like(rgb)
    small_ws = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_bwd(grid, mlp, rays, bg, d_rgb, cache, workspace=small_ws)
    assert e.value.status == lp.LP_ERR_WORKSPACE
    odd = lp_inputs.make_small(VOXEL, channels=5, mlp_dims=(5, 7, 4), n_rays=10)
    g2, m2, r2, _ = lp.to_device(odd)
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_fwd(g2, m2, r2, bg, lp.LP_MATH_BF16X3)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED
    for bad in (-0.5, 2.5, float("nan")):
        with pytest.raises(lp.LightplaneError) as e:
            lp.render_fwd(dataclasses.replace(grid, contract_a=bad), mlp, rays, bg)
        assert e.value.status == lp.LP_ERR_INVALID_ARG


def test_forward_is_bit_reproducible_and_gradients_accumulate(lp):
    import torch
    inp = lp_inputs.make_inputs("tiny")
    grid, mlp, rays, bg = lp.to_device(inp)
    a = lp.render_fwd(grid, mlp, rays, bg)
    b = lp.render_fwd(grid, mlp, rays, bg)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    d_rgb = torch.randn_like(a[0]) / rays.n_rays
    g1 = lp.render_bwd(grid, mlp, rays, bg, d_rgb, a[3])
    # second call accumulates into the same buffers: result doubles
    ws = torch.empty(lp.lp_bwd_workspace_bytes(grid, mlp, rays), dtype=torch.uint8, device="cuda:0")
    d_grid = [t.clone() for t in g1[0]]; dW = [t.clone() for t in g1[1]]; db = [t.clone() for t in g1[2]]
    lp.lp_render_bwd(grid, mlp, rays, bg, d_rgb, None, None, a[3], d_grid, dW, db, ws)
    torch.cuda.synchronize()
    for once, twice in zip(g1[0] + g1[1] + g1[2], d_grid + dW + db):
        close(twice.cpu().numpy(), 2.0 * once.cpu().numpy().astype(np.float64), BWD_RTOL, "accumulate")


def test_activation_memory_independent_of_samples(lp):
    """Section 3.4: the only state kept between forward and backward is one scalar per ray;
    the library allocates nothing and its workspace does not grow with S."""
    import gc
    import torch
    inp = lp_inputs.make_inputs("tiny")
    peaks, ws_bytes = [], []
    gc.collect()   # tensors of earlier tests still held by reference cycles would be freed mid-measurement
    for s in (64, 256):
        q = dataclasses.replace(inp, samples=s)
        grid, mlp, rays, bg = lp.to_device(q)
        ws_bytes.append(lp.lp_bwd_workspace_bytes(grid, mlp, rays))
        d_rgb = torch.zeros((rays.n_rays, 3), device="cuda:0")
        torch.cuda.synchronize(); torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        out = lp.render_fwd(grid, mlp, rays, bg)
        lp.render_bwd(grid, mlp, rays, bg, d_rgb, out[3])
        torch.cuda.synchronize()
        peaks.append(torch.cuda.max_memory_allocated() - base)
        del out
    assert ws_bytes[0] == ws_bytes[1]
    assert peaks[0] == peaks[1], peaks


# ------------------------------------------------------------------ full size, bench launch configuration

@pytest.fixture(scope="module")
def large_full(lp):
    """The largest configuration at full size on the GPU (640 000 rays x 512 samples), as bench.py runs it."""
    import torch
    inp = lp_inputs.make_inputs("large")
    grid, mlp, rays, bg = lp.to_device(inp)
    out = lp.render_fwd(grid, mlp, rays, bg)
    torch.cuda.synchronize()
    return inp, grid, mlp, rays, bg, out


def test_large_full_size_forward_on_sampled_rays(lp, oracle, large_full):
    """Full-size forward launch; 600 sampled rays (every 1066th, plus the first and last rays of
    the launch and of each XCD's range) against the oracle, ray by ray."""
    inp, grid, mlp, rays, bg, (rgb, alpha, depth, cache) = large_full
    m = inp.n_rays
    per_xcd = (m + 7) // 8
    edges = [x for k in range(8) for x in (k * per_xcd, min(m, (k + 1) * per_xcd) - 1)]
    idx = np.unique(np.concatenate([lp_inputs.strided_ray_subset(m, 580, offset=11), np.array(edges + [0, m - 1])]))
    o_rgb, o_alpha, o_depth = oracle.render_fwd(inp.subset(idx))
    close(rgb.cpu().numpy()[idx], o_rgb, FWD_RTOL, "large full rgb")
    close(alpha.cpu().numpy()[idx], o_alpha, FWD_RTOL, "large full alpha")
    close(depth.cpu().numpy()[idx], o_depth, FWD_RTOL, "large full depth")
    # the cached scalar is the optical depth: alpha = 1 - exp(-cache)
    np.testing.assert_allclose(1.0 - np.exp(-cache.cpu().numpy()[idx].astype(np.float64)), o_alpha, rtol=2e-4, atol=1e-6)


def test_large_full_size_gradient_properties(lp, large_full):
    """Properties that hold at any size, in the launch configuration bench.py times:
    (1) gradients are additive over a partition of the rays (the full launch equals the sum of two
        half launches, up to summation order);
    (2) the bias gradient of the output layer predicts the change of the loss under a small shift
        of those biases (central difference of two more forward launches, fp64 loss sums)."""
    import torch
    inp, grid, mlp, rays, bg, (rgb, alpha, depth, cache) = large_full
    m = inp.n_rays
    target = torch.from_numpy(inp.target).to("cuda:0")
    d_rgb = (2.0 * (rgb - target) / (3.0 * m)).contiguous()
    full = lp.render_bwd(grid, mlp, rays, bg, d_rgb, cache)
    half = m // 2 + 37

    def part(lo, hi):
        r = lp.Rays(origins=rays.origins[lo:hi].contiguous(), dirs=rays.dirs[lo:hi].contiguous(),
                    near=rays.near[lo:hi].contiguous(), far=rays.far[lo:hi].contiguous(), samples=rays.samples)
        return lp.render_bwd(grid, mlp, r, bg, d_rgb[lo:hi].contiguous(), cache[lo:hi].contiguous())

    a, b = part(0, half), part(half, m)
    torch.cuda.synchronize()
    for grp in range(3):
        for f, x, y in zip(full[grp], a[grp], b[grp]):
            f64 = f.double()
            s64 = x.double() + y.double()
            l2 = float((f64 - s64).norm() / f64.norm())
            assert l2 < 1e-4, (grp, l2)

    # directional derivative along a shift of the output-layer biases
    direction = torch.tensor([0.3, -0.5, 0.7, 0.2], device="cuda:0")
    eps = 2e-2

    def loss(shift):
        biases = [b.clone() for b in mlp.biases]
        biases[-1] = biases[-1] + shift * direction
        r, _, _, _ = lp.render_fwd(grid, lp.Mlp(weights=mlp.weights, biases=biases), rays, bg)
        return float(((r.double() - target.double()) ** 2).sum() / (3.0 * m))

    fd = (loss(+eps) - loss(-eps)) / (2 * eps)
    predicted = float((full[2][-1].double() * direction.double()).sum())
    assert predicted == pytest.approx(fd, rel=2e-3), (predicted, fd)


@pytest.mark.parametrize("name", ["voxel", "batched"])
def test_full_size_forward_and_gradient_properties_of_the_other_large_configs(lp, oracle, name):
    """The voxel (64^3 x 32, 262 144 rays x 256 samples) and batched (8 triplanes 256^2 x 32, 2 097 152 rays
    x 192 samples) configurations at full size, as bench.py launches them: the forward of 500 sampled
    rays (plus the first and last ray of every XCD's range) against the oracle ray by ray, and the
    gradient of the full launch against the sum over two parts of the rays."""
    import torch
    inp = lp_inputs.make_inputs(name)
    grid, mlp, rays, bg = lp.to_device(inp)
    rgb, alpha, depth, cache = lp.render_fwd(grid, mlp, rays, bg)
    torch.cuda.synchronize()
    m = inp.n_rays
    per_xcd = (m + 7) // 8
    edges = [x for k in range(8) for x in (k * per_xcd, min(m, (k + 1) * per_xcd) - 1)]
    idx = np.unique(np.concatenate([lp_inputs.strided_ray_subset(m, 480, offset=5), np.array(edges + [0, m - 1])]))
    o_rgb, o_alpha, o_depth = oracle.render_fwd(inp.subset(idx))
    close(rgb.cpu().numpy()[idx], o_rgb, FWD_RTOL, f"{name} full rgb")
    close(alpha.cpu().numpy()[idx], o_alpha, FWD_RTOL, f"{name} full alpha")
    close(depth.cpu().numpy()[idx], o_depth, FWD_RTOL, f"{name} full depth")

    target = torch.from_numpy(inp.target).to("cuda:0")
    d_rgb = (2.0 * (rgb - target) / (3.0 * m)).contiguous()
    full = lp.render_bwd(grid, mlp, rays, bg, d_rgb, cache)
    cut = m // 2 + 41

    def part(lo, hi):
        r = lp.Rays(origins=rays.origins[lo:hi].contiguous(), dirs=rays.dirs[lo:hi].contiguous(),
                    near=rays.near[lo:hi].contiguous(), far=rays.far[lo:hi].contiguous(), samples=rays.samples,
                    scene=None if rays.scene is None else rays.scene[lo:hi].contiguous())
        return lp.render_bwd(grid, mlp, r, bg, d_rgb[lo:hi].contiguous(), cache[lo:hi].contiguous())

    a, b = part(0, cut), part(cut, m)
    torch.cuda.synchronize()
    for grp in range(3):
        for f, x, y in zip(full[grp], a[grp], b[grp]):
            f64 = f.double()
            l2 = float((f64 - (x.double() + y.double())).norm() / f64.norm())
            assert l2 < 1e-4, (name, grp, l2)
