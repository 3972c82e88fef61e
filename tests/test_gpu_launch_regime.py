"""GPU parity in the launch regime the benchmark runs: more rays than resident wavefronts.

With at most 1024 rays every wavefront of the matrix-core backward marches one ray and the ray
groups are visited in order.  Beyond that a wavefront marches several rays in a row (carrying
the next ray's first samples over the ray boundary, prefetching its features), and beyond
31 676 rays the ray groups are visited in a scrambled order.  These cases put every backward
kernel family into that regime and compare forward outputs and every gradient tensor with the
CPU oracle, element by element (Section 3.4, Eq. (2)): once with a strided subset of the rays
and once with a contiguous block of pixels, whose neighbouring rays add into the same
gradient lines within one launch."""
import numpy as np
import pytest

import lp_inputs
from lp_inputs import TRIPLANE, VOXEL

from parity import check_case, check_case_dec, summary

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _pixel_block(image: int, lo: int, hi: int) -> np.ndarray:
    v, u = np.meshgrid(np.arange(lo, hi), np.arange(lo, hi), indexing="ij")
    return (v * image + u).reshape(-1).astype(np.int64)


@pytest.mark.parametrize("pick", ["every_16th_ray", "block_of_200x200_pixels"])
def test_large_config_with_40000_rays(lp, oracle, pick):
    """Largest configuration (voxel 256^3 x 16, MLP 16-64-64-4, 512 samples per ray), 40 000 rays:
    10 000 ray groups, about 10 rays per wavefront, scrambled group order, the next step's and the
    next ray's texel loads issued early."""
    inp = lp_inputs.make_inputs("large")
    idx = np.arange(0, inp.n_rays, 16) if pick == "every_16th_ray" else _pixel_block(800, 300, 500)
    assert idx.size == 40000
    sub = inp.subset(idx)
    worst = check_case(lp, oracle, sub, lp.LP_MATH_BF16X3, label=f"large {pick}")
    print(summary(worst), flush=True)


@pytest.mark.parametrize("pick", ["strided", "block"])
def test_voxel_config_with_many_rays(lp, oracle, pick):
    """Voxel 64^3 x 32 configuration: 36 864 rays strided over the four views, or a 192 x 192 pixel
    block of the first view (32 channels: corner carry-over across cells, no cross-step prefetch)."""
    inp = lp_inputs.make_inputs("voxel")
    idx = lp_inputs.strided_ray_subset(inp.n_rays, 36864, offset=3) if pick == "strided" else _pixel_block(256, 32, 224)
    worst = check_case(lp, oracle, inp.subset(idx), lp.LP_MATH_BF16X3, label=f"voxel {pick}")
    print(summary(worst), flush=True)


def test_batched_config_block_of_each_scene(lp, oracle):
    """Batched triplanes (8 scenes x 3 x 256^2 x 32): a 64 x 64 pixel block of the first view of
    every scene, 32 768 rays."""
    inp = lp_inputs.make_inputs("batched")
    per_scene = 4 * 256 * 256
    idx = np.concatenate([b * per_scene + _pixel_block(256, 96, 160) for b in range(8)])
    worst = check_case(lp, oracle, inp.subset(idx), lp.LP_MATH_BF16X3, label="batched blocks")
    print(summary(worst), flush=True)


@pytest.mark.parametrize("dims", [(16, 64, 64, 4), (16, 32, 4)])
def test_triplane_16_channels_with_many_rays(lp, oracle, dims):
    """16-channel triplane (the tiny configuration's grid kind) with more rays than wavefronts: the
    features of the next step are sampled before the current step's scatter, without early loads."""
    w = lp_inputs.WORKLOADS["single_scene"]
    rays = lp_inputs.make_inputs("single_scene", with_grid=False)
    small = lp_inputs.make_small(TRIPLANE, channels=16, res=(48, 40, 44), mlp_dims=dims, n_rays=8, samples=96,
                                 seed=131, grid_std=0.3, aabb_min=(-2.75,) * 3, aabb_max=(2.75,) * 3)
    idx = _pixel_block(w.image, 24, 104)         # 6400 neighbouring rays of a 128 x 128 image
    import dataclasses
    inp = dataclasses.replace(small, origins=np.ascontiguousarray(rays.origins[idx]),
                              dirs=np.ascontiguousarray(rays.dirs[idx]), near=np.ascontiguousarray(rays.near[idx]),
                              far=np.ascontiguousarray(rays.far[idx]), scene=None,
                              target=np.ascontiguousarray(rays.target[idx]))
    worst = check_case(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"triplane16 {dims}")
    print(summary(worst), flush=True)


@pytest.mark.parametrize("dtype", ["float32", "bfloat16"])
def test_two_wave_backward_with_contract_coordinates_and_many_rays(lp, oracle, dtype):
    """The two-wave backward's other instantiations (contract coordinates compiled in for fp32 grids, a
    run-time branch for grids stored in bf16) with several rays per pair of waves: a 16-channel voxel
    grid, MLP 16-64-64-4, a block of 6 400 neighbouring rays that start inside the unit cube."""
    import dataclasses
    import torch
    w = lp_inputs.WORKLOADS["single_scene"]
    rays = lp_inputs.make_inputs("single_scene", with_grid=False)
    small = lp_inputs.make_small(VOXEL, channels=16, res=(48, 40, 44), mlp_dims=(16, 64, 64, 4), n_rays=8, samples=96,
                                 seed=137, grid_std=0.3)
    idx = _pixel_block(w.image, 24, 104)
    inp = dataclasses.replace(small, origins=np.ascontiguousarray(rays.origins[idx] * 0.3),
                              dirs=np.ascontiguousarray(rays.dirs[idx]), near=np.ascontiguousarray(rays.near[idx] * 0.0),
                              far=np.ascontiguousarray(rays.far[idx] * 3.0), scene=None,
                              target=np.ascontiguousarray(rays.target[idx]), contract_a=1.3)
    tdt = getattr(torch, dtype)
    if dtype != "float32":
        stored = [torch.from_numpy(g).to(tdt) for g in inp.grid]
        inp = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored])
    worst = check_case(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"two-wave contract {dtype}",
                       grid_dtype=None if dtype == "float32" else tdt)
    print(summary(worst), flush=True)


@pytest.mark.parametrize("pick", ["every_2nd_ray", "block_of_96x96_pixels"])
def test_hash_workload_with_many_rays(lp, oracle, pick):
    """The hash-table workload (2^19 entries x 16 channels over a 128^3 lattice, MLP 16-64-64-4, 128
    samples per ray) on the matrix-core kernels with about eight rays per wavefront: neighbouring
    rays add into the same table entries within one launch, colliding corners included."""
    inp = lp_inputs.make_inputs("hash")
    idx = np.arange(0, inp.n_rays, 2) if pick == "every_2nd_ray" else _pixel_block(128, 16, 112)
    sub = inp.subset(idx)
    grid, mlp, _, _ = lp.to_device(sub)
    assert lp.lp_has_fast_path(grid, mlp)
    worst = check_case(lp, oracle, sub, lp.LP_MATH_BF16X3, label=f"hash {pick}")
    print(summary(worst), flush=True)


def test_hexplane_workload_with_many_rays(lp, oracle):
    """The HexPlane workload (three 128^2 spatial and three 128 x 16 space-time planes of 16 channels,
    MLP 16-64-64-4, 128 samples per ray, a frame time per ray) on the matrix-core kernels: a 96 x 96
    pixel block, about nine rays per wavefront, neighbouring rays adding into the same texels."""
    inp = lp_inputs.make_inputs("hexplane")
    sub = inp.subset(_pixel_block(128, 16, 112))
    grid, mlp, _, _ = lp.to_device(sub)
    assert lp.lp_has_fast_path(grid, mlp)
    # (an entry of the small space-time planes sums some hundred thousand sample contributions, so a
    # larger share of their entries contains at least one ReLU decision inside the kink band: seen 3.8 %)
    worst = check_case(lp, oracle, sub, lp.LP_MATH_BF16X3, label="hexplane block", max_strict_fail=0.08)
    print(summary(worst), flush=True)


def test_contract_workload_with_many_rays(lp, oracle):
    """The paper's experimental Renderer shape with contract coordinates: every second ray of the
    256^2 image (32 768 rays x 384 samples, 160^3 x 32 voxels)."""
    inp = lp_inputs.make_inputs("contract")
    worst = check_case(lp, oracle, inp.subset(np.arange(0, inp.n_rays, 2)), lp.LP_MATH_BF16X3, label="contract half")
    print(summary(worst), flush=True)


def test_decoder_workload_with_many_rays(lp, oracle):
    """Merged two-MLP decoder on the matrix-core kernels (16 grid channels + direction inputs in the
    second lane group): a 128 x 128 pixel block, 16 384 rays x 256 samples."""
    inp = lp_inputs.make_inputs("decoder")
    sub = inp.subset(_pixel_block(256, 64, 192))
    worst = check_case_dec(lp, oracle, sub, lp.LP_MATH_BF16X3, label="decoder block")
    print(summary(worst), flush=True)


def test_two_chain_decoder_with_many_rays(lp, oracle):
    """The decoder at the paper's size (two chains, two-pass backward): every second ray of the
    256^2 image, 32 768 rays x 384 samples with contract coordinates."""
    inp = lp_inputs.make_inputs("decoder_paper")
    sub = inp.subset(np.arange(0, inp.n_rays, 2))
    worst = check_case_dec(lp, oracle, sub, lp.LP_MATH_BF16X3, label="decoder_paper half")
    print(summary(worst), flush=True)
