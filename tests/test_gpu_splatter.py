"""GPU parity of the Splatter against the CPU oracle, through the C ABI."""
import dataclasses

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HASH, TRIPLANE, VOXEL

from parity import WIDTH_CAP_SPLAT_BORDER, check_case_splat

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_naive_splatter(lp, oracle, kind):
    """No MLP: every point pushes its pixel's feature vector."""
    sp = lp_inputs.make_splat_small(kind, channels=5, res=(9, 8, 10), n_rays=131, samples=37, seed=91, n_scenes=3)
    print(check_case_splat(lp, oracle, sp, label=f"naive splat kind={kind}"), flush=True)


@pytest.mark.parametrize("hash_size", [1, 97, 4096])
@pytest.mark.parametrize("channels,hidden,prior_channels,contract", [(5, None, 0, 0.0), (16, None, 0, 1.3), (32, None, 0, 0.0),
                                                                     (6, (8, 7), 3, 0.0), (32, (64,), 32, 0.0)])
def test_splatter_into_a_hash_table(lp, oracle, hash_size, channels, hidden, prior_channels, contract):
    """Hash-table targets (and priors): colliding lattice corners pool what is pushed into them.  The naive
    Splatter runs on the wavefront-per-ray kernel for 16 or 32 channels and a table size that is a power
    of two; everything else, and every MLP, on the generic kernels."""
    kw = dict(far=(2.2, 6.0)) if contract else {}
    sp = lp_inputs.make_splat_small(HASH, channels=channels, res=(9, 8, 10), n_in=None if hidden is None else 4,
                                    hidden=hidden, n_freq=-1 if hidden is None else 1, prior_channels=prior_channels,
                                    prior_res=(7, 6, 5), n_rays=131, samples=37, seed=95 + hash_size % 7, n_scenes=2,
                                    hash_size=hash_size, prior_hash_size=211 if prior_channels else 0, **kw)
    sp = dataclasses.replace(sp, contract_a=contract)
    target, _, splat = lp.splat_to_device(sp)
    fast = hidden is None and channels in (16, 32) and hash_size & (hash_size - 1) == 0
    assert lp.lp_splat_has_fast_path(target, splat) == fast
    print(check_case_splat(lp, oracle, sp, label=f"splat hash T={hash_size} C={channels} hidden={hidden}"), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("channels", [16, 32])
@pytest.mark.parametrize("samples", [1, 32, 75])
def test_naive_splatter_wave_per_ray(lp, oracle, kind, channels, samples):
    """16 / 32 channels run on the wavefront-per-ray kernel: ragged point counts, several scenes,
    once with contract coordinates."""
    sp = lp_inputs.make_splat_small(kind, channels=channels, res=(12, 10, 11), n_rays=203, samples=samples,
                                    seed=97 + samples, n_scenes=2, far=(2.2, 6.0))
    if samples == 75:
        sp = dataclasses.replace(sp, contract_a=1.3)
    print(check_case_splat(lp, oracle, sp, label=f"naive splat fast kind={kind} C={channels} S={samples}"), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("hidden,n_freq,prior_channels", [((9,), -1, 0), ((8, 7), 1, 3), ((), 0, 2)])
def test_splatter_with_mlp(lp, oracle, kind, hidden, n_freq, prior_channels):
    """MLP on [pixel feature ; prior read ; direction encoding], ragged ray and sample counts."""
    sp = lp_inputs.make_splat_small(kind, channels=6, res=(9, 8, 10), n_in=4, hidden=hidden, n_freq=n_freq,
                                    prior_channels=prior_channels, prior_res=(7, 6, 5), n_rays=131, samples=37,
                                    seed=93, n_scenes=2)
    print(check_case_splat(lp, oracle, sp, label=f"splat kind={kind} hidden={hidden}"), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("channels,n_in,hidden,n_freq", [(16, 5, (64,), -1), (16, 16, (64, 64), 0),
                                                         (32, 7, (64, 64), 1), (32, 32, (64,), 1),
                                                         (32, 33, (64, 64), 2)])
def test_splatter_mlp_on_matrix_cores(lp, oracle, kind, channels, n_in, hidden, n_freq):
    """Prior and target of 16 / 32 channels, hidden width 64: the forward runs on the
    wavefront-per-ray matrix-core kernel (1, 2 or 3 K-steps of per-ray inputs; point counts that
    are not a multiple of the 32-point step; several scenes)."""
    sp = lp_inputs.make_splat_small(kind, channels=channels, res=(12, 10, 11), n_in=n_in, hidden=hidden,
                                    n_freq=n_freq, prior_channels=channels, prior_res=(7, 6, 5), n_rays=203,
                                    samples=41, seed=101 + n_in, n_scenes=2, bias_std=0.1, far=(2.2, 6.0))
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    # the rays run out of the prior's box (far up to 6): the clamped points of a ray share every
    # MLP input and flip together, so the whole-tensor error may use the envelope's full width and a
    # larger share of the small prior-gradient tensor misses the plain tolerance
    print(check_case_splat(lp, oracle, sp, label=f"splat mfma kind={kind} C={channels} n_in={n_in}",
                           width_cap=WIDTH_CAP_SPLAT_BORDER, max_strict_fail=0.06), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("channels", [16, 32])
def test_splatter_mlp_on_matrix_cores_with_contract_coordinates(lp, oracle, kind, channels):
    """The paper's experimental setting uses the Splatter's MLP together with contract coordinates
    (appendix, "Experimental Details"): rays that start inside the unit cube and run far beyond
    it, prior and target contracted alike, matrix-core kernels forward and backward."""
    sp = lp_inputs.make_splat_small(kind, channels=channels, res=(14, 12, 13), n_in=channels, hidden=(64, 64),
                                    n_freq=0, prior_channels=channels, prior_res=(9, 8, 7), n_rays=150, samples=70,
                                    seed=121, n_scenes=2, bias_std=0.1, origin_radius=0.8, near=(0.0, 0.3),
                                    far=(6.0, 30.0))
    sp = dataclasses.replace(sp, contract_a=1.4)
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label=f"splat mfma contract kind={kind} C={channels}",
                           max_strict_fail=0.06), flush=True)


@pytest.mark.parametrize("n_rays,samples", [(1, 1), (5, 33), (3, 32)])
def test_splatter_mlp_on_matrix_cores_degenerate_sizes(lp, oracle, n_rays, samples):
    """Fewer rays than a workgroup has waves, a single point, point counts around the 32-point step."""
    sp = lp_inputs.make_splat_small(TRIPLANE, channels=16, res=(6, 5, 7), n_in=9, hidden=(64, 64), n_freq=0,
                                    prior_channels=16, prior_res=(4, 5, 3), n_rays=n_rays, samples=samples, seed=111,
                                    bias_std=0.1)
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label=f"splat mfma M={n_rays} S={samples}"), flush=True)


def test_splatter_fast_path_query(lp):
    for kw, fast in [(dict(channels=32, n_in=32, hidden=(64, 64), n_freq=0, prior_channels=32), True),
                     (dict(channels=32, n_in=32, hidden=(64, 32), n_freq=0, prior_channels=32), False),
                     (dict(channels=32, n_in=32, hidden=(64,), n_freq=0, prior_channels=16), False),
                     (dict(channels=32, n_in=32, hidden=(64,), n_freq=2, prior_channels=32), True),
                     (dict(channels=32, n_in=34, hidden=(64,), n_freq=2, prior_channels=32), False),
                     (dict(channels=16), True), (dict(channels=6), False)]:
        sp = lp_inputs.make_splat_small(VOXEL, n_rays=5, **kw)
        target, _, splat = lp.splat_to_device(sp)
        assert lp.lp_splat_has_fast_path(target, splat) == fast, kw


def test_splatter_with_the_papers_mlp_size(lp, oracle):
    """32-channel features, prior and target, 3-layer MLP of width 64 (appendix, "Experimental
    Details"): runs on the matrix-core kernels, forward and backward."""
    sp = lp_inputs.make_splat_small(VOXEL, channels=32, res=(9, 8, 10), n_in=32, hidden=(64, 64), n_freq=0,
                                    prior_channels=32, prior_res=(7, 6, 5), n_rays=150, samples=20, seed=99,
                                    bias_std=0.1)
    assert sp.mlp_dims == (67, 64, 64, 32)
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label="splat paper-size MLP"), flush=True)


def test_splatter_generic_kernel_with_a_large_mlp(lp, oracle):
    """An MLP of about the same size that the matrix-core kernels do not cover (hidden widths 64
    and 60): two copies of the parameters no longer fit in LDS, so the generic backward
    accumulates the MLP gradients in its records instead."""
    sp = lp_inputs.make_splat_small(VOXEL, channels=32, res=(9, 8, 10), n_in=32, hidden=(64, 60), n_freq=0,
                                    prior_channels=32, prior_res=(7, 6, 5), n_rays=150, samples=20, seed=99,
                                    bias_std=0.1)
    target, _, splat = lp.splat_to_device(sp)
    assert not lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label="splat large generic MLP"), flush=True)


def test_splat_naive_workload_at_full_size(lp, oracle):
    """The benchmark's naive Splatter workload (160^3 x 32 voxels, 65 536 rays of 160 points),
    whole: every cell of the result, the weight sums and the pixel-feature gradients."""
    sp = lp_inputs.make_splat_inputs("splat_naive")
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label="splat_naive workload"), flush=True)


def test_splat_mlp_workload_at_full_size(lp, oracle):
    """The benchmark's Splatter workload with MLP (160^3 x 32 voxels, prior of the same size, MLP
    67-64-64-32, 16 384 rays of 160 points), whole, in the launch configuration the benchmark
    times: every cell of the result and every gradient against the oracle."""
    sp = lp_inputs.make_splat_inputs("splat_mlp")
    target, _, splat = lp.splat_to_device(sp)
    assert lp.lp_splat_has_fast_path(target, splat)
    print(check_case_splat(lp, oracle, sp, label="splat_mlp workload"), flush=True)


def test_splatter_with_contraction_and_empty_cells(lp, oracle):
    """Contract coordinates; a fine target that most rays never touch (cells with zero weight)."""
    sp = lp_inputs.make_splat_small(VOXEL, channels=4, res=(20, 18, 22), n_in=3, hidden=(8,), n_freq=0,
                                    n_rays=40, samples=30, seed=95, origin_radius=1.5, near=(0.0, 0.3), far=(6.0, 20.0))
    sp = dataclasses.replace(sp, contract_a=1.2)
    w = check_case_splat(lp, oracle, sp, label="splat contract")
    print(w, flush=True)


def test_splatter_errors_and_empty_input(lp):
    import torch
    sp = lp_inputs.make_splat_small(VOXEL, channels=4, n_rays=5)
    target, rays, splat = lp.splat_to_device(sp)
    with pytest.raises(lp.LightplaneError) as e:       # naive Splatter needs n_in == channels
        lp.splat_fwd(lp.target_struct(VOXEL, 1, 3, sp.res), rays, splat)
    assert e.value.status == lp.LP_ERR_INVALID_ARG
    with pytest.raises(lp.LightplaneError) as e:
        lp.splat_fwd(target, rays, dataclasses.replace(splat, n_freq=1))   # encoding without an MLP
    assert e.value.status == lp.LP_ERR_INVALID_ARG
    none = dataclasses.replace(sp, origins=sp.origins[:0], dirs=sp.dirs[:0], near=sp.near[:0], far=sp.far[:0],
                               feats=sp.feats[:0])
    target, rays, splat = lp.splat_to_device(none)
    theta, theta_w = lp.splat_fwd(target, rays, splat)
    torch.cuda.synchronize()
    assert float(theta[0].abs().max()) == 0.0 and float(theta_w[0].abs().max()) == 0.0
