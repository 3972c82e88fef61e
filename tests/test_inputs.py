"""The seeded input generators: deterministic, shaped as the configurations say, rays as the
library requires them (unit directions, every sample inside the grid box).  CPU only."""
import numpy as np
import pytest

import lp_inputs


def test_workload_table_matches_the_configurations():
    w = lp_inputs.WORKLOADS
    assert [w[k].cfg_id for k in lp_inputs.WORKLOAD_ORDER] == [1, 2, 3, 4, 5]
    assert (w["tiny"].rays, w["tiny"].samples, w["tiny"].mlp_dims) == (1024, 64, (16, 32, 4))
    assert (w["single_scene"].rays, w["single_scene"].ray_samples) == (16384, 2097152)
    assert (w["voxel"].rays, w["voxel"].ray_samples, w["voxel"].gather_bytes_per_sample) == (262144, 67108864, 1024)
    assert (w["batched"].rays, w["batched"].ray_samples, w["batched"].gather_bytes_per_sample) == (2097152, 402653184, 1536)
    assert (w["large"].rays, w["large"].ray_samples, w["large"].gather_bytes_per_sample) == (640000, 327680000, 512)
    assert w["large"].mlp_flop_per_sample == 10752 and w["single_scene"].mlp_flop_per_sample == 12800


@pytest.mark.parametrize("name", ["tiny", "single_scene"])
def test_inputs_are_deterministic_and_well_formed(name):
    a = lp_inputs.make_inputs(name)
    b = lp_inputs.make_inputs(name)
    for x, y in zip(a.grid + a.weights + a.biases + [a.origins, a.dirs, a.near, a.far, a.target],
                    b.grid + b.weights + b.biases + [b.origins, b.dirs, b.near, b.far, b.target]):
        assert x.dtype == np.float32 and x.flags["C_CONTIGUOUS"] and np.array_equal(x, y)
    w = lp_inputs.WORKLOADS[name]
    assert [g.shape for g in a.grid] == lp_inputs.grid_shapes(w.kind, w.n_scenes, w.res, w.channels)
    assert abs(float(np.std(a.grid[0])) - w.grid_std) < 0.02 * w.grid_std
    # unit directions to float32 rounding
    n = np.linalg.norm(a.dirs.astype(np.float64), axis=1)
    assert np.abs(n - 1.0).max() < 2e-7
    # every sample of every ray lies inside the grid box, so no sample is clamped
    t = np.array([w.near, w.far])
    pts = a.origins[:, None, :].astype(np.float64) + t[None, :, None] * a.dirs[:, None, :].astype(np.float64)
    assert np.abs(pts).max() < w.aabb


def test_four_camera_rays_and_scene_indices():
    w = lp_inputs.WORKLOADS["batched"]
    o, d, near, far, scene = lp_inputs.make_rays(w)
    assert o.shape == (w.rays, 3) and scene.dtype == np.int32
    assert np.array_equal(np.bincount(scene), np.full(8, 4 * 256 * 256))
    cams = lp_inputs.cameras_for(w)
    assert len(cams) == 4
    for rot, pos in cams:
        assert abs(np.linalg.norm(pos) - 2.5) < 1e-12
        assert np.allclose(rot.T @ rot, np.eye(3), atol=1e-12)
        assert np.allclose(rot[:, 2], pos / 2.5)          # the camera looks at the origin


def test_strided_subset_is_a_deterministic_set_of_distinct_rays():
    idx = lp_inputs.strided_ray_subset(640000, 768, offset=3)
    assert len(idx) == 768 and len(set(idx.tolist())) == 768 and idx.max() < 640000
    assert np.array_equal(idx, lp_inputs.strided_ray_subset(640000, 768, offset=3))


def test_contract_workload_has_the_papers_experimental_shape():
    """Appendix, "Experimental Details": 160^3 voxels x 32 features, 3-layer width-64 MLP,
    256 x 256 image, 384 points per ray, contract coordinates over the [-1, 1] cube."""
    w = lp_inputs.WORKLOADS["contract"]
    assert (w.res, w.channels, w.mlp_dims, w.image, w.samples) == ((160, 160, 160), 32, (32, 64, 64, 4), 256, 384)
    inp = lp_inputs.make_inputs("contract", with_grid=False)
    assert inp.contract_a == 1.0 and inp.aabb_min == (-1.0, -1.0, -1.0) and inp.aabb_max == (1.0, 1.0, 1.0)
    assert inp.n_rays == 256 * 256 and float(inp.far.max()) > 10.0


def test_splat_workloads():
    """Appendix, "Experimental Details": 160^3 voxel grid, 160 points per ray; the naive workload
    carries the 32-dimensional features of the paper."""
    w = lp_inputs.SPLAT_WORKLOADS["splat_naive"]
    assert (w.res, w.channels, w.n_in, w.samples) == ((160, 160, 160), 32, 32, 160)
    sp = lp_inputs.make_splat_inputs("splat_mlp")
    assert sp.mlp_dims == (32 + 32 + 3, 64, 64, 32) and sp.prior[0].shape == (1, 160, 160, 160, 32)
    assert sp.n_rays == 4 * 64 * 64 and sp.feats.shape == (sp.n_rays, 32)
    a = lp_inputs.make_splat_inputs("splat_mlp")
    assert np.array_equal(a.feats, sp.feats) and np.array_equal(a.weights[1], sp.weights[1])
