"""GPU parity of the Renderer with the paper's two-MLP, view-dependent decoder against the
CPU oracle, through the C ABI (tolerances as in test_gpu_parity.py)."""
import dataclasses

import numpy as np
import pytest

import lp_inputs
from lp_inputs import HASH, HEXPLANE, TRIPLANE, VOXEL

from parity import check_case_dec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def problem(kind, *, channels, hidden_s, hidden_v, n_freq, n_feat, feat_act=0, seed=0, n_rays=100, samples=40,
            n_scenes=1, bias_std=0.2, **kw):
    inp = lp_inputs.make_small(kind, channels=channels, mlp_dims=(channels, 4), n_rays=n_rays, samples=samples,
                               seed=seed, n_scenes=n_scenes, **kw)
    dec = lp_inputs.make_decoder(channels, hidden_s, hidden_v, n_freq, n_feat, seed + 100, bias_std, feat_act)
    rng = np.random.default_rng(seed + 7)
    return dataclasses.replace(inp, decoder=dec, bg=tuple(rng.random(n_feat).astype(np.float32).tolist()),
                               target=rng.random((n_rays, n_feat), dtype=np.float32))


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("hidden_s,hidden_v,n_freq,n_feat,feat_act", [
    ((7,), (9,), 0, 3, 0),          # equal depth, raw direction
    ((6,), (9, 8), 1, 5, 1),        # shallower opacity MLP (identity carry), identity features
    ((8, 5), (7,), 2, 1, 0),        # shallower feature MLP, one rendered channel
    ((16, 16), (24, 24), 4, 16, 0),  # the limits: four octaves, 16 features
])
def test_decoder_generic(lp, oracle, kind, hidden_s, hidden_v, n_freq, n_feat, feat_act):
    inp = problem(kind, channels=5, hidden_s=hidden_s, hidden_v=hidden_v, n_freq=n_freq, n_feat=n_feat,
                  feat_act=feat_act, seed=71, n_rays=131, samples=37, n_scenes=3, res=(6, 5, 7))
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_GENERIC, label=f"dec kind={kind} {hidden_s}/{hidden_v}"),
          flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("hidden_s,hidden_v,n_freq,samples", [
    ((16,), (16,), 0, 64),           # merged: 32 inputs (16 grid + 3 direction + zeros), width 32, one hidden layer
    ((32, 32), (32, 32), 2, 150),    # width 64, two hidden layers, 15 direction inputs
    ((24,), (40, 40), 1, 37),        # unequal widths, the opacity MLP carried through an identity block
])
def test_decoder_matrix_core(lp, oracle, kind, hidden_s, hidden_v, n_freq, samples):
    """16 grid channels, three sigmoid features: the merged MLP fits the matrix-core kernels."""
    inp = problem(kind, channels=16, hidden_s=hidden_s, hidden_v=hidden_v, n_freq=n_freq, n_feat=3, seed=83,
                  n_rays=203, samples=samples, n_scenes=2, res=(12, 10, 11), grid_std=0.3,
                  aabb_min=(-1.5, -1.5, -1.5), aabb_max=(1.5, 1.5, 1.5))
    grid, _, _, _ = lp.to_device(inp)
    assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    for mode in (lp.LP_MATH_GENERIC, lp.LP_MATH_BF16X3):
        print(mode, check_case_dec(lp, oracle, inp, mode, label=f"dec mfma kind={kind} {hidden_s}/{hidden_v} mode={mode}"),
              flush=True)


@pytest.mark.parametrize("kind,extra", [(HASH, dict(hash_size=4096)), (HEXPLANE, dict(n_time=4, t_range=(-0.5, 1.5)))])
@pytest.mark.parametrize("hidden_s,hidden_v,n_freq,contract,stored", [
    ((16,), (16,), 0, 0.0, None),
    ((32, 32), (32, 32), 2, 1.3, None),      # width 64, two hidden layers, 15 direction inputs, contraction
    ((24,), (40,), 1, 0.0, "bfloat16"),
    ((16, 16), (16, 16), 1, 0.0, None),
])
def test_decoder_matrix_core_on_hash_tables_and_hexplanes(lp, oracle, kind, extra, hidden_s, hidden_v, n_freq, contract, stored):
    """The merged two-MLP decoder (16 channels + direction inputs) over a hash table of a power-of-two
    size and over a HexPlane with a time per ray, on the matrix-core kernels, both arithmetic modes."""
    import torch
    kw = dict(origin_radius=1.5, near=(0.0, 0.3), far=(6.0, 20.0)) if contract else {}
    inp = problem(kind, channels=16, hidden_s=hidden_s, hidden_v=hidden_v, n_freq=n_freq, n_feat=3, seed=89,
                  n_rays=150, samples=70, n_scenes=2, res=(12, 10, 11), grid_std=0.3, **extra, **kw)
    inp = dataclasses.replace(inp, contract_a=contract)
    dtype = None
    if stored:
        dtype = getattr(torch, stored)
        kept = [torch.from_numpy(g).to(dtype) for g in inp.grid]
        inp = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in kept])
    grid, _, _, _ = lp.to_device(inp)
    assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    for mode in (lp.LP_MATH_GENERIC, lp.LP_MATH_BF16X3):
        print(mode, check_case_dec(lp, oracle, inp, mode, label=f"dec mfma kind={kind} {hidden_s}/{hidden_v} mode={mode}",
                                   max_strict_fail=0.05, grid_dtype=dtype), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("hidden_s,hidden_v,n_freq", [((16,), (16,), 0), ((32, 32), (32, 32), 2), ((16, 16), (16, 16), 1),
                                                      ((24,), (40,), 1)])
def test_decoder_matrix_core_with_contract_coordinates(lp, oracle, kind, hidden_s, hidden_v, n_freq):
    """The two-MLP decoder together with contract coordinates: rays that run far beyond the box."""
    inp = problem(kind, channels=16, hidden_s=hidden_s, hidden_v=hidden_v, n_freq=n_freq, n_feat=3, seed=87,
                  n_rays=150, samples=70, n_scenes=2, res=(12, 10, 11), grid_std=0.3, origin_radius=1.5,
                  near=(0.0, 0.3), far=(6.0, 20.0))
    inp = dataclasses.replace(inp, contract_a=1.3)
    grid, _, _, _ = lp.to_device(inp)
    assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"dec mfma contract kind={kind} {hidden_s}/{hidden_v}"),
          flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("channels,n_freq,contract", [(32, 2, 0.0), (16, 1, 0.0), (32, 0, 1.3), (16, 4, 0.0)])
def test_decoder_at_the_papers_size(lp, oracle, kind, channels, n_freq, contract):
    """Two 3-layer MLPs of width 64 (appendix, "Experimental Details") on 16 / 32 grid channels:
    merged they would be 128 wide; they run as two chains on the matrix cores, the backward in
    two passes.  Ragged sample counts, several scenes, once with contract coordinates."""
    kw = dict(origin_radius=1.5, near=(0.0, 0.3), far=(6.0, 20.0)) if contract else {}
    inp = problem(kind, channels=channels, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=n_freq, n_feat=3, seed=89,
                  n_rays=203, samples=75, n_scenes=2, res=(12, 10, 11), grid_std=0.3, bias_std=0.1, **kw)
    if contract:
        inp = dataclasses.replace(inp, contract_a=contract)
    grid, _, _, _ = lp.to_device(inp)
    assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    # 1 320 texels take 15 000 samples: a grid-gradient element here sums dozens of samples of many
    # rays, so one unit whose sign decision differs reaches a larger share of this small tensor
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"dec two chains kind={kind} C={channels}",
                         max_strict_fail=0.05), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
@pytest.mark.parametrize("dtype", ["bfloat16", "float16"])
def test_decoder_on_reduced_precision_grids(lp, oracle, kind, dtype):
    """Grids stored in bf16 / fp16 under the two-MLP decoder: the merged matrix-core kernels (16 grid
    channels + direction inputs) and the two chains at the paper's size, the latter with contract
    coordinates.  The stored values are exactly representable, so the oracle receives them widened."""
    import torch
    tdt = getattr(torch, dtype)
    cases = [dict(channels=16, hidden_s=(32, 32), hidden_v=(32, 32), n_freq=2, contract=0.0),
             dict(channels=32, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=1, contract=1.3)]
    for c in cases:
        kw = dict(origin_radius=1.5, near=(0.0, 0.3), far=(6.0, 20.0)) if c["contract"] else {}
        inp = problem(kind, channels=c["channels"], hidden_s=c["hidden_s"], hidden_v=c["hidden_v"], n_freq=c["n_freq"],
                      n_feat=3, seed=97, n_rays=203, samples=75, n_scenes=2, res=(12, 10, 11), grid_std=0.3,
                      bias_std=0.1, **kw)
        stored = [torch.from_numpy(g).to(tdt) for g in inp.grid]
        inp = dataclasses.replace(inp, grid=[t.to(torch.float32).numpy() for t in stored], contract_a=c["contract"])
        grid, _, _, _ = lp.to_device(inp)
        grid.data = [t.to(tdt) for t in grid.data]
        assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
        print(check_case_dec(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"dec {dtype} kind={kind} C={c['channels']}",
                             max_strict_fail=0.05, grid_dtype=tdt), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_decoder_identity_features_on_the_matrix_cores(lp, oracle, kind):
    """Rendered features without the sigmoid (feat_act = identity), three of them: the merged
    matrix-core kernels and the two chains at the paper's size, the latter with contract coordinates."""
    cases = [dict(channels=16, hidden_s=(32, 32), hidden_v=(32, 32), n_freq=2, contract=0.0),
             dict(channels=16, hidden_s=(24,), hidden_v=(40,), n_freq=1, contract=1.3),
             dict(channels=32, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=1, contract=1.3),
             dict(channels=16, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=2, contract=0.0)]
    for c in cases:
        kw = dict(origin_radius=1.5, near=(0.0, 0.3), far=(6.0, 20.0)) if c["contract"] else {}
        inp = problem(kind, channels=c["channels"], hidden_s=c["hidden_s"], hidden_v=c["hidden_v"], n_freq=c["n_freq"],
                      n_feat=3, feat_act=1, seed=101, n_rays=203, samples=75, n_scenes=2, res=(12, 10, 11), grid_std=0.3,
                      bias_std=0.1, **kw)
        inp = dataclasses.replace(inp, contract_a=c["contract"])
        grid, _, _, _ = lp.to_device(inp)
        assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
        print(check_case_dec(lp, oracle, inp, lp.LP_MATH_BF16X3, label=f"dec identity kind={kind} C={c['channels']} {c['hidden_v']}",
                             max_strict_fail=0.05), flush=True)


@pytest.mark.parametrize("n_rays,samples", [(1, 1), (5, 33), (3, 64), (259, 2)])
def test_decoder_two_chains_degenerate_sizes(lp, oracle, n_rays, samples):
    """Fewer rays than a workgroup has waves, a single sample, sample counts around the 32- and
    64-sample steps."""
    inp = problem(VOXEL, channels=32, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=1, n_feat=3, seed=97,
                  n_rays=n_rays, samples=samples, res=(6, 5, 7), grid_std=0.3, bias_std=0.1)
    grid, _, _, _ = lp.to_device(inp)
    assert lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_DEFAULT, label=f"dec two chains M={n_rays} S={samples}"), flush=True)


@pytest.mark.parametrize("kind", [VOXEL, TRIPLANE])
def test_decoder_at_the_papers_size_on_the_generic_kernels(lp, oracle, kind):
    """The same decoder on the generic kernels: the merged MLP is too large for 64 rays'
    activations beside it in LDS, so they run blocks of fewer rays (partial wavefronts) and
    accumulate the MLP gradients in their records."""
    inp = problem(kind, channels=32, hidden_s=(64, 64), hidden_v=(64, 64), n_freq=2, n_feat=3, seed=89,
                  n_rays=150, samples=24, n_scenes=2, res=(8, 7, 9), grid_std=0.3, bias_std=0.1)
    print(check_case_dec(lp, oracle, inp, lp.LP_MATH_GENERIC, label=f"dec paper size generic kind={kind}"), flush=True)


def test_decoder_fast_path_limits(lp):
    mk = lambda **kw: problem(VOXEL, **{**dict(channels=16, hidden_s=(16,), hidden_v=(16,), n_freq=1, n_feat=3, n_rays=8), **kw})
    def fast(inp):
        grid, _, _, _ = lp.to_device(inp)
        return lp.lp_dec_has_fast_path(grid, lp.decoder_to_device(inp.decoder))
    assert fast(mk())
    assert not fast(mk(n_feat=4))                      # three features only
    assert fast(mk(feat_act=1))                        # sigmoid or identity
    assert not fast(mk(hidden_s=(16,), hidden_v=(20,)))  # merged width must be 32 or 64
    assert not fast(mk(channels=32, hidden_s=(16,), hidden_v=(16,)))
    assert fast(dataclasses.replace(mk(), contract_a=1.0))
    inp = mk(n_feat=4)
    grid, _, rays, bg = lp.to_device(inp)
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_dec_fwd(grid, lp.decoder_to_device(inp.decoder), rays, bg, lp.LP_MATH_BF16X3)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED


def test_decoder_errors(lp):
    import torch
    inp = problem(VOXEL, channels=4, hidden_s=(6,), hidden_v=(6,), n_freq=1, n_feat=3, n_rays=9)
    grid, _, rays, bg = lp.to_device(inp)
    dec = lp.decoder_to_device(inp.decoder)
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_dec_fwd(grid, dataclasses.replace(dec, n_freq=2), rays, bg)     # input width no longer fits
    assert e.value.status == lp.LP_ERR_INVALID_ARG
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_dec_fwd(grid, dataclasses.replace(dec, n_feat=2), rays, bg)
    assert e.value.status == lp.LP_ERR_INVALID_ARG
    lin = lp.Mlp(dec.opacity.weights[:1], dec.opacity.biases[:1])                   # no hidden layer
    with pytest.raises(lp.LightplaneError) as e:
        lp.render_dec_fwd(grid, dataclasses.replace(dec, opacity=lin), rays, bg)
    assert e.value.status == lp.LP_ERR_UNSUPPORTED
    out = torch.empty((9, 3), device="cuda:0")
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(lp.LightplaneError) as e:
        lp.lp_render_dec_fwd(grid, dec, rays, bg, out, None, None, None, tiny)
    assert e.value.status == lp.LP_ERR_WORKSPACE


def test_decoder_workload_on_a_ray_subset(lp, oracle):
    """The `decoder` workload of bench.py (128^3 x 16 voxels, two hidden layers of 32 + 32, two
    octaves of direction encoding), a strided subset of its rays, matrix-core kernels."""
    inp = lp_inputs.make_inputs("decoder")
    sub = inp.subset(lp_inputs.strided_ray_subset(inp.n_rays, 1024, offset=5))
    print(check_case_dec(lp, oracle, sub, lp.LP_MATH_BF16X3, aux_grads=False, label="decoder workload subset",
                         max_strict_fail=0.03), flush=True)
