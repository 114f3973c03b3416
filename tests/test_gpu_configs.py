"""Parity at the full sizes of the workloads the benchmark is quoted on, in the
launch configurations the tuner picks (what bench.py times) and in fixed ones."""
import numpy as np
import pytest
import torch

from oracle import sparse_conv as oc
from workloads import generators as gen
from _util import TOL, coords_dev, make_layer, norm_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import paper_2311_12862_amd as sp
    return sp


def _cfg(sp, **kw):
    c = sp.Config()
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_config2_lidar_100k_fp16_64(sp):
    """~100k-voxel LiDAR-like scan, fp16, 64 -> 64, submanifold: fwd + dgrad + wgrad."""
    c = gen.lidar_scene(2000)
    assert 95_000 <= len(c) <= 105_000
    ref = oc.build_kmap(c, 3, 1)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(km.export_mask().cpu().numpy().view(np.uint32), oc.bitmask(ref.M))
    assert km.n_pairs() == int((ref.M >= 0).sum())
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 2001)
    want_f = oc.forward(x32, w32, ref.M)
    want_d = oc.dgrad(g32, w32, ref.M, ref.n_in)
    want_w = oc.wgrad(x32, g32, ref.M)
    # the configurations bench.py runs: whatever the tuner returns for each op
    for layers in (1, 1000):
        cf, _ = sp.tune(km, 64, 64, torch.float16, sp.OP_FWD, layers)
        cd, _ = sp.tune(km, 64, 64, torch.float16, sp.OP_DGRAD, layers)
        assert norm_err(sp.fwd(x, w, km, cf), want_f) <= TOL["f16"], repr(cf)
        assert norm_err(sp.dgrad(g, w, km, cd), want_d) <= TOL["f16"], repr(cd)
    cw, _ = sp.tune(km, 64, 64, torch.float16, sp.OP_WGRAD, 1)
    assert norm_err(sp.wgrad(x, g, km, cw), want_w) <= 1e-4, repr(cw)
    # and fixed points of the design space, both kernels
    for cfg in (_cfg(sp, n_split=0, kernel=1, tile_n=32), _cfg(sp, n_split=1, kernel=1, tile_n=32),
                _cfg(sp, n_split=2, kernel=1, tile_n=64), _cfg(sp, n_split=0, kernel=2, tile_m=128),
                _cfg(sp, n_split=3, kernel=2, tile_m=64), _cfg(sp, kernel=3)):
        assert norm_err(sp.fwd(x, w, km, cfg), want_f) <= TOL["f16"], repr(cfg)
        assert norm_err(sp.dgrad(g, w, km, cfg), want_d) <= TOL["f16"], repr(cfg)


def test_config3_strided_then_transposed_200k(sp):
    """Two scans (~200k voxels): stride-2 conv 64 -> 128, then the matching transposed conv 128 -> 64."""
    c = gen.lidar_batch(3000, 2)
    assert 190_000 <= len(c) <= 210_000
    down_ref = oc.build_kmap(c, 3, 2)
    up_ref = oc.build_kmap(c, 3, 2, transposed=True)
    dev = coords_dev(c)
    down = sp.build_kmap(dev, 3, 2)
    up = sp.build_kmap(dev, 3, 2, transposed=True)
    np.testing.assert_array_equal(down.export().cpu().numpy(), down_ref.M)
    np.testing.assert_array_equal(down.out_coords().cpu().numpy(), down_ref.out_coords)
    np.testing.assert_array_equal(up.export().cpu().numpy(), up_ref.M)
    np.testing.assert_array_equal(up.in_coords().cpu().numpy(), down_ref.out_coords)
    assert ((up_ref.M >= 0).sum(axis=1) <= 8).all()
    (x32, x), (w32, w), _ = make_layer(down_ref.n_in, down_ref.n_out, 64, 128, 27, "f16", 3001)
    w2_32, w2r = gen.weights(27, 128, 64, "f16", 3002)
    w2 = torch.from_numpy(w2r).cuda()
    want_c = oc.forward(x32, w32, down_ref.M)
    got_c = sp.fwd(x, w, down)
    assert norm_err(got_c, want_c) <= TOL["f16"]
    # the decoder consumes what the encoder produced: feed the GPU's own fp16 output to both sides
    got_c32 = got_c.float().cpu().numpy()
    want_f = oc.forward(got_c32, w2_32, up_ref.M)
    for cfg in (None, _cfg(sp, n_split=2, kernel=2)):
        assert norm_err(sp.fwd(got_c, w2, up, cfg), want_f) <= TOL["f16"]


@pytest.fixture(scope="module")
def room(sp):
    c = gen.room_scene(4000)
    assert 285_000 <= len(c) <= 315_000
    return c, oc.build_kmap(c, 3, 1)


def test_config4_room_300k_kmap(sp, room):
    c, ref = room
    km = sp.build_kmap(coords_dev(c), 3, 1)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    assert km.n_pairs() == int((ref.M >= 0).sum())


@pytest.mark.parametrize("width", [32, 96, 256])
def test_config4_room_300k_bf16(sp, room, width):
    """~300k-voxel indoor cloud, bf16, C -> C for C in 32 / 96 / 256: fwd + dgrad + wgrad."""
    c, ref = room
    km = sp.build_kmap(coords_dev(c), 3, 1)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, width, width, 27, "bf16", 4000 + width)
    assert norm_err(sp.fwd(x, w, km), oc.forward(x32, w32, ref.M)) <= TOL["bf16"]
    assert norm_err(sp.fwd(x, w, km, _cfg(sp, n_split=2)), oc.forward(x32, w32, ref.M)) <= TOL["bf16"]
    assert norm_err(sp.fwd(x, w, km, _cfg(sp, kernel=3)), oc.forward(x32, w32, ref.M)) <= TOL["bf16"]   # fetch-on-demand
    assert norm_err(sp.dgrad(g, w, km), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["bf16"]
    assert norm_err(sp.dgrad(g, w, km, _cfg(sp, kernel=3, tile_m=128)), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["bf16"]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4


def test_detection_style_stack(sp):
    """A second workload shape (anisotropic 0.1 x 0.1 x 0.15 m voxels, a regular stack of
    submanifold and stride-2 convolutions with 16..64 channels, as 3-D detectors use): maps
    bit-exact at every level, every layer of the stack against the oracle under the group tuner."""
    lvl = gen.detection_scene(6000)
    assert 60_000 <= len(lvl) <= 100_000
    widths = (16, 32, 64)
    seed = 6100
    for i, c in enumerate(widths):
        ref = oc.build_kmap(lvl, 3, 1)
        km = sp.build_kmap(coords_dev(lvl), 3, 1)
        np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
        f, _, _, us = sp.tune_group(km, [(c, c), (c, c)], torch.float16)
        (x32, x), (w32, w), _ = make_layer(ref.n_in, ref.n_out, c, c, 27, "f16", seed + 10 * i)
        assert norm_err(sp.fwd(x, w, km, f[0]), oc.forward(x32, w32, ref.M)) <= TOL["f16"], repr(f[0])
        nu = (ref.M >= 0).sum() / ref.n_out
        print(f"level {i}: {ref.n_out} voxels, nu={nu:.1f}, C={c}: group of two layers {us:.0f} us, "
              f"n_split={f[0].n_split}, kernel={f[0].kernel}")
        if i + 1 < len(widths):
            dref = oc.build_kmap(lvl, 3, 2)
            dkm = sp.build_kmap(coords_dev(lvl), 3, 2)
            np.testing.assert_array_equal(dkm.export().cpu().numpy(), dref.M)
            np.testing.assert_array_equal(dkm.out_coords().cpu().numpy(), dref.out_coords)
            co = widths[i + 1]
            (x32, x), (w32, w), _ = make_layer(dref.n_in, dref.n_out, c, co, 27, "f16", seed + 10 * i + 5)
            fd, _, _, _ = sp.tune_group(dkm, [(c, co)], torch.float16)
            assert norm_err(sp.fwd(x, w, dkm, fd[0]), oc.forward(x32, w32, dref.M)) <= TOL["f16"], repr(fd[0])
            lvl = dref.out_coords


def test_pair_lists_of_a_1_35m_voxel_cloud(sp):
    """Beyond ~1.3M rows the per-chunk pair counts are scanned by launches of their own instead of
    by the fill kernel (below, every fill workgroup adds them up itself): the weight gradient over
    those pair lists against the plain definition, with the map bit-exact on the way."""
    c = gen.uniform_cloud(1_350_000, 256, seed=77)
    ref = oc.build_kmap(c, 3, 1)
    (x32, x), _, (g32, g) = make_layer(ref.n_in, ref.n_out, 8, 8, 27, "f16", 9100)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    assert km.n_pairs() == int((ref.M >= 0).sum())
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
