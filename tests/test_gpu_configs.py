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
                _cfg(sp, n_split=3, kernel=2, tile_m=64)):
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
    assert norm_err(sp.dgrad(g, w, km), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["bf16"]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
