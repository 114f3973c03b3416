"""Feature kernels (fwd, dgrad, wgrad) of the HIP library against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import sparse_conv as oc
from workloads import generators as gen
from _util import TOL, coords_dev, make_layer, norm_err, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import paper_2311_12862_amd as sp
    return sp


@pytest.fixture(scope="module")
def cloud():
    """A cloud that spans several 256-row tiles with a ragged tail and mixed neighbour counts."""
    c = gen.lidar_scene(77, target_n=2900)
    return c, oc.build_kmap(c, 3, 1)


def _cfg(sp, n_split=0, tile_m=0, tile_n=0, wgrad_pairs=0, kernel=0):
    c = sp.Config()
    c.n_split, c.tile_m, c.tile_n, c.wgrad_pairs, c.kernel = n_split, tile_m, tile_n, wgrad_pairs, kernel
    return c


def test_config1_tiny_fp32_forward(sp):
    """2,000 voxels in 64^3, fp32, 16 -> 16, forward only."""
    c = gen.uniform_cloud(2000, 64, seed=1000)
    ref = oc.build_kmap(c, 3, 1)
    (x32, x), (w32, w), _ = make_layer(2000, 2000, 16, 16, 27, "f32", 1001)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    want = oc.forward(x32, w32, ref.M)
    for n_split in range(5):
        got = sp.fwd(x, w, km, _cfg(sp, n_split))
        assert norm_err(got, want) <= TOL["f32"], n_split


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("kernel", [1, 2])
@pytest.mark.parametrize("c_in,c_out", [(64, 64), (32, 96), (96, 32), (8, 16), (128, 256), (256, 128), (24, 40)])
def test_forward_and_dgrad_channels(sp, cloud, dtype, kernel, c_in, c_out):
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, c_in, c_out, 27, dtype, 5)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    for n_split in (0, 3):
        cfg = _cfg(sp, n_split, kernel=kernel)
        if kernel == 1 and c_in > 128:     # the LDS-resident kernel reduces over at most 128 channels
            with pytest.raises(sp.SpconvError) as e:
                sp.fwd(x, w, km, cfg)
            assert e.value.status == -1
        else:
            assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL[dtype]
        if kernel == 1 and c_out > 128:
            with pytest.raises(sp.SpconvError):
                sp.dgrad(g, w, km, cfg)
        else:
            assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL[dtype]


@pytest.mark.parametrize("n_split", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("kernel,tile_m,tile_n", [(2, 64, 0), (2, 128, 0), (2, 256, 0), (1, 0, 16), (1, 0, 32), (1, 0, 64)])
def test_forward_design_space(sp, cloud, n_split, kernel, tile_m, tile_n):
    """Sorting and splitting change the work, never the result (Sections 2.2.3, 4.1)."""
    c, ref = cloud
    (x32, x), (w32, w), _ = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 6)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    want = oc.forward(x32, w32, ref.M)
    cfg = _cfg(sp, n_split, tile_m, tile_n, kernel=kernel)
    if kernel == 1 and tile_n == 64 and n_split < 2:
        # 27 offsets x 64 x 64 fp16 weights do not fit in LDS: the call must refuse, not fall back
        with pytest.raises(sp.SpconvError) as e:
            sp.fwd(x, w, km, cfg)
        assert e.value.status == -1
        return
    got = sp.fwd(x, w, km, cfg)
    assert norm_err(got, want) <= TOL["f16"]
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("c_in,c_out", [(128, 128), (64, 192), (256, 64), (128, 72)])
def test_tiles_of_256_rows_by_128_columns(sp, cloud, dtype, c_in, c_out):
    """The largest tile of the tiled kernel with 64-channel reduction chunks: all split counts (sorted
    and unsorted maps), a column tile that is partly or wholly past the last channel, forward and
    input gradient (whose reduction then runs over c_out)."""
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, c_in, c_out, 27, dtype, 21)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    want_f, want_d = oc.forward(x32, w32, ref.M), oc.dgrad(g32, w32, ref.M, ref.n_in)
    for n_split in range(5):
        cfg = _cfg(sp, n_split, 256, 128, kernel=2)
        assert norm_err(sp.fwd(x, w, km, cfg), want_f) <= TOL[dtype], n_split
        assert norm_err(sp.dgrad(g, w, km, cfg), want_d) <= TOL[dtype], n_split


@pytest.mark.parametrize("stride,transposed", [(2, False), (2, True)])
def test_tiles_of_256_rows_on_strided_and_transposed_maps(sp, stride, transposed):
    """The same tile on maps whose two sides differ: the strided map and its transpose, which reads
    the weights mirrored."""
    c = gen.lidar_scene(79, target_n=2600)
    ref = oc.build_kmap(c, 3, stride, transposed)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 128, 27, "f16", 22)
    km = sp.build_kmap(coords_dev(c), 3, stride, transposed)
    for n_split in (0, 1, 3):
        cfg = _cfg(sp, n_split, 256, 128, kernel=2)
        assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL["f16"], n_split
        assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"], n_split


@pytest.mark.parametrize("tile_n", [32, 64, 128])
def test_forward_tile_n(sp, cloud, tile_n):
    c, ref = cloud
    (x32, x), (w32, w), _ = make_layer(ref.n_in, ref.n_out, 64, 96, 27, "bf16", 7)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    got = sp.fwd(x, w, km, _cfg(sp, 1, 128, tile_n, kernel=2))
    assert norm_err(got, oc.forward(x32, w32, ref.M)) <= TOL["bf16"]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("stride,transposed", [(1, False), (2, False), (2, True), (1, True)])
def test_fwd_dgrad_wgrad_all_map_kinds(sp, dtype, stride, transposed):
    c = gen.lidar_scene(78, target_n=2500)
    ref = oc.build_kmap(c, 3, stride, transposed)
    c_in, c_out = (16, 24) if dtype == "f32" else (32, 64)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, c_in, c_out, 27, dtype, 11)
    km = sp.build_kmap(coords_dev(c), 3, stride, transposed)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    for n_split in (0, 1, 3):
        for kernel in ((2,) if dtype == "f32" else (1, 2)):
            cfg = _cfg(sp, n_split, kernel=kernel)
            assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL[dtype]
            assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL[dtype]
    dw = sp.wgrad(x, g, km)
    assert dw.dtype == torch.float32
    # dW is produced in fp32 from exactly representable inputs: only the summation order differs
    assert norm_err(dw, oc.wgrad(x32, g32, ref.M)) <= 1e-4
    dw2 = sp.wgrad(x, g, km, _cfg(sp, wgrad_pairs=1500))
    assert norm_err(dw2, oc.wgrad(x32, g32, ref.M)) <= 1e-4


def test_k1_is_linear_layer(sp):
    c = gen.uniform_cloud(1500, 16, seed=3)
    (x32, x), (w32, w), (g32, g) = make_layer(1500, 1500, 64, 32, 1, "f16", 21)
    km = sp.build_kmap(coords_dev(c), 1, 1)
    assert norm_err(sp.fwd(x, w, km), x32.astype(np.float64) @ w32[0].astype(np.float64)) <= TOL["f16"]
    assert norm_err(sp.dgrad(g, w, km), g32.astype(np.float64) @ w32[0].astype(np.float64).T) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, km), (x32.astype(np.float64).T @ g32.astype(np.float64))[None]) <= 1e-4


def test_isolated_points_and_dense_cube(sp):
    # every point isolated: only the centre offset is present
    iso = gen.uniform_cloud(300, 10, seed=2) * np.array([1, 3, 3, 3], dtype=np.int32)
    ref = oc.build_kmap(iso, 3, 1)
    assert (ref.M >= 0).sum() == 300
    (x32, x), (w32, w), (g32, g) = make_layer(300, 300, 32, 32, 27, "f16", 31)
    km = sp.build_kmap(coords_dev(iso), 3, 1)
    assert norm_err(sp.fwd(x, w, km), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
    # fully occupied cube: all 27 offsets present in the interior
    cube = gen.full_grid(9, 2, seed=4)
    ref = oc.build_kmap(cube, 3, 1)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 32, 32, 27, "f16", 32)
    km = sp.build_kmap(coords_dev(cube), 3, 1)
    for n_split in (0, 2):
        assert norm_err(sp.fwd(x, w, km, _cfg(sp, n_split)), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
        assert norm_err(sp.dgrad(g, w, km, _cfg(sp, n_split)), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4


def test_single_point_and_empty(sp):
    one = np.array([[0, 1, 2, 3]], dtype=np.int32)
    (x32, x), (w32, w), (g32, g) = make_layer(1, 1, 16, 16, 27, "f16", 41)
    km = sp.build_kmap(coords_dev(one), 3, 1)
    assert norm_err(sp.fwd(x, w, km), x32.astype(np.float64) @ w32[13].astype(np.float64)) <= TOL["f16"]
    assert norm_err(sp.dgrad(g, w, km), g32.astype(np.float64) @ w32[13].astype(np.float64).T) <= TOL["f16"]
    dw = sp.wgrad(x, g, km).cpu().numpy()
    assert np.abs(dw[np.arange(27) != 13]).max() == 0
    empty = sp.build_kmap(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 3, 1)
    e = torch.empty((0, 16), dtype=torch.float16, device="cuda")
    assert sp.fwd(e, w, empty).shape == (0, 16)
    assert sp.wgrad(e, e, empty).abs().max().item() == 0


def test_shape_and_config_errors(sp, cloud):
    c, ref = cloud
    (x32, x), (w32, w), _ = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 51)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    with pytest.raises(sp.SpconvError) as e:
        sp.fwd(x[:-1].contiguous(), w, km)
    assert e.value.status == -5
    with pytest.raises(sp.SpconvError) as e:
        sp.fwd(x, w, km, _cfg(sp, 9))
    assert e.value.status == -1
    with pytest.raises(sp.SpconvError) as e:
        sp.fwd(x, w, km, _cfg(sp, 1, 100))
    assert e.value.status == -1
    x12 = torch.zeros((ref.n_in, 12), dtype=torch.float16, device="cuda")
    w12 = torch.zeros((27, 12, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(sp.SpconvError) as e:
        sp.fwd(x12, w12, km)
    assert e.value.status == -1        # channel counts that are not a multiple of 8
    # a caller-supplied output of the wrong shape, type or layout never reaches the library
    for bad in (torch.empty((ref.n_out, 32), dtype=torch.float16, device="cuda"),
                torch.empty((ref.n_out - 1, 64), dtype=torch.float16, device="cuda"),
                torch.empty((ref.n_out, 64), dtype=torch.bfloat16, device="cuda"),
                torch.empty((ref.n_out, 128), dtype=torch.float16, device="cuda")[:, ::2],
                torch.empty((ref.n_out, 64), dtype=torch.float16)):
        for call in (lambda o: sp.fwd(x, w, km, out=o), lambda o: sp.dgrad(x, w, km, out=o)):
            with pytest.raises((sp.SpconvError, ValueError)):
                call(bad)
    with pytest.raises((sp.SpconvError, ValueError)):
        sp.wgrad(x, x, km, out=torch.empty((27, 64, 32), dtype=torch.float32, device="cuda"))


@pytest.mark.parametrize("n_split", [1, 2, 4])
def test_sort_invariants(sp, cloud, n_split):
    """Any order of equal keys is valid; what is unique is checked: each perm is a
    bijection, its keys ascend, and (this library sorts stably) ties keep row order."""
    c, ref = cloud
    km = sp.build_kmap(coords_dev(c), 3, 1)
    mask = oc.bitmask(ref.M).astype(np.uint64)
    cfg = _cfg(sp, n_split)
    for i, (lo, hi) in enumerate(oc.split_ranges(27, n_split)):
        perm = km.export_perm(sp.OP_FWD, cfg, i).cpu().numpy()
        assert sorted(perm.tolist()) == list(range(ref.n_out))
        key = (mask[perm] >> np.uint64(lo)) & np.uint64((1 << (hi - lo)) - 1)
        assert (np.diff(key.astype(np.int64)) >= 0).all()
        same = np.diff(key.astype(np.int64)) == 0
        assert (np.diff(perm)[same] > 0).all()


def _check_order(perm, key, rows):
    assert sorted(perm.tolist()) == list(range(rows))
    k = key[perm].astype(np.int64)
    assert (np.diff(k) >= 0).all()
    assert (np.diff(perm)[np.diff(k) == 0] > 0).all()


@pytest.mark.parametrize("n_split", [1, 2, 3])
def test_sort_invariants_on_the_input_side_of_a_strided_map(sp, n_split):
    """dgrad of a strided map walks the input-side map T[j][k] = n  <=>  M[n][k] = j; its rows are
    sorted by their own bitmasks (which offsets reach input j), part by part."""
    c = gen.lidar_scene(78, target_n=2900)
    ref = oc.build_kmap(c, 3, 2)
    km = sp.build_kmap(coords_dev(c), 3, 2)
    T = np.full((ref.n_in, 27), -1, np.int64)
    n, k = np.nonzero(ref.M >= 0)
    T[ref.M[n, k], k] = n
    mask = oc.bitmask(T).astype(np.uint64)
    cfg = _cfg(sp, n_split)
    for i, (lo, hi) in enumerate(oc.split_ranges(27, n_split)):
        perm = km.export_perm(sp.OP_DGRAD, cfg, i).cpu().numpy()
        _check_order(perm, (mask >> np.uint64(lo)) & np.uint64((1 << (hi - lo)) - 1), ref.n_in)


@pytest.mark.parametrize("target_n", [2048, 2049, 131072, 140000])
def test_sort_invariants_across_the_sizes_that_change_the_sort(sp, target_n):
    """One workgroup of the few-launch sort, one row more, its largest map (64 workgroups), and a
    map beyond it (the general radix sort).  The masks come from the library's own map, which
    test_gpu_kmap holds against the oracle bit by bit; here only the order is at stake."""
    c = gen.lidar_scene(79, target_n=target_n + 200)[:target_n]
    km = sp.build_kmap(coords_dev(c), 3, 1)
    M = km.export().cpu().numpy()
    mask = oc.bitmask(M).astype(np.uint64)
    for n_split in (1, 2):
        cfg = _cfg(sp, n_split)
        for i, (lo, hi) in enumerate(oc.split_ranges(27, n_split)):
            perm = km.export_perm(sp.OP_FWD, cfg, i).cpu().numpy()
            _check_order(perm, (mask >> np.uint64(lo)) & np.uint64((1 << (hi - lo)) - 1), len(c))


@pytest.mark.parametrize("kernel", [1, 2])
@pytest.mark.parametrize("n_split", [1, 2, 3])
def test_spatial_slabs_in_front_of_the_sort_keys(sp, cloud, kernel, n_split):
    """SPCONV_FLAG_SLABS: rows are visited slab by slab (eight equal slabs along the longest axis)
    and in stable bitmask order inside a slab.  Any order is valid, so the results are checked
    against the oracle as always, and the order against the rule the header states."""
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 32, 27, "f16", 91)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    cfg = _cfg(sp, n_split, kernel=kernel)
    cfg.flags = sp.FLAG_SLABS
    assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
    assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
    ext = c[:, 1:].max(0).astype(np.int64) - c[:, 1:].min(0) + 1
    axis = int(np.argmax(ext))                  # first of the longest axes
    slab = (c[:, 1 + axis].astype(np.int64) - c[:, 1 + axis].min()) * 8 // ext[axis]
    mask = oc.bitmask(ref.M).astype(np.uint64)
    for i, (lo, hi) in enumerate(oc.split_ranges(27, n_split)):
        perm = km.export_perm(sp.OP_FWD, cfg, i).cpu().numpy()
        assert sorted(perm.tolist()) == list(range(ref.n_out))
        key = (slab[perm] << 27) | ((mask[perm] >> np.uint64(lo)) & np.uint64((1 << (hi - lo)) - 1)).astype(np.int64)
        assert (np.diff(key) >= 0).all()
        assert (np.diff(perm)[np.diff(key) == 0] > 0).all()
    plain = _cfg(sp, n_split, kernel=kernel)    # the plan without slabs is a different plan
    assert not np.array_equal(km.export_perm(sp.OP_FWD, plain, 0).cpu().numpy(),
                              km.export_perm(sp.OP_FWD, cfg, 0).cpu().numpy())


@pytest.mark.parametrize("n_split", [0, 1, 2, 3])
def test_mac_units_match_oracle_model(sp, cloud, n_split):
    c, ref = cloud
    km = sp.build_kmap(coords_dev(c), 3, 1)
    ex, eff = km.mac_units(sp.OP_FWD, _cfg(sp, n_split))
    assert (ex, eff) == oc.redundancy(ref.M, 16, n_split)


def test_results_are_reproducible(sp, cloud):
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 61)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    for cfg in (_cfg(sp, 0), _cfg(sp, 2)):
        assert torch.equal(sp.fwd(x, w, km, cfg), sp.fwd(x, w, km, cfg))
    assert torch.equal(sp.wgrad(x, g, km), sp.wgrad(x, g, km))


def test_tune_returns_a_valid_config(sp, cloud):
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 71)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    for op in (sp.OP_FWD, sp.OP_DGRAD, sp.OP_WGRAD):
        best, us = sp.tune(km, 64, 64, torch.float16, op, 4)
        assert us > 0
        assert 0 <= best.n_split <= 4
    best, _ = sp.tune(km, 64, 64, torch.float16, sp.OP_FWD, 1)
    assert norm_err(sp.fwd(x, w, km, best), oc.forward(x32, w32, ref.M)) <= TOL["f16"]


def test_layer_on_a_pending_asynchronous_kmap(sp, cloud):
    """fwd / dgrad / wgrad may run before the build's status has been read (wgrad then sizes its
    work list from the bound n_out * 27)."""
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 81)
    km = sp.build_kmap(coords_dev(c), 3, 1, asynchronous=True)
    y, dx, dw = sp.fwd(x, w, km), sp.dgrad(g, w, km), sp.wgrad(x, g, km)
    km.status()
    assert norm_err(y, oc.forward(x32, w32, ref.M)) <= TOL["f16"]
    assert norm_err(dx, oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
    assert norm_err(dw, oc.wgrad(x32, g32, ref.M)) <= 1e-4
    assert torch.equal(dw, sp.wgrad(x, g, km))


def test_kernel_size_one_maps_tune_and_reject_empty_splits(sp):
    """A K = 1 map has one offset: it cannot be split, and the tuner must not try."""
    c = gen.uniform_cloud(3000, 20, seed=41)
    km = sp.build_kmap(coords_dev(c), 1, 1)
    ref = oc.build_kmap(c, 1, 1)
    x32, xr = gen.features(len(c), 64, "f16", 42)
    w32, wr = gen.weights(1, 64, 32, "f16", 43)
    x, w = to_dev(xr, "f16"), to_dev(wr, "f16")
    want = oc.forward(x32, w32, ref.M)
    for op in (sp.OP_FWD, sp.OP_DGRAD, sp.OP_WGRAD):
        best, us = sp.tune(km, 64, 32, torch.float16, op, 2)
        assert best.n_split <= 1 and us > 0
    cfg = sp.tune(km, 64, 32, torch.float16, sp.OP_FWD, 2)[0]
    assert norm_err(sp.fwd(x, w, km, cfg), want) <= TOL["f16"]
    bad = sp.Config()
    bad.n_split = 2
    with pytest.raises(sp.SpconvError) as e:
        sp.fwd(x, w, km, bad)
    assert e.value.status == -1


@pytest.mark.parametrize("stride,bind", [(1, True), (2, False)])
def test_group_tuner(sp, stride, bind):
    """spconv_tune_group: one split count per group (fwd and dgrad bound or not), a configuration per
    layer, one wgrad item size for the group; every returned configuration computes the layer."""
    c = gen.lidar_scene(77, target_n=6000)
    km = sp.build_kmap(coords_dev(c), 3, stride)
    ref = oc.build_kmap(c, 3, stride)
    layers = [(16, 16), (16, 32), (16, 16), (32, 16)]
    f, d, w, us = sp.tune_group(km, layers, torch.float16, training=True, bind_fwd_dgrad=bind)
    assert len(f) == len(d) == len(w) == 4 and us > 0
    assert len({x.n_split for x in f}) == 1 and len({x.n_split for x in d}) == 1
    assert len({x.wgrad_pairs for x in w}) == 1 and w[0].wgrad_pairs > 0
    if bind:
        assert f[0].n_split == d[0].n_split
    assert f[0].n_split == f[2].n_split and repr(f[0]) == repr(f[2])      # equal shapes, equal choice
    fi, _, _, us_inf = sp.tune_group(km, layers, torch.float16)
    assert len(fi) == 4 and 0 < us_inf
    for i, (ci, co) in enumerate(layers):
        (x32, x), (w32, wt), (g32, g) = make_layer(ref.n_in, ref.n_out, ci, co, 27, "f16", 900 + i)
        assert norm_err(sp.fwd(x, wt, km, f[i]), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
        assert norm_err(sp.dgrad(g, wt, km, d[i]), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
        assert norm_err(sp.wgrad(x, g, km, w[i]), oc.wgrad(x32, g32, ref.M)) <= 1e-4
    with pytest.raises(sp.SpconvError):
        sp.tune_group(km, [(16, 12)], torch.float16)   # channel counts must be multiples of 8


def test_group_tuner_fp32(sp):
    """fp32 layers have one implicit-GEMM kernel and one fetch-on-demand kernel: the group tuner varies the splits
    and the dataflow; whatever it picks is correct."""
    c = gen.lidar_scene(78, target_n=3000)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    ref = oc.build_kmap(c, 3, 1)
    f, d, w, us = sp.tune_group(km, [(16, 24), (24, 16)], torch.float32, training=True)
    assert us > 0
    (x32, x), (w32, wt), (g32, g) = make_layer(ref.n_in, ref.n_out, 16, 24, 27, "f32", 950)
    assert norm_err(sp.fwd(x, wt, km, f[0]), oc.forward(x32, w32, ref.M)) <= TOL["f32"]
    assert norm_err(sp.dgrad(g, wt, km, d[0]), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f32"]
    assert norm_err(sp.wgrad(x, g, km, w[0]), oc.wgrad(x32, g32, ref.M)) <= 1e-4


@pytest.mark.parametrize("transposed", [False, True])
def test_even_kernel_layers(sp, transposed):
    """fwd / dgrad / wgrad on K = s = 2 maps (8 offsets), automatic and explicit configurations."""
    c = gen.lidar_scene(91, target_n=9000)
    km = sp.build_kmap(coords_dev(c), 2, 2, transposed)
    ref = oc.build_kmap(c, 2, 2, transposed)
    ci, co = (32, 64) if not transposed else (64, 32)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, ci, co, 8, "f16", 92)
    want_f, want_d = oc.forward(x32, w32, ref.M), oc.dgrad(g32, w32, ref.M, ref.n_in)
    cfgs = [None]
    for kw in (dict(kernel=1, tile_n=32), dict(kernel=1, n_split=2, tile_n=32), dict(kernel=2, tile_m=64),
               dict(kernel=2, n_split=4, tile_m=128)):
        cfg = sp.Config()
        for k, v in kw.items():
            setattr(cfg, k, v)
        cfgs.append(cfg)
    for cfg in cfgs:
        assert norm_err(sp.fwd(x, w, km, cfg), want_f) <= TOL["f16"], repr(cfg)
        assert norm_err(sp.dgrad(g, w, km, cfg), want_d) <= TOL["f16"], repr(cfg)
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
    f, d, wg, us = sp.tune_group(km, [(ci, co)], torch.float16, training=True)
    assert norm_err(sp.fwd(x, w, km, f[0]), want_f) <= TOL["f16"]
    assert norm_err(sp.dgrad(g, w, km, d[0]), want_d) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, km, wg[0]), oc.wgrad(x32, g32, ref.M)) <= 1e-4


def test_layer_replays_in_a_hip_graph(sp, cloud):
    """Once plans and scratch exist, fwd / dgrad / wgrad only launch kernels (buffers are cleared by
    fill kernels, never by memset nodes), so a layer can be captured and replayed; every replay,
    with eager work in between, must equal the eager result on the inputs of that moment."""
    c, ref = cloud
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 91)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    fod = _cfg(sp, kernel=3)
    cfgs = [_cfg(sp, 0), _cfg(sp, 2, 64, kernel=2), fod]
    outs = [sp.fwd(x, w, km, cf) for cf in cfgs]          # warm-up: plans, scratch, kernel attributes
    dx, dw = sp.dgrad(g, w, km), sp.wgrad(x, g, km)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for cf, o in zip(cfgs, outs):
            sp.fwd(x, w, km, cf, out=o)
        sp.dgrad(g, w, km, out=dx)
        sp.wgrad(x, g, km, out=dw)
    for rep in range(3):
        x.copy_((torch.randn_like(x, dtype=torch.float32) * 0.5).half())      # eager work between replays
        g.copy_((torch.randn_like(g, dtype=torch.float32) * 0.5).half())
        for o in outs + [dx, dw]:
            o.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        want = sp.fwd(x, w, km, cfgs[0])
        assert torch.equal(outs[0], want), rep
        assert torch.equal(outs[1], sp.fwd(x, w, km, cfgs[1])), rep
        assert norm_err(outs[2], want.double().cpu().numpy()) <= TOL["f16"], rep   # atomics: order varies
        assert torch.equal(dx, sp.dgrad(g, w, km)), rep
        assert torch.equal(dw, sp.wgrad(x, g, km)), rep


def test_two_kmaps_on_two_streams(sp):
    """Different kmaps may be driven from different streams at the same time (each kmap keeps to
    one stream); the library's block pool hands a freed block only to the stream that used it."""
    clouds = [gen.lidar_scene(101 + i, target_n=2500 + 300 * i) for i in range(2)]
    refs = [oc.build_kmap(c, 3, 1) for c in clouds]
    layers = [make_layer(r.n_in, r.n_out, 32, 64, 27, "f16", 120 + i) for i, r in enumerate(refs)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    cfg = _cfg(sp, 2, 64, kernel=2)                     # sorted plan, split partial sums: allocations inside
    torch.cuda.synchronize()
    outs = [None, None]
    for rep in range(3):                                # interleave the two streams' calls
        kms = []
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                kms.append(sp.build_kmap(coords_dev(clouds[i]), 3, 1, asynchronous=True))
        for i, st in enumerate(streams):
            (x32, x), (w32, w), (g32, g) = layers[i]
            with torch.cuda.stream(st):
                y = sp.fwd(x, w, kms[i], cfg)
                dx = sp.dgrad(g, w, kms[i])
                dw = sp.wgrad(x, g, kms[i])
                outs[i] = (y, dx, dw)
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                kms[i].status()
                kms[i].destroy()
    torch.cuda.synchronize()
    for i, r in enumerate(refs):
        (x32, x), (w32, w), (g32, g) = layers[i]
        y, dx, dw = outs[i]
        assert norm_err(y, oc.forward(x32, w32, r.M)) <= TOL["f16"]
        assert norm_err(dx, oc.dgrad(g32, w32, r.M, r.n_in)) <= TOL["f16"]
        assert norm_err(dw, oc.wgrad(x32, g32, r.M)) <= 1e-4


@pytest.fixture(scope="module")
def cloud5():
    """A cloud for the 5 x 5 x 5 neighbourhood: several 256-row tiles, a ragged tail, two batches."""
    c = gen.uniform_cloud(2500, 18, seed=555)
    c[:900, 0] = 1
    return c, oc.build_kmap(c, 5, 1)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("n_split,kernel", [(0, 0), (1, 1), (2, 2), (3, 0)])
def test_k5_forward_dgrad_wgrad(sp, cloud5, dtype, n_split, kernel):
    """K = 5 submanifold layer (Equation 1 over the 125 offsets of Section 2.1): the sum over five
    25-offset planes, each run like a map of its own, against the oracle on the whole map."""
    if dtype == "f32" and kernel == 1:
        pytest.skip("kernel 1 is a 16-bit kernel")
    c, ref = cloud5
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 32, 64, 125, dtype, 123)
    km = sp.build_kmap(coords_dev(c), 5, 1)
    cfg = _cfg(sp, n_split, kernel=kernel)
    assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL[dtype]
    assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL[dtype]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
    ex, eff = km.mac_units(sp.OP_FWD, cfg)
    assert eff == int((ref.M >= 0).sum()) and ex >= eff
    km.destroy()


def test_k5_sort_order_per_plane(sp, cloud5):
    """Sorted K = 5 plans: every plane's rows in stable ascending order of that plane's 25-bit mask."""
    c, ref = cloud5
    km = sp.build_kmap(coords_dev(c), 5, 1)
    cfg = _cfg(sp, 1)
    big = oc.bitmask(ref.M)
    for g in range(5):
        key = np.array([(int(m) >> (25 * g)) & ((1 << 25) - 1) for m in big], np.int64)
        _check_order(km.export_perm(sp.OP_FWD, cfg, g).cpu().numpy(), key, ref.n_out)
    km.destroy()


def test_steps_alternating_between_three_streams(sp):
    """The launch pattern that bench.py times: asynchronous kmap build, forward, dgrad and wgrad of one
    batch on one stream, the next batch on the next stream, no synchronisation in between, every
    stream with kmaps and outputs of its own.  Each stream gets a cloud, features and weights of its
    own here, so that anything taken from a neighbouring stream shows; all results against the oracle."""
    lanes = []
    for i, ts in enumerate([torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream()]):
        c = gen.lidar_scene(300 + i, target_n=2600 + 700 * i)
        ref = oc.build_kmap(c, 3, 1)
        (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 64, 64, 27, "f16", 40 + i)
        lanes.append(dict(ts=ts, s=ts.cuda_stream, coords=coords_dev(c), ref=ref, x=x, w=w, g=g,
                          want=(oc.forward(x32, w32, ref.M), oc.dgrad(g32, w32, ref.M, ref.n_in),
                                oc.wgrad(x32, g32, ref.M)),
                          y=torch.empty(ref.n_out, 64, dtype=torch.float16, device="cuda"),
                          dx=torch.empty(ref.n_in, 64, dtype=torch.float16, device="cuda"),
                          dw=torch.empty(27, 64, 64, dtype=torch.float32, device="cuda"), prev=[]))
    torch.cuda.synchronize()  # (the inputs were made on the current stream)
    cfg = _cfg(sp, 0, 0, 32, kernel=1)
    for step in range(12):
        ln = lanes[step % 3]
        k = sp.build_kmap(ln["coords"], 3, 1, stream=ln["s"], asynchronous=True)
        sp.fwd(ln["x"], ln["w"], k, cfg, out=ln["y"], stream=ln["s"])
        sp.dgrad(ln["g"], ln["w"], k, cfg, out=ln["dx"], stream=ln["s"])
        sp.wgrad(ln["x"], ln["g"], k, out=ln["dw"], stream=ln["s"])
        if ln["prev"]:
            old = ln["prev"].pop()
            old.status(stream=ln["s"])  # (raises on a build error)
            old.destroy()
        ln["prev"].append(k)
    torch.cuda.synchronize()
    for ln in lanes:
        k = ln["prev"].pop()
        k.status(stream=ln["s"])
        m = k.export(stream=ln["s"])
        ln["ts"].synchronize()  # (the copy runs on the lane's stream, .cpu() on the current one)
        np.testing.assert_array_equal(m.cpu().numpy(), ln["ref"].M)
        k.destroy()
        for got, want in zip((ln["y"], ln["dx"], ln["dw"]), ln["want"]):
            assert norm_err(got, want) <= TOL["f16"]
