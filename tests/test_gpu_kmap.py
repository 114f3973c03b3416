"""Kernel maps built by the HIP library against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

from oracle import sparse_conv as oc
from workloads import generators as gen
from _util import coords_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import paper_2311_12862_amd as sp
    return sp


def _check_kmap(sp, c, K, stride, transposed):
    ref = oc.build_kmap(c, K, stride, transposed)
    km = sp.build_kmap(coords_dev(c), K, stride, transposed)
    assert (km.n_in, km.n_out) == (ref.n_in, ref.n_out)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(km.out_coords().cpu().numpy(), ref.out_coords)
    np.testing.assert_array_equal(km.in_coords().cpu().numpy(), ref.in_coords)
    mask = km.export_mask().cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(mask, oc.bitmask(ref.M))
    assert km.n_pairs() == int((ref.M >= 0).sum())
    km.destroy()
    return ref


@pytest.mark.parametrize("n,grid,lo", [(2000, 64, 0), (3000, 16, -8), (700, 9, 100)])
def test_submanifold(sp, n, grid, lo):
    c = gen.uniform_cloud(n, grid, seed=n, lo=lo)
    c[: n // 3, 0] = 2
    _check_kmap(sp, c, 3, 1, False)


@pytest.mark.parametrize("stride", [2, 3])
@pytest.mark.parametrize("lo", [0, -7])
def test_strided(sp, stride, lo):
    c = gen.uniform_cloud(4000, 20, seed=17 + stride, lo=lo)
    c[:1500, 0] = 1
    ref = _check_kmap(sp, c, 3, stride, False)
    assert ref.n_out < 4000


@pytest.mark.parametrize("transposed", [False, True])
def test_even_kernel_stride2(sp, transposed):
    """K = s = 2: the non-overlapping 2x2x2 layer and its transposed counterpart (8 offsets)."""
    c = gen.uniform_cloud(4000, 20, seed=29, lo=-6)
    c[:1300, 0] = 1
    ref = _check_kmap(sp, c, 2, 2, transposed)
    assert ref.M.shape[1] == 8
    _check_kmap(sp, gen.lidar_scene(31, target_n=30_000), 2, 2, transposed)
    _check_kmap(sp, np.array([[0, -1, 0, 3]], dtype=np.int32), 2, 2, transposed)
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(c), 2, 1, transposed)   # the even kernel exists for stride 2 only
    assert e.value.status == -1


@pytest.mark.parametrize("stride", [1, 2])
def test_transposed(sp, stride):
    c = gen.uniform_cloud(3500, 18, seed=23, lo=-5)
    c[:1000, 0] = 3
    _check_kmap(sp, c, 3, stride, True)


def test_k1(sp):
    c = gen.uniform_cloud(1000, 12, seed=5)
    _check_kmap(sp, c, 1, 1, False)
    _check_kmap(sp, c, 1, 2, False)


def test_lidar_scene_small(sp):
    c = gen.lidar_scene(2000, target_n=20_000)
    _check_kmap(sp, c, 3, 1, False)
    _check_kmap(sp, c, 3, 2, False)


def test_empty_single_and_limits(sp):
    km = sp.build_kmap(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 3, 1)
    assert (km.n_in, km.n_out, km.n_pairs()) == (0, 0, 0)
    assert km.export().shape == (0, 27)
    km.destroy()
    _check_kmap(sp, np.array([[0, 5, -3, 7]], dtype=np.int32), 3, 1, False)
    _check_kmap(sp, np.array([[0, 5, -3, 7]], dtype=np.int32), 3, 2, False)
    lim = np.array([[65534, 32767, 32767, 32767], [65534, 32766, 32767, 32766], [0, -32768, -32768, -32768],
                    [0, -32767, -32768, -32768], [0, -32768, 32767, 0]], dtype=np.int32)
    _check_kmap(sp, lim, 3, 1, False)
    _check_kmap(sp, lim, 3, 2, False)
    _check_kmap(sp, lim, 3, 2, True)


def test_errors(sp):
    c = gen.uniform_cloud(500, 10, seed=1)
    dup = c.copy()
    dup[100] = dup[400]
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(dup), 3, 1)
    assert e.value.status == -3
    with pytest.raises(ValueError):
        oc.build_kmap(dup, 3, 1)
    # duplicates and range errors are reported by every kind of build
    for stride, transposed in ((2, False), (3, False), (2, True), (1, True)):
        with pytest.raises(sp.SpconvError) as e:
            sp.build_kmap(coords_dev(dup), 3, stride, transposed)
        assert e.value.status == -3, (stride, transposed)
    r = c.copy()
    r[7] = [0, 32768, 0, 0]
    for stride, transposed in ((2, False), (2, True)):
        with pytest.raises(sp.SpconvError) as e:
            sp.build_kmap(coords_dev(r), 3, stride, transposed)
        assert e.value.status == -2, (stride, transposed)
    for bad in ([0, 32768, 0, 0], [0, 0, -32769, 0], [65535, 0, 0, 0], [-1, 0, 0, 0]):
        r = c.copy()
        r[7] = bad
        with pytest.raises(sp.SpconvError) as e:
            sp.build_kmap(coords_dev(r), 3, 1)
        assert e.value.status == -2
    for K, stride in ((2, 1), (5, 2), (7, 1), (3, 0), (3, 65)):
        with pytest.raises(sp.SpconvError) as e:
            sp.build_kmap(coords_dev(c), K, stride)
        assert e.value.status == -1
    # the library still works after the error paths
    _check_kmap(sp, c, 3, 1, False)


def test_planar_and_line_sets(sp):
    """Degenerate sets (constant z, constant y and z) load one slot class of the hash table."""
    rng = np.random.default_rng(5)
    xy = rng.permutation(90 * 90)[:5000]
    plane = np.stack([np.zeros(5000, np.int64), xy // 90, xy % 90, np.full(5000, 8)], axis=1).astype(np.int32)
    _check_kmap(sp, plane, 3, 1, False)
    _check_kmap(sp, plane, 3, 2, False)
    line = np.stack([np.zeros(3000, np.int64), rng.permutation(6000)[:3000] - 3000, np.full(3000, -4),
                     np.full(3000, 12)], axis=1).astype(np.int32)
    _check_kmap(sp, line, 3, 1, False)
    _check_kmap(sp, line, 3, 2, True)


def test_build_is_deterministic(sp):
    c = gen.uniform_cloud(5000, 24, seed=9)
    a = sp.build_kmap(coords_dev(c), 3, 2)
    b = sp.build_kmap(coords_dev(c), 3, 2)
    assert torch.equal(a.export(), b.export())
    assert torch.equal(a.out_coords(), b.out_coords())


def test_asynchronous_build(sp):
    """spconv_build_kmap_async returns at once; errors and the pair count arrive with spconv_kmap_status."""
    c = gen.lidar_scene(11, target_n=6000)
    ref = oc.build_kmap(c, 3, 1)
    km = sp.build_kmap(coords_dev(c), 3, 1, asynchronous=True)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(km.export_mask().cpu().numpy().view(np.uint32), oc.bitmask(ref.M))
    km.status()
    assert km.n_pairs() == int((ref.M >= 0).sum())
    dup = c.copy()
    dup[5] = dup[77]
    km = sp.build_kmap(coords_dev(dup), 3, 1, asynchronous=True)
    with pytest.raises(sp.SpconvError) as e:
        km.status()
    assert e.value.status == -3
    with pytest.raises(sp.SpconvError) as e:   # the verdict stays with the kmap
        km.status()
    assert e.value.status == -3
    # calls that resolve the pending build on their own (pair count, executed MACs, tuner) do not swallow it
    import torch
    for resolve in (lambda k: k.n_pairs(), lambda k: k.mac_units(sp.OP_FWD),
                    lambda k: sp.tune(k, 16, 16, torch.float16, sp.OP_WGRAD, 1)):
        km = sp.build_kmap(coords_dev(dup), 3, 1, asynchronous=True)
        resolve(km)
        with pytest.raises(sp.SpconvError) as e:
            km.status()
        assert e.value.status == -3
    bad = c.copy()
    bad[9, 2] = 40000
    km = sp.build_kmap(coords_dev(bad), 3, 1, asynchronous=True)
    with pytest.raises(sp.SpconvError) as e:
        km.status()
    assert e.value.status == -2
    # map kinds without an asynchronous path are built synchronously by the same call
    km = sp.build_kmap(coords_dev(c), 3, 2, asynchronous=True)
    np.testing.assert_array_equal(km.export().cpu().numpy(), oc.build_kmap(c, 3, 2).M)


def test_caller_allocator_backs_every_device_allocation(sp):
    """spconv_set_allocator: with PyTorch's caching allocator installed, builds, plans and
    kernels run out of its blocks, results do not change, and every block comes back."""
    import torch
    from _util import TOL, make_layer, norm_err
    c = gen.lidar_scene(91, target_n=3000)
    ref = oc.build_kmap(c, 3, 2)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 32, 64, 27, "f16", 92)
    live, calls = {}, [0, 0]

    def alloc(n, stream):
        t = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
        live[t.data_ptr()] = t
        calls[0] += 1
        return t.data_ptr()

    def free(ptr, stream):
        calls[1] += 1
        live.pop(ptr)

    sp.set_allocator(alloc, free)
    try:
        km = sp.build_kmap(coords_dev(c), 3, 2)
        np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
        cfg = sp.Config()
        cfg.n_split, cfg.kernel = 2, 2                     # sorted plan and split partial sums
        assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
        assert norm_err(sp.dgrad(g, w, km), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
        assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
        assert calls[0] > 5 and live
        torch.cuda.synchronize()
        km.destroy()
        assert not live and calls[0] == calls[1]
    finally:
        sp.set_allocator(None, None)
    km = sp.build_kmap(coords_dev(c), 3, 2)                # the library's own pool serves again
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)


def test_stream_ordered_allocator_on_a_side_stream(sp):
    """The allocator callbacks receive the stream of the call in progress.  A stream-ordered
    caching allocator (PyTorch's, which only reuses a block on the stream it was allocated on)
    backs a kmap that lives entirely on a non-default stream: every callback names that stream,
    results match the oracle, and every block comes back."""
    import torch
    from _util import TOL, make_layer, norm_err
    c = gen.lidar_scene(95, target_n=3000)
    ref = oc.build_kmap(c, 3, 2)
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 32, 64, 27, "f16", 96)
    side = torch.cuda.Stream()
    live, seen = {}, set()

    def alloc(n, stream):
        seen.add(stream)
        with torch.cuda.stream(torch.cuda.ExternalStream(stream) if stream else torch.cuda.default_stream()):
            t = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")   # the caching allocator files it under that stream
        live[t.data_ptr()] = t
        return t.data_ptr()

    def free(ptr, stream):
        seen.add(stream)
        live.pop(ptr)        # back to the allocator's pool of the stream it was allocated on

    coords = coords_dev(c)
    torch.cuda.synchronize()
    sp.set_allocator(alloc, free)
    try:
        with torch.cuda.stream(side):
            for rep in range(3):                            # blocks are recycled between the rounds
                km = sp.build_kmap(coords, 3, 2)
                cfg = sp.Config()
                cfg.n_split, cfg.kernel = 2, 1 + rep % 2
                y = sp.fwd(x, w, km, cfg)
                dx = sp.dgrad(g, w, km, cfg)
                dw = sp.wgrad(x, g, km)
                m = km.export()
                km.destroy()
                side.synchronize()
                np.testing.assert_array_equal(m.cpu().numpy(), ref.M)
                assert norm_err(y, oc.forward(x32, w32, ref.M)) <= TOL["f16"]
                assert norm_err(dx, oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
                assert norm_err(dw, oc.wgrad(x32, g32, ref.M)) <= 1e-4
                assert not live
        assert seen == {side.cuda_stream}
    finally:
        sp.set_allocator(None, None)


@pytest.mark.parametrize("K,stride", [(3, 2), (2, 2), (3, 1), (3, 3), (1, 1)])
def test_transpose_equals_transposed_build(sp, K, stride):
    """spconv_kmap_transpose: the paired transposed convolution's kmap, derived without a rebuild,
    is bit for bit what a build with `transposed` flipped returns (and what the oracle defines)."""
    from _util import TOL, make_layer, norm_err
    c = gen.lidar_scene(93, target_n=2600)
    ref = oc.build_kmap(c, K, stride, False)
    ref_t = oc.build_kmap(c, K, stride, True)
    km = sp.build_kmap(coords_dev(c), K, stride)
    kt = km.transpose()
    assert (kt.n_in, kt.n_out) == (ref_t.n_in, ref_t.n_out) == (km.n_out, km.n_in)
    assert kt.n_pairs() == km.n_pairs() == int((ref.M >= 0).sum())
    np.testing.assert_array_equal(kt.export().cpu().numpy(), ref_t.M)
    direct = sp.build_kmap(coords_dev(c), K, stride, transposed=True)
    np.testing.assert_array_equal(kt.export_mask().cpu().numpy(), direct.export_mask().cpu().numpy())
    np.testing.assert_array_equal(kt.out_coords().cpu().numpy(), direct.out_coords().cpu().numpy())
    np.testing.assert_array_equal(kt.in_coords().cpu().numpy(), direct.in_coords().cpu().numpy())
    # the derived kmap runs every operator, under sorted plans as well
    (x32, x), (w32, w), (g32, g) = make_layer(ref_t.n_in, ref_t.n_out, 32, 16, K ** 3, "f16", 94)
    cfg = sp.Config()
    cfg.n_split = 1
    assert norm_err(sp.fwd(x, w, kt, cfg), oc.forward(x32, w32, ref_t.M)) <= TOL["f16"]
    assert norm_err(sp.dgrad(g, w, kt, cfg), oc.dgrad(g32, w32, ref_t.M, ref_t.n_in)) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, kt), oc.wgrad(x32, g32, ref_t.M)) <= 1e-4
    # and transposing twice gives the original structure back (also from a transposed build)
    np.testing.assert_array_equal(kt.transpose().export().cpu().numpy(), ref.M)
    back = direct.transpose()
    np.testing.assert_array_equal(back.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(back.out_coords().cpu().numpy(), km.out_coords().cpu().numpy())
    np.testing.assert_array_equal(back.in_coords().cpu().numpy(), km.in_coords().cpu().numpy())


def test_transpose_of_empty_and_pending_builds(sp):
    import torch
    empty = sp.build_kmap(torch.zeros((0, 4), dtype=torch.int32, device="cuda"), 3, 2)
    t = empty.transpose()
    assert (t.n_in, t.n_out) == (0, 0)
    c = gen.lidar_scene(95, target_n=1500)
    ref_t = oc.build_kmap(c, 3, 1, True)
    km = sp.build_kmap(coords_dev(c), 3, 1, asynchronous=True)
    np.testing.assert_array_equal(km.transpose().export().cpu().numpy(), ref_t.M)   # resolves the build first
    dup = np.vstack([c, c[:1]])
    bad = sp.build_kmap(coords_dev(dup), 3, 1, asynchronous=True)
    with pytest.raises(sp.SpconvError) as e:
        bad.transpose()
    assert e.value.status == -3          # SPCONV_EDUP


@pytest.mark.parametrize("stride,transposed", [(1, False), (1, True), (2, False), (2, True), (3, False)])
def test_pointwise_equals_a_k1_build(sp, stride, transposed):
    """spconv_kmap_pointwise: the K = 1 kmap over either row set of a kmap is what a K = 1 build on
    those rows returns (map, mask, coordinates, sizes), and a 1x1x1 layer through it is X . W[0]."""
    import torch
    from _util import make_layer, norm_err, TOL
    c = gen.lidar_scene(96, target_n=2200)
    ref = oc.build_kmap(c, 3, stride, transposed)
    km = sp.build_kmap(coords_dev(c), 3, stride, transposed)
    for on_outputs, rows_ref in ((False, ref.in_coords), (True, ref.out_coords)):
        one_ref = oc.build_kmap(rows_ref, 1, 1)
        got = km.pointwise(on_outputs)
        want = sp.build_kmap(coords_dev(rows_ref), 1, 1)
        assert (got.n_in, got.n_out, got.n_pairs()) == (one_ref.n_in, one_ref.n_out, len(rows_ref))
        np.testing.assert_array_equal(got.export().cpu().numpy(), one_ref.M)
        np.testing.assert_array_equal(got.export().cpu().numpy(), want.export().cpu().numpy())
        np.testing.assert_array_equal(got.export_mask().cpu().numpy(), want.export_mask().cpu().numpy())
        np.testing.assert_array_equal(got.out_coords().cpu().numpy(), rows_ref)
        (x32, x), (w32, w), (g32, g) = make_layer(one_ref.n_in, one_ref.n_out, 32, 48, 1, "f16", 61)
        assert norm_err(sp.fwd(x, w, got), x32.astype(np.float64) @ w32[0].astype(np.float64)) <= TOL["f16"]
        assert norm_err(sp.dgrad(g, w, got), oc.dgrad(g32, w32, one_ref.M, one_ref.n_in)) <= TOL["f16"]
        assert norm_err(sp.wgrad(x, g, got), oc.wgrad(x32, g32, one_ref.M)) <= 1e-4


def test_pointwise_of_empty_and_pending_builds(sp):
    import torch
    empty = sp.build_kmap(torch.zeros((0, 4), dtype=torch.int32, device="cuda"), 3, 1)
    one = empty.pointwise()
    assert (one.n_in, one.n_out, one.n_pairs()) == (0, 0, 0)
    c = gen.lidar_scene(97, target_n=1500)
    km = sp.build_kmap(coords_dev(c), 3, 1, asynchronous=True)
    np.testing.assert_array_equal(km.pointwise().export().cpu().numpy(), np.arange(len(c), dtype=np.int32)[:, None])
    bad = sp.build_kmap(coords_dev(np.vstack([c, c[:1]])), 3, 1, asynchronous=True)
    with pytest.raises(sp.SpconvError) as e:
        bad.pointwise()
    assert e.value.status == -3          # SPCONV_EDUP


def test_transposed_partner_outlives_its_source(sp):
    """A kmap and its transpose share their tables by reference count: either may be destroyed
    first, and dropping the source's plans leaves the partner's map intact."""
    c = gen.lidar_scene(98, target_n=1800)
    ref_t = oc.build_kmap(c, 3, 2, True)
    down = sp.build_kmap(coords_dev(c), 3, 2)
    up = down.transpose()
    down.drop_plans()
    np.testing.assert_array_equal(up.export().cpu().numpy(), ref_t.M)
    down.destroy()
    np.testing.assert_array_equal(up.export().cpu().numpy(), ref_t.M)
    np.testing.assert_array_equal(up.out_coords().cpu().numpy(), ref_t.out_coords)
    again = up.transpose()          # back to the strided map, from the partner alone
    np.testing.assert_array_equal(again.export().cpu().numpy(), oc.build_kmap(c, 3, 2).M)
    up.destroy()
    np.testing.assert_array_equal(again.export().cpu().numpy(), oc.build_kmap(c, 3, 2).M)


@pytest.mark.parametrize("seed,n", [(51, 40), (52, 3000)])
def test_dilated_stride1_output_set(sp, seed, n):
    """spconv_build_kmap_dilated: P_out = every point with an input in its neighbourhood (Eq. 1 with
    P_out != P_in).  Output set, map and masks bit-exact against the oracle; features within tolerance."""
    import torch
    from _util import TOL, make_layer, norm_err
    c = gen.lidar_scene(seed, target_n=n) if n > 100 else gen.uniform_cloud(n, 6, seed, lo=-3)
    ref = oc.build_kmap(c, 3, 1, dilate=True)
    km = sp.build_kmap(coords_dev(c), 3, 1, dilate=True)
    assert (km.n_in, km.n_out) == (ref.n_in, ref.n_out) and km.n_out > km.n_in
    np.testing.assert_array_equal(km.out_coords().cpu().numpy(), ref.out_coords)
    np.testing.assert_array_equal(km.in_coords().cpu().numpy(), c)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(km.export_mask().cpu().numpy().view(np.uint32), oc.bitmask(ref.M))
    assert km.n_pairs() == int((ref.M >= 0).sum()) == 27 * ref.n_in      # every input is read by 27 outputs
    (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, 32, 64, 27, "f16", seed)
    for n_split, kernel in ((0, 0), (1, 1), (2, 2)):
        cfg = sp.Config()
        cfg.n_split, cfg.kernel = n_split, kernel
        assert norm_err(sp.fwd(x, w, km, cfg), oc.forward(x32, w32, ref.M)) <= TOL["f16"]
        assert norm_err(sp.dgrad(g, w, km, cfg), oc.dgrad(g32, w32, ref.M, ref.n_in)) <= TOL["f16"]
    assert norm_err(sp.wgrad(x, g, km), oc.wgrad(x32, g32, ref.M)) <= 1e-4
    pw = km.pointwise(on_outputs=True)                                   # 1x1x1 layer over the dilated rows
    np.testing.assert_array_equal(pw.out_coords().cpu().numpy(), ref.out_coords)
    with pytest.raises(sp.SpconvError) as e:
        km.transpose()
    assert e.value.status == -1


def test_dilated_errors_and_k1(sp):
    import torch
    c = gen.uniform_cloud(200, 9, 53)
    ref = oc.build_kmap(c, 1, 1, dilate=True)                            # K = 1: the inputs, sorted
    km = sp.build_kmap(coords_dev(c), 1, 1, dilate=True)
    np.testing.assert_array_equal(km.out_coords().cpu().numpy(), ref.out_coords)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    edge = c.copy()
    edge[3] = (0, -32768, 5, 5)                                          # its neighbour at x - 1 cannot be packed
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(edge), 3, 1, dilate=True)
    assert e.value.status == -2
    dup = c.copy()
    dup[7] = dup[9]
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(dup), 3, 1, dilate=True)
    assert e.value.status == -3
    lib = sp.load_library()
    import ctypes
    out = ctypes.c_void_p()
    assert lib.spconv_build_kmap_dilated(None, 0, 5, None, ctypes.byref(out)) == -1
    assert lib.spconv_build_kmap_dilated(None, 0, 2, None, ctypes.byref(out)) == -1
    empty = sp.build_kmap(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 3, 1, dilate=True)
    assert empty.n_out == 0


def _mask_words(big, words):
    """Python-int bitmasks -> uint32 [n][words], bit k in bit k % 32 of word k // 32."""
    out = np.zeros((len(big), words), np.uint32)
    for r, m in enumerate(big):
        m = int(m)
        for w in range(words):
            out[r, w] = (m >> (32 * w)) & 0xFFFFFFFF
    return out


@pytest.mark.parametrize("n,grid,lo", [(2000, 20, 0), (3000, 16, -8), (300, 7, 32760)])
def test_k5_submanifold_map_and_masks(sp, n, grid, lo):
    """K = 5 (125 offsets, Section 2.1's neighbourhood for any odd K): the library holds the map as five
    25-offset planes; what it exports is the whole map, bit for bit the oracle's, with 125-bit masks."""
    c = gen.uniform_cloud(n, grid, seed=500 + n, lo=lo)
    c[: n // 4, 0] = 3
    ref = oc.build_kmap(c, 5, 1)
    km = sp.build_kmap(coords_dev(c), 5, 1)
    assert (km.n_in, km.n_out, km.V) == (ref.n_in, ref.n_out, 125)
    np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M)
    np.testing.assert_array_equal(km.in_coords().cpu().numpy(), ref.in_coords)
    np.testing.assert_array_equal(km.out_coords().cpu().numpy(), ref.out_coords)
    words = km.export_mask().cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(words, _mask_words(oc.bitmask(ref.M), 4))
    assert km.n_pairs() == int((ref.M >= 0).sum())
    km.destroy()


def test_k5_refusals(sp):
    """K = 5 exists as a submanifold map only; duplicates and rows beside the range fail as for K = 3."""
    c = gen.uniform_cloud(500, 16, seed=77)
    for stride, transposed in ((2, False), (1, True)):
        with pytest.raises(sp.SpconvError) as e:
            sp.build_kmap(coords_dev(c), 5, stride, transposed)
        assert e.value.status == -1
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(c), 5, 1, asynchronous=True)
    assert e.value.status == -1
    dup = np.concatenate([c, c[:1]])
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(dup), 5, 1)
    assert e.value.status == -3
    far = c.copy()
    far[3, 2] = 40000
    with pytest.raises(sp.SpconvError) as e:
        sp.build_kmap(coords_dev(far), 5, 1)
    assert e.value.status == -2
    km = sp.build_kmap(coords_dev(c), 5, 1)
    with pytest.raises(sp.SpconvError) as e:
        km.transpose()
    assert e.value.status == -1
    km.destroy()
