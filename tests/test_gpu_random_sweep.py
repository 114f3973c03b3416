"""Seeded random sweep: cloud kind and size, map kind, dtype, channel counts and configuration are
drawn together, so that combinations no hand-written case names get exercised (ragged sizes,
channel counts that fill no tile, splits of narrow maps, every kernel and tile).  Every case:
kmap bit-exact, forward / dgrad / wgrad against the plain definition; a configuration that does
not fit the shape must be refused with SPCONV_EINVAL, never miscomputed."""
import numpy as np
import pytest

from oracle import sparse_conv as oc
from workloads import generators as gen
from _util import TOL, coords_dev, make_layer, norm_err

pytestmark = pytest.mark.gpu

MAP_KINDS = [(3, 1, False), (3, 1, False), (3, 2, False), (3, 2, True), (2, 2, False), (2, 2, True), (1, 1, False),
             (3, 3, False), (3, 1, True)]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_layers(seed):
    import paper_2311_12862_amd as sp
    rng = np.random.default_rng(seed)
    for case in range(40):
        kind = int(rng.integers(0, 3))
        n = int(rng.choice([1, 7, 63, 64, 65, 300, 1023, 2500, 6000]))
        if kind == 0:
            grid = int(max(4, round((n * rng.uniform(2, 30)) ** (1 / 3)) + 1))
            c = gen.uniform_cloud(n, grid, seed=int(rng.integers(1 << 30)))
        elif kind == 1:
            c = gen.lidar_scene(int(rng.integers(1 << 20)), target_n=max(n, 500))
        else:
            c = gen.full_grid(int(rng.integers(3, 9)), 2, seed=int(rng.integers(1 << 30)))
        K, stride, transposed = MAP_KINDS[int(rng.integers(0, len(MAP_KINDS)))]
        dtype = ["f16", "bf16", "f32"][int(rng.integers(0, 3))]
        q = 4 if dtype == "f32" else 8
        c_in, c_out = int(rng.integers(1, 18)) * q, int(rng.integers(1, 18)) * q
        what = f"seed {seed} case {case}: n={len(c)} K={K} stride={stride} transposed={transposed} {dtype} {c_in}->{c_out}"
        ref = oc.build_kmap(c, K, stride, transposed)
        (x32, x), (w32, w), (g32, g) = make_layer(ref.n_in, ref.n_out, c_in, c_out, K ** 3, dtype,
                                                  int(rng.integers(1 << 20)))
        km = sp.build_kmap(coords_dev(c), K, stride, transposed)
        np.testing.assert_array_equal(km.export().cpu().numpy(), ref.M, err_msg=what)
        want = {"fwd": oc.forward(x32, w32, ref.M), "dgrad": oc.dgrad(g32, w32, ref.M, ref.n_in),
                "wgrad": oc.wgrad(x32, g32, ref.M)}
        cfgs = [None]
        for _ in range(3):
            cf = sp.Config()
            cf.kernel, cf.n_split = int(rng.integers(0, 4)), int(rng.integers(0, 5))
            cf.tile_m, cf.tile_n = int(rng.choice([0, 64, 128, 256])), int(rng.choice([0, 16, 32, 64, 128]))
            cf.wgrad_pairs = int(rng.choice([0, 0, 100, 1024, 5000]))
            cfgs.append(cf)
        for cf in cfgs:
            for op, run, tol in (("fwd", lambda: sp.fwd(x, w, km, cf), TOL[dtype]),
                                 ("dgrad", lambda: sp.dgrad(g, w, km, cf), TOL[dtype]),
                                 ("wgrad", lambda: sp.wgrad(x, g, km, cf), 1e-4)):
                try:
                    got = run()
                except sp.SpconvError as e:
                    assert e.status == -1, (what, op, repr(cf), e)   # refused: SPCONV_EINVAL only
                    continue
                if want[op].size:
                    assert norm_err(got, want[op]) <= tol, (what, op, repr(cf))
        km.destroy()
