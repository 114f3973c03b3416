"""spconv_fwd_noalloc (the entry point for callers that cannot allocate) against spconv_fwd:
same kernels, partial sums in the library's fixed scratch array instead of a kmap buffer.
Two calls in a row, the second on a smaller input, each checked against spconv_fwd and the oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2311_12862_amd as sp
from oracle import sparse_conv as oc
from workloads import generators as gen

from _util import TOL, coords_dev, make_layer, norm_err

pytestmark = pytest.mark.gpu


def _case(seed, n, c_in, c_out, dtype="f16"):
    c = gen.lidar_scene(seed, target_n=n)
    ref = oc.build_kmap(c, 3, 1)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    (x32, x), (w32, w), _ = make_layer(ref.n_in, ref.n_out, c_in, c_out, 27, dtype, seed)
    return ref, km, x32, x, w32, w


def _raw_noalloc(x, w, km, c_in, c_out, cfg, out):
    """The C call itself, arguments marshalled by hand."""
    lib = sp.load_library()
    return lib.spconv_fwd_noalloc(x.data_ptr(), w.data_ptr(), km.handle, c_in, c_out, 1, C.byref(cfg),
                                  out.data_ptr(), torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("kernel,n_split", [(1, 2), (2, 3), (1, 4)])
def test_two_calls_in_a_row_second_smaller(kernel, n_split):
    cfg = sp.Config()
    cfg.kernel, cfg.n_split = kernel, n_split
    big = _case(31, 20000, 64, 64)
    small = _case(32, 3000, 64, 32)
    outs = []
    for ref, km, x32, x, w32, w in (big, small):
        c_in, c_out = w.shape[1], w.shape[2]
        out = torch.full((km.n_out, c_out), float("nan"), dtype=torch.float16, device="cuda")
        # no plan yet: refused, nothing written
        assert _raw_noalloc(x, w, km, c_in, c_out, cfg, out) == -7
        assert torch.isnan(out).all()
        km.prepare(sp.OP_FWD, cfg)
        want = sp.fwd(x, w, km, cfg)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        assert _raw_noalloc(x, w, km, c_in, c_out, cfg, out) == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        outs.append((out, want, x32, w32, ref))
    for out, want, x32, w32, ref in outs:
        assert torch.equal(out, want)          # same kernels, same order of additions
        assert norm_err(out, oc.forward(x32, w32, ref.M)) <= TOL["f16"]
    # the big case once more after the small one: the shared array holds the small call's sums
    ref, km, x32, x, w32, w = big
    out = sp.fwd_noalloc(x, w, km, torch.empty_like(outs[0][0]), cfg)
    assert torch.equal(out, outs[0][1])


def test_unsplit_plan_and_limits():
    ref, km, x32, x, w32, w = _case(33, 3000, 64, 64)
    out = torch.empty((km.n_out, 64), dtype=torch.float16, device="cuda")
    cfg = sp.Config()
    cfg.kernel, cfg.n_split = 1, 1
    km.prepare(sp.OP_FWD, cfg)
    assert torch.equal(sp.fwd_noalloc(x, w, km, out, cfg), sp.fwd(x, w, km, cfg))
    fod = sp.Config()
    fod.kernel = 3
    assert _raw_noalloc(x, w, km, 64, 64, fod, out) == -1
    lib = sp.load_library()
    assert lib.spconv_strerror(-7).decode().startswith("no prepared plan")
    assert lib.spconv_strerror(-8).decode().startswith("partial sums exceed")


def test_partial_sums_beyond_the_fixed_array_are_refused():
    # 4 parts x 70k rows x 64 channels x 4 B = 71.7 MB > 64 MiB
    c = gen.lidar_scene(34, target_n=70000)
    km = sp.build_kmap(coords_dev(c), 3, 1)
    x = torch.zeros((km.n_in, 64), dtype=torch.float16, device="cuda")
    w = torch.zeros((27, 64, 64), dtype=torch.float16, device="cuda")
    out = torch.full((km.n_out, 64), float("nan"), dtype=torch.float16, device="cuda")
    cfg = sp.Config()
    cfg.kernel, cfg.n_split = 1, 4
    km.prepare(sp.OP_FWD, cfg)
    assert 4 * km.n_out * 64 * 4 > (64 << 20)
    assert _raw_noalloc(x, w, km, 64, 64, cfg, out) == -8
    torch.cuda.synchronize()
    assert torch.isnan(out).all()
    cfg.n_split = 2
    km.prepare(sp.OP_FWD, cfg)
    assert _raw_noalloc(x, w, km, 64, 64, cfg, out) == 0
    torch.cuda.synchronize()
    assert (out == 0).all()
