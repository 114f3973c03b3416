"""Launch arithmetic of the forward / dgrad kernels, checked on the CPU (no GPU call).

spconv_describe_launch reports what the library's run functions derive from a layer's shape
(they take it from the same host functions).  Here the index formulas of the two GEMM kernels
are walked over a grid of shapes - row counts around every tile boundary, every split count,
channel counts from 8 to 256, every tile shape - and every index a kernel can form is shown to
stay inside the table it addresses, every block to be visited exactly once, and every LDS plan
to fit the CU.  Degenerate shapes must be refused with SPCONV_EINVAL, not launched."""
import itertools

import pytest
import torch

import paper_2311_12862_amd as sp

LDS_PER_CU = 160 * 1024
ROWS = [1, 15, 16, 17, 255, 256, 257, 4097, 100049]
CHANNELS = [8, 16, 24, 32, 64, 96, 128, 256]


def _describe(K, rows, c_red, c_cols, dtype, dgrad=False, rows_src=None, **cfg_fields):
    cfg = sp.Config()
    for k, v in cfg_fields.items():
        setattr(cfg, k, v)
    try:
        return sp.describe_launch(K, rows, rows if rows_src is None else rows_src, c_red, c_cols, dtype, cfg, dgrad)
    except sp.SpconvError as e:
        assert e.status == -1, e
        return None


def _wave_blocks(info, x):
    """Blocks that workgroup x of a slice draws (the kernel's block_of over its tickets)."""
    n_blocks, gx = info.n_tiles, info.grid[0]
    n_rng = 8 if info.xcd_ranges else 1
    rng, wi = (x & 7, x >> 3) if info.xcd_ranges else (0, x)
    wpr = gx // n_rng
    rlo, rhi = n_blocks * rng // n_rng, n_blocks * (rng + 1) // n_rng
    nj = (rhi - rlo - wi + wpr - 1) // wpr if rhi - rlo > wi else 0
    return [rlo + (nj - 1 - t) * wpr + wi for t in range(nj)]


def _check_kernel1(info, V, rows, c_red, c_cols, n_split):
    assert info.tile_m == 16 and info.threads == 64 * info.waves and info.threads in (512, 1024)
    assert info.parts == max(1, n_split) and info.grid[2] == info.parts
    assert info.tile_n in (16, 32, 64) and info.grid[1] == -(-c_cols // info.tile_n)
    assert info.k_steps == -(-c_red // 32) <= 4
    max_width = max(info.width[:info.parts])
    assert sum(info.width[:info.parts]) == V and info.lo[0] == 0
    # LDS: resident weights of the widest part + one slab per wave (map rows, then the output tile)
    assert info.slab_map_bytes >= 16 * max_width * 4
    assert info.slab_bytes >= info.slab_map_bytes + (16 * info.tile_n * 2 if info.parts == 1 else 0)
    assert info.lds_bytes == max_width * info.tile_n * info.k_steps * 64 + info.waves * info.slab_bytes
    assert info.lds_bytes + 64 <= LDS_PER_CU
    assert info.n_tiles == -(-rows // 16) and info.rows_pad % 256 == 0 and info.rows_pad >= rows
    gx = info.grid[0]
    assert 1 <= gx and gx * info.grid[1] * info.grid[2] <= 256 + 7
    if info.xcd_ranges:
        assert gx % 8 == 0
    seen = []
    for x in range(gx):
        seen += _wave_blocks(info, x)
    assert sorted(seen) == list(range(info.n_tiles))          # every block once, none beyond the last
    b = info.n_tiles - 1
    for i in range(info.parts):
        width = V if n_split == 0 else info.width[i]
        assert (b + 1) * 16 * width <= info.map_elems[i]       # last map element a lane reads
    assert b * 16 + 15 < info.rows_pad                          # permutation / row-mask entry


def _check_kernel2(info, V, rows, c_red, c_cols, n_split, f32):
    assert info.tile_m in (64, 128, 256) and info.threads == 64 * info.waves and info.waves in (4, 8)
    assert info.grid[0] == info.n_tiles == -(-rows // info.tile_m) and info.grid[2] == info.parts == max(1, n_split)
    assert info.grid[1] == -(-c_cols // info.tile_n)
    assert 0 < info.lds_bytes <= LDS_PER_CU
    assert info.rows_pad % 256 == 0 and info.n_tiles * info.tile_m <= info.rows_pad   # a tile's slab ends inside the map
    for i in range(info.parts):
        width = V if n_split == 0 else info.width[i]
        assert info.n_tiles * info.tile_m * width <= info.map_elems[i]
    if not f32:
        assert info.k_steps == (64 if c_red % 64 == 0 else 32)


@pytest.mark.parametrize("K", [1, 2, 3])
def test_every_index_stays_in_range(K):
    V = K ** 3
    checked = refused = 0
    for rows, c_red, c_cols, n_split in itertools.product(ROWS, CHANNELS, [8, 32, 64, 96, 256], range(5)):
        for kernel, tile_m, tile_n in [(0, 0, 0), (1, 0, 16), (1, 0, 32), (1, 0, 64), (2, 64, 0), (2, 128, 32),
                                       (2, 256, 64), (2, 128, 128)]:
            for flags in ((0, 1) if kernel != 2 and n_split else (0,)):
                info = _describe(K, rows, c_red, c_cols, torch.float16, n_split=n_split, kernel=kernel, tile_m=tile_m,
                                 tile_n=tile_n, flags=flags)
                if info is None:
                    refused += 1
                    assert n_split > V or kernel == 1 or (kernel == 2 and tile_n == 16)
                    continue
                checked += 1
                if info.kernel == 1:
                    _check_kernel1(info, V, rows, c_red, c_cols, n_split)
                else:
                    _check_kernel2(info, V, rows, c_red, c_cols, n_split, False)
    assert checked > 1000 and refused > 0


def test_fp32_path_and_dgrad_layout():
    for rows, c in itertools.product(ROWS, [4, 12, 16, 64]):
        for n_split in range(5):
            info = _describe(3, rows, c, c, torch.float32, n_split=n_split)
            assert info.kernel == 2 and info.tile_m == 64 and info.threads == 256
            _check_kernel2(info, 27, rows, c, c, n_split, True)
    for rows, c_red, c_cols in itertools.product(ROWS, CHANNELS, CHANNELS):
        info = _describe(3, rows, c_red, c_cols, torch.bfloat16, dgrad=True, kernel=2, tile_m=128)
        _check_kernel2(info, 27, rows, c_red, c_cols, 0, False)


def test_degenerate_shapes_are_refused():
    lib = sp.load_library()
    ok = lambda **kw: _describe(3, 1000, 64, 64, torch.float16, **kw)
    assert ok() is not None
    assert ok(n_split=5) is None and ok(n_split=-1) is None
    assert ok(tile_m=100) is None and ok(tile_n=48) is None and ok(kernel=7) is None and ok(flags=2) is None
    assert ok(kernel=1, tile_n=64) is None                      # 27 x 64 x 64 fp16 weights do not fit in LDS
    assert ok(kernel=1, tile_n=64, n_split=2) is not None
    assert _describe(1, 1000, 64, 64, torch.float16, n_split=2) is None   # more parts than offsets
    assert _describe(2, 1000, 64, 64, torch.float16, n_split=4) is not None
    assert _describe(3, 1000, 60, 64, torch.float16) is None and _describe(3, 1000, 64, 0, torch.float16) is None
    assert _describe(3, 1000, 160, 64, torch.float16, kernel=1) is None   # kernel 1 reduces over at most 128 channels
    assert _describe(3, 1000, 64, 64, torch.float16, kernel=3) is None
    # a gathered tensor that 32-bit buffer offsets cannot address
    assert _describe(3, 1000, 64, 64, torch.float16, rows_src=40_000_000) is None
    assert _describe(3, 1000, 24, 64, torch.float16, rows_src=50_000_000, kernel=1) is None
    # an empty side launches nothing
    info = _describe(3, 0, 64, 64, torch.float16)
    assert info.kernel == 0 and list(info.grid) == [0, 0, 0] and info.lds_bytes == 0
    out = sp.LaunchInfo()
    assert lib.spconv_describe_launch(4, 10, 10, 64, 64, 1, None, 0, out) == -1
    assert lib.spconv_describe_launch(3, -1, 10, 64, 64, 1, None, 0, out) == -1
    assert lib.spconv_describe_launch(3, 10, 10, 64, 64, 1, None, 0, None) == -1
