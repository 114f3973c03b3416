"""Seeded synthetic point clouds, features and weights.

The paper measures on real LiDAR scans (64- and 32-beam spinning sensors,
Section 5.1) voxelised by floor(p / v) followed by Unique (Section 2).  None
of those datasets is available here, so these generators stand in for them
with the same structure: a ground plane plus vertical objects seen from one
sensor with surface density falling as 1/r^2, or the surfaces of a furnished
room, quantised with the paper's rule.  Everything is drawn from
numpy.random.default_rng(seed); row order is shuffled so that no spatial
ordering comes for free.

Only input generation lives here (no part of the method's arithmetic).
"""
from __future__ import annotations

import numpy as np

# Raw-sample pools.  Each scene draws this many raw points from its seed and
# then keeps the deterministic subset (a prefix of the shuffled pool for the
# LiDAR scene, a sight radius for the room) whose voxel count is closest to
# the requested one, found by bisection.
LIDAR_RAW_GROUND = 45_000
LIDAR_RAW_OBJECT = 375_000
ROOM_RAW = 6_000_000


def uniform_cloud(n: int, grid: int, seed: int, batch: int = 0, lo: int = 0) -> np.ndarray:
    """n distinct cells drawn without replacement from a grid^3 cube whose
    lowest corner is at (lo, lo, lo)."""
    rng = np.random.default_rng(seed)
    cells = rng.choice(grid ** 3, size=n, replace=False)
    x, rem = np.divmod(cells, grid * grid)
    y, z = np.divmod(rem, grid)
    c = np.stack([np.full(n, batch), x + lo, y + lo, z + lo], axis=1)
    return c.astype(np.int32)


def full_grid(G: int, batches: int = 1, lo: int = 0, seed: int | None = None) -> np.ndarray:
    """Every cell of a G^3 cube for each batch index; rows shuffled if seeded."""
    b, x, y, z = np.meshgrid(np.arange(batches), np.arange(G) + lo, np.arange(G) + lo,
                             np.arange(G) + lo, indexing="ij")
    c = np.stack([b.ravel(), x.ravel(), y.ravel(), z.ravel()], axis=1).astype(np.int32)
    if seed is not None:
        np.random.default_rng(seed).shuffle(c, axis=0)
    return c


def _lidar_points(rng, n_ground: int, n_object: int) -> np.ndarray:
    sensor_h = 1.8
    r_min, r_max = 2.0, 50.0
    # ground: log-uniform range and uniform azimuth give areal density ~ 1/r^2
    r = np.exp(rng.uniform(np.log(r_min), np.log(r_max), n_ground))
    th = rng.uniform(0.0, 2 * np.pi, n_ground)
    ground = np.stack([r * np.cos(th), r * np.sin(th),
                       rng.normal(0.0, 0.01, n_ground)], axis=1)
    # 40 vertical objects inside the 50 m disc
    pts = [ground]
    n_obj = 40
    kinds = rng.integers(0, 2, n_obj)
    rad = np.sqrt(rng.uniform((r_min + 1) ** 2, r_max ** 2, n_obj))
    ang = rng.uniform(0, 2 * np.pi, n_obj)
    cx, cy = rad * np.cos(ang), rad * np.sin(ang)
    height = rng.uniform(1.0, 4.0, n_obj)
    cyl_r = rng.uniform(0.2, 1.0, n_obj)
    box_a = rng.uniform(1.0, 5.0, n_obj)
    box_b = rng.uniform(1.0, 5.0, n_obj)
    side_area = np.where(kinds == 0, 2 * np.pi * cyl_r * height, 2 * (box_a + box_b) * height)
    # samples per object ~ lateral area / r^2
    w = side_area / np.maximum(rad, r_min) ** 2
    counts = rng.multinomial(n_object, w / w.sum())
    for i in range(n_obj):
        m = int(counts[i])
        if m == 0:
            continue
        zc = rng.uniform(0.0, height[i], m)
        if kinds[i] == 0:
            a = rng.uniform(0, 2 * np.pi, m)
            px = cx[i] + cyl_r[i] * np.cos(a)
            py = cy[i] + cyl_r[i] * np.sin(a)
        else:
            t = rng.uniform(0, 2 * (box_a[i] + box_b[i]), m)
            ha, hb = box_a[i] / 2, box_b[i] / 2
            px = np.where(t < box_a[i], -ha + t,
                 np.where(t < box_a[i] + box_b[i], ha,
                 np.where(t < 2 * box_a[i] + box_b[i], ha - (t - box_a[i] - box_b[i]), -ha)))
            py = np.where(t < box_a[i], -hb,
                 np.where(t < box_a[i] + box_b[i], -hb + (t - box_a[i]),
                 np.where(t < 2 * box_a[i] + box_b[i], hb, hb - (t - 2 * box_a[i] - box_b[i]))))
            px, py = px + cx[i], py + cy[i]
        pts.append(np.stack([px, py, zc], axis=1))
    p = np.concatenate(pts, axis=0)
    p[:, 2] -= sensor_h  # sensor frame
    return p


def _quantize_unique(points_xyz: np.ndarray, voxel) -> np.ndarray:
    """floor(p / v) then Unique (Section 2); v a scalar or one size per axis; rows come back in sorted order."""
    q = np.floor(points_xyz / voxel).astype(np.int64)
    lo = q.min(axis=0)
    span = q.max(axis=0) - lo + 1
    flat = ((q[:, 0] - lo[0]) * span[1] + (q[:, 1] - lo[1])) * span[2] + (q[:, 2] - lo[2])
    flat = np.unique(flat)
    x, rem = np.divmod(flat, span[1] * span[2])
    y, z = np.divmod(rem, span[2])
    return np.stack([x + lo[0], y + lo[1], z + lo[2]], axis=1)


def _finish(q: np.ndarray, batch: int, rng) -> np.ndarray:
    """Shift to min 0 per axis, shuffle rows, prepend the batch index."""
    q = q - q.min(axis=0, keepdims=True)
    rng.shuffle(q, axis=0)
    b = np.full((q.shape[0], 1), batch, dtype=np.int64)
    return np.concatenate([b, q], axis=1).astype(np.int32)


def lidar_scene(seed: int, batch: int = 0, target_n: int = 100_000) -> np.ndarray:
    """One LiDAR-like scan voxelised at 0.05 m: int32 [N, 4] = (b, x, y, z)
    with N within about 1% of target_n (target_n up to ~110k)."""
    rng = np.random.default_rng(seed)
    p = _lidar_points(rng, LIDAR_RAW_GROUND, LIDAR_RAW_OBJECT)
    rng.shuffle(p, axis=0)
    lo, hi = 1, p.shape[0]
    for _ in range(12):  # N(prefix length) is monotone
        mid = (lo + hi) // 2
        if _quantize_unique(p[:mid], 0.05).shape[0] < target_n:
            lo = mid
        else:
            hi = mid
    return _finish(_quantize_unique(p[:hi], 0.05), batch, rng)


def detection_scene(seed: int, batch: int = 0) -> np.ndarray:
    """The same scan model voxelised the way 3-D detectors do (Section 2: anisotropic voxels of
    0.1 x 0.1 x 0.15 m), every raw point used: coarser cells, denser neighbourhoods."""
    rng = np.random.default_rng(seed)
    p = _lidar_points(rng, LIDAR_RAW_GROUND, LIDAR_RAW_OBJECT)
    return _finish(_quantize_unique(p, np.array([0.1, 0.1, 0.15])), batch, rng)


def lidar_batch(seed: int, batches: int, target_n: int = 100_000) -> np.ndarray:
    """`batches` independent scans (target_n voxels each) stacked with batch
    indices 0..batches-1 and the rows of the whole batch shuffled."""
    rng = np.random.default_rng(seed + 7919)
    parts = [lidar_scene(seed + 31 * b, b, target_n) for b in range(batches)]
    c = np.concatenate(parts, axis=0)
    rng.shuffle(c, axis=0)
    return c


def _rect(rng, m, origin, u, v):
    s, t = rng.uniform(0, 1, m), rng.uniform(0, 1, m)
    return origin[None, :] + s[:, None] * u[None, :] + t[:, None] * v[None, :]


def _box_faces(lo, hi):
    """Six faces of an axis-aligned box as (origin, u, v, area)."""
    d = hi - lo
    faces = []
    for ax in range(3):
        a1, a2 = (ax + 1) % 3, (ax + 2) % 3
        u = np.zeros(3); u[a1] = d[a1]
        v = np.zeros(3); v[a2] = d[a2]
        for side in (lo, hi):
            o = lo.copy(); o[ax] = side[ax]
            faces.append((o, u, v, d[a1] * d[a2]))
    return faces


def room_scene(seed: int, batch: int = 0, target_n: int = 300_000) -> np.ndarray:
    """Surfaces of a 10 x 10 x 3 m room with 30 axis-aligned boxes on the floor,
    densely sampled by area and voxelised at 0.02 m, of which a scanner in the
    middle of the room sees everything within a sight radius; the radius is
    bisected so that N is within about 1% of target_n (up to ~1M)."""
    rng = np.random.default_rng(seed)
    faces = _box_faces(np.zeros(3), np.array([10.0, 10.0, 3.0]))
    for _ in range(30):
        size = rng.uniform(0.3, 2.0, 3)
        lo = np.array([rng.uniform(0, 10 - size[0]), rng.uniform(0, 10 - size[1]), 0.0])
        faces.extend(_box_faces(lo, lo + size))
    area = np.array([f[3] for f in faces])
    counts = rng.multinomial(ROOM_RAW, area / area.sum())
    pts = [_rect(rng, int(m), f[0], f[1], f[2]) for f, m in zip(faces, counts) if m > 0]
    p = np.concatenate(pts, axis=0)
    q = _quantize_unique(p, 0.02)
    centre = (q + 0.5) * 0.02 - np.array([5.0, 5.0, 1.5])[None, :]
    r = np.sort(np.sqrt((centre ** 2).sum(axis=1)))
    radius = r[min(target_n, r.shape[0]) - 1]
    keep = np.sqrt((centre ** 2).sum(axis=1)) <= radius
    return _finish(q[keep], batch, rng)


def round_to_dtype(x32: np.ndarray, dtype: str):
    """Round float32 values to `dtype` ('f32' | 'f16' | 'bf16').  Returns
    (values as float32 that are exactly representable in dtype, raw storage
    array to upload: float32, float16, or uint16 bit patterns for bf16)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f32":
        return x32, x32
    if dtype == "f16":
        h = x32.astype(np.float16)
        return h.astype(np.float32), h
    if dtype == "bf16":
        bits = x32.view(np.uint32).astype(np.uint64)
        rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)
        back = (rounded.astype(np.uint32) << 16).view(np.float32)
        return back.reshape(x32.shape), rounded.reshape(x32.shape)
    raise ValueError(dtype)


def features(n: int, c: int, dtype: str, seed: int):
    """[n, c] ~ N(0, 1), rounded to dtype; see round_to_dtype for the return."""
    rng = np.random.default_rng(seed)
    return round_to_dtype(rng.standard_normal((n, c), dtype=np.float32), dtype)


def weights(V: int, c_in: int, c_out: int, dtype: str, seed: int):
    """[V, c_in, c_out] ~ N(0, 1/sqrt(V*c_in)) (standard deviation), rounded."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((V, c_in, c_out), dtype=np.float32) / np.float32(np.sqrt(V * c_in))
    return round_to_dtype(w, dtype)


