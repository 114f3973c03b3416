"""The synthetic inputs keep to their recipe (shapes and statistics the paper states for its
workloads: voxelised scans with unique rows, a few neighbours per voxel, batch index as a coordinate).
CPU only; the oracle's kmap supplies the neighbour counts."""
import numpy as np
import pytest

from oracle import sparse_conv as oc
from workloads import generators as gen


def _neighbours_per_voxel(c):
    km = oc.build_kmap(c, 3, 1)
    return (km.M >= 0).sum() / len(c)


def _common(c, batches=1):
    assert c.dtype == np.int32 and c.ndim == 2 and c.shape[1] == 4
    assert len(np.unique(c, axis=0)) == len(c)                       # Unique was applied (Section 2)
    assert (c[:, 1:].min(axis=0) == 0).all()                         # shifted to the origin
    assert set(np.unique(c[:, 0])) == set(range(batches))
    order = np.lexsort((c[:, 3], c[:, 2], c[:, 1], c[:, 0]))
    assert not np.array_equal(order, np.arange(len(c)))              # no spatial order for free


def test_lidar_scene_headline_workload():
    c = gen.lidar_scene(2000)
    _common(c)
    assert 95_000 <= len(c) <= 105_000
    assert 3.0 <= _neighbours_per_voxel(c) <= 10.0                   # "4-10 neighbours" incl. the centre
    assert np.array_equal(c, gen.lidar_scene(2000))                  # seeded
    assert not np.array_equal(c, gen.lidar_scene(2001))
    assert c[:, 3].max() < 0.1 * c[:, 1].max()                       # a scan is flat: metres high, tens of metres wide


def test_detection_scene_is_denser_per_voxel():
    c = gen.detection_scene(6000)
    _common(c)
    assert 60_000 <= len(c) <= 100_000
    assert _neighbours_per_voxel(c) > _neighbours_per_voxel(gen.lidar_scene(2000, target_n=30_000))


def test_room_scene_is_planar_and_dense():
    c = gen.room_scene(4000, target_n=60_000)
    _common(c)
    assert abs(len(c) - 60_000) <= 0.02 * 60_000
    assert 8.0 <= _neighbours_per_voxel(c) <= 10.0                   # a plane has 9 of the 27 neighbours


def test_lidar_batch_keeps_samples_apart():
    c = gen.lidar_batch(3000, 2, target_n=20_000)
    _common(c, batches=2)
    km = oc.build_kmap(c, 3, 1)
    src = km.M[km.M >= 0]
    rows = np.repeat(np.arange(len(c)), (km.M >= 0).sum(axis=1))
    assert (c[src, 0] == c[rows, 0]).all()                           # no pair crosses a batch boundary


@pytest.mark.parametrize("dtype,eps", [("f16", 2.0 ** -11), ("bf16", 2.0 ** -8), ("f32", 0.0)])
def test_features_and_weights_are_exact_in_their_dtype(dtype, eps):
    x32, raw = gen.features(500, 16, dtype, 7)
    w32, wraw = gen.weights(27, 16, 8, dtype, 8)
    assert x32.dtype == np.float32 and x32.shape == (500, 16) and w32.shape == (27, 16, 8)
    assert abs(float(x32.std()) - 1.0) < 0.1
    assert abs(float(w32.std()) - 1.0 / np.sqrt(27 * 16)) < 0.2 / np.sqrt(27 * 16)
    again, _ = gen.round_to_dtype(x32, dtype)
    assert np.array_equal(again, x32)                                # already representable: rounding is idempotent


def test_bench_refuses_more_than_one_gpu_and_bad_layer_configs():
    """bench.py runs on one GPU only and says so; argument errors surface before any GPU work."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "no_such_workload"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "invalid choice" in r.stderr
