"""Pins for the CPU oracle: each test checks oracle/sparse_conv.py against
something other than itself (brute force, a closed form, a torch dense
convolution, an adjoint identity, finite differences)."""
import itertools

import numpy as np
import pytest
import torch

from oracle import sparse_conv as oc
from workloads import generators as gen


# ----------------------------------------------------------------- offsets
def test_offsets_order_and_centre():
    offs = oc.offsets(3)
    assert len(offs) == 27
    assert offs[0] == (-1, -1, -1) and offs[26] == (1, 1, 1)
    assert offs[13] == (0, 0, 0)
    assert offs[1] == (-1, -1, 0)          # z fastest
    assert offs[9] == (0, -1, -1)          # x slowest
    for k, (dx, dy, dz) in enumerate(offs):
        assert k == 9 * (dx + 1) + 3 * (dy + 1) + (dz + 1)
    assert oc.offsets(1) == [(0, 0, 0)]
    # even K (the paper defines odd K only): {0..K-1}^3 in the same order
    assert oc.offsets(2) == [(0, 0, 0), (0, 0, 1), (0, 1, 0), (0, 1, 1), (1, 0, 0), (1, 0, 1), (1, 1, 0), (1, 1, 1)]
    with pytest.raises(ValueError):
        oc.offsets(0)


# ------------------------------------------------------ kmap vs brute force
def _brute_kmap(in_pts, out_pts, K, stride):
    """O(N_out * N_in * K^3): test every (output, input) pair against Eq. 1."""
    lo, hi = (-((K - 1) // 2), (K - 1) // 2) if K % 2 else (0, K - 1)
    M = -np.ones((len(out_pts), K ** 3), dtype=np.int64)
    for n, q in enumerate(out_pts):
        for j, p in enumerate(in_pts):
            if p[0] != q[0]:
                continue
            d = [int(p[a]) - stride * int(q[a]) for a in (1, 2, 3)]
            if all(lo <= v <= hi for v in d):
                k = ((d[0] - lo) * K + (d[1] - lo)) * K + (d[2] - lo)
                assert M[n, k] == -1
                M[n, k] = j
    return M


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("lo", [0, -5])
def test_kmap_submanifold_bruteforce(seed, lo):
    c = gen.uniform_cloud(150, 9, seed, lo=lo)
    c[:75, 0] = 1  # two batch samples that must not mix
    km = oc.build_kmap(c, 3, 1)
    assert km.n_in == km.n_out == 150
    np.testing.assert_array_equal(km.out_coords, c)
    np.testing.assert_array_equal(km.M, _brute_kmap(c, c, 3, 1))


@pytest.mark.parametrize("seed", [4, 5])
@pytest.mark.parametrize("stride", [2, 3])
def test_kmap_strided_bruteforce(seed, stride):
    c = gen.uniform_cloud(200, 11, seed, lo=-4)
    km = oc.build_kmap(c, 3, stride)
    # P_out: brute-force floor division, sorted lexicographically, unique
    q = sorted({(int(b), int(np.floor(x / stride)), int(np.floor(y / stride)), int(np.floor(z / stride)))
                for b, x, y, z in c})
    np.testing.assert_array_equal(km.out_coords, np.array(q))
    np.testing.assert_array_equal(km.M, _brute_kmap(c, np.array(q), 3, stride))
    if stride == 2:
        # p -> floor(p/2) always exists and p - 2*floor(p/2) is in {0,1}^3
        assert set(np.unique(km.M[km.M >= 0])) == set(range(200))


@pytest.mark.parametrize("seed", [6, 7])
def test_kmap_transposed_is_transpose_of_strided(seed):
    c = gen.uniform_cloud(220, 10, seed, lo=-3)
    fwd = oc.build_kmap(c, 3, 2)
    tr = oc.build_kmap(c, 3, 2, transposed=True)
    assert tr.n_in == fwd.n_out and tr.n_out == fwd.n_in == 220
    np.testing.assert_array_equal(tr.in_coords, fwd.out_coords)
    pairs_f = {(int(fwd.M[n, k]), n, k) for n in range(fwd.n_out) for k in range(27) if fwd.M[n, k] >= 0}
    pairs_t = {(j, int(tr.M[j, k]), k) for j in range(tr.n_out) for k in range(27) if tr.M[j, k] >= 0}
    assert pairs_f == pairs_t
    assert ((tr.M >= 0).sum(axis=1) <= 8).all()      # K=3, s=2: at most 2^3 parents
    assert ((tr.M >= 0).sum(axis=1) >= 1).all()


def test_kmap_symmetry_and_centre():
    c = gen.uniform_cloud(400, 10, 11)
    km = oc.build_kmap(c, 3, 1)
    M = km.M
    np.testing.assert_array_equal(M[:, 13], np.arange(400))
    for n in range(400):
        for k in range(27):
            j = M[n, k]
            if j >= 0:
                assert M[j, 26 - k] == n
    m = oc.bitmask(M)
    assert ((m >> 13) & 1).all()
    assert sum(bin(int(v)).count("1") for v in m) == (M >= 0).sum()


def test_duplicates_raise():
    c = gen.uniform_cloud(10, 4, 0)
    c[3] = c[7]
    with pytest.raises(ValueError):
        oc.build_kmap(c, 3, 1)


# --------------------------------------------------------------- forward
def test_forward_k1_is_linear_layer():
    rng = np.random.default_rng(0)
    c = gen.uniform_cloud(300, 8, 3)
    X = rng.standard_normal((300, 12))
    W = rng.standard_normal((1, 12, 7))
    km = oc.build_kmap(c, 1, 1)
    np.testing.assert_array_equal(km.M[:, 0], np.arange(300))
    np.testing.assert_allclose(oc.forward(X, W, km.M), X @ W[0], rtol=1e-13, atol=1e-13)


def _dense_from_sparse(coords, X, B, G):
    C = X.shape[1]
    d = torch.zeros(B, C, G, G, G, dtype=torch.float64)
    for (b, x, y, z), row in zip(coords, X):
        d[b, :, x, y, z] = torch.from_numpy(row)
    return d


def _torch_weight(W, K):
    """w[co, ci, dx+r, dy+r, dz+r] = W[k(dx,dy,dz)][ci, co]."""
    V, ci, co = W.shape
    return torch.from_numpy(W).reshape(K, K, K, ci, co).permute(4, 3, 0, 1, 2).contiguous()


@pytest.mark.parametrize("G,B", [(6, 2), (7, 1)])
def test_forward_full_grid_is_dense_conv3d(G, B):
    rng = np.random.default_rng(G)
    c = gen.full_grid(G, B, seed=5)
    X = rng.standard_normal((len(c), 5))
    W = rng.standard_normal((27, 5, 4))
    km = oc.build_kmap(c, 3, 1)
    Y = oc.forward(X, W, km.M)
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, B, G), _torch_weight(W, 3), padding=1)
    for (b, x, y, z), row in zip(c, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)


def test_forward_sparse_equals_dense_conv_at_occupied_sites():
    """Submanifold conv on a sparse set == dense conv of the zero-filled grid,
    read at the occupied sites (absent neighbours contribute nothing)."""
    rng = np.random.default_rng(9)
    G = 9
    c = gen.uniform_cloud(200, G, 21)
    X = rng.standard_normal((200, 3))
    W = rng.standard_normal((27, 3, 6))
    Y = oc.forward(X, W, oc.build_kmap(c, 3, 1).M)
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, 1, G), _torch_weight(W, 3), padding=1)
    for (b, x, y, z), row in zip(c, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)


def test_strided_forward_full_even_grid_is_strided_conv3d():
    rng = np.random.default_rng(3)
    G, B = 8, 2
    c = gen.full_grid(G, B, seed=1)
    X = rng.standard_normal((len(c), 4))
    W = rng.standard_normal((27, 4, 3))
    km = oc.build_kmap(c, 3, 2)
    assert km.n_out == B * (G // 2) ** 3
    Y = oc.forward(X, W, km.M)
    # out[q] reads in[2q + delta], delta in {-1,0,1}: conv3d(stride 2, padding 1) at index q
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, B, G), _torch_weight(W, 3), stride=2, padding=1)
    for (b, x, y, z), row in zip(km.out_coords, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)


def test_even_kernel_stride2_is_conv3d_kernel2_and_partitions_the_inputs():
    """K = s = 2: out[q] reads in[2q + delta], delta in {0,1}^3 = conv3d(kernel 2, stride 2, no
    padding); on any cloud every input row appears in exactly one map entry."""
    rng = np.random.default_rng(12)
    G, B = 6, 2
    c = gen.full_grid(G, B, seed=5)
    X = rng.standard_normal((len(c), 3))
    W = rng.standard_normal((8, 3, 4))
    km = oc.build_kmap(c, 2, 2)
    assert km.M.shape == (B * (G // 2) ** 3, 8)
    Y = oc.forward(X, W, km.M)
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, B, G), _torch_weight(W, 2), stride=2)
    for (b, x, y, z), row in zip(km.out_coords, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)
    cloud = gen.uniform_cloud(500, 12, seed=8, lo=-5)
    ks = oc.build_kmap(cloud, 2, 2)
    hit = np.sort(ks.M[ks.M >= 0])
    np.testing.assert_array_equal(hit, np.arange(len(cloud)))
    np.testing.assert_array_equal(ks.M, _brute_kmap(cloud, ks.out_coords, 2, 2))
    # transposed: the adjoint structure = conv_transpose3d(kernel 2, stride 2)
    fine = gen.full_grid(G, 1, seed=6)
    kt = oc.build_kmap(fine, 2, 2, transposed=True)
    Xq = rng.standard_normal((kt.n_in, 2))
    Wt = rng.standard_normal((8, 2, 3))
    Yt = oc.forward(Xq, Wt, kt.M)
    wt = torch.from_numpy(Wt).reshape(2, 2, 2, 2, 3).permute(3, 4, 0, 1, 2).contiguous()
    reft = torch.nn.functional.conv_transpose3d(_dense_from_sparse(kt.in_coords, Xq, 1, G // 2), wt, stride=2)
    for (b, x, y, z), row in zip(fine, Yt):
        np.testing.assert_allclose(row, reft[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)


def test_transposed_forward_full_grid_is_conv_transpose3d():
    rng = np.random.default_rng(4)
    G, B = 8, 1
    fine = gen.full_grid(G, B, seed=2)
    km = oc.build_kmap(fine, 3, 2, transposed=True)
    assert km.n_in == (G // 2) ** 3
    Xq = rng.standard_normal((km.n_in, 3))
    W = rng.standard_normal((27, 3, 5))
    Y = oc.forward(Xq, W, km.M)
    dense_q = _dense_from_sparse(km.in_coords, Xq, B, G // 2)
    # y[p] = sum_{q,delta: p = 2q + delta} x[q] W[delta]; conv_transpose3d writes
    # out[2q - padding + kidx] += x[q] w[ci, co, kidx], so kidx = delta + 1 with padding 1,
    # and output_padding 1 restores the even size G.
    wt = torch.from_numpy(W).reshape(3, 3, 3, 3, 5).permute(3, 4, 0, 1, 2).contiguous()
    ref = torch.nn.functional.conv_transpose3d(dense_q, wt, stride=2, padding=1, output_padding=1)
    assert ref.shape[-1] == G
    for (b, x, y, z), row in zip(fine, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)


def test_forward_permutation_equivariance_and_linearity():
    rng = np.random.default_rng(12)
    c = gen.uniform_cloud(150, 7, 8)
    X = rng.standard_normal((150, 4))
    X2 = rng.standard_normal((150, 4))
    W = rng.standard_normal((27, 4, 4))
    Y = oc.forward(X, W, oc.build_kmap(c, 3, 1).M)
    perm = rng.permutation(150)
    Yp = oc.forward(X[perm], W, oc.build_kmap(c[perm], 3, 1).M)
    np.testing.assert_allclose(Yp, Y[perm], rtol=1e-12, atol=1e-12)
    M = oc.build_kmap(c, 3, 1).M
    np.testing.assert_allclose(oc.forward(2 * X - 3 * X2, W, M),
                               2 * Y - 3 * oc.forward(X2, W, M), rtol=1e-11, atol=1e-11)


# ------------------------------------------------------------ gradients
@pytest.mark.parametrize("stride,transposed", [(1, False), (2, False), (2, True)])
def test_adjoint_identities(stride, transposed):
    rng = np.random.default_rng(5)
    c = gen.uniform_cloud(180, 8, 13, lo=-2)
    km = oc.build_kmap(c, 3, stride, transposed)
    X = rng.standard_normal((km.n_in, 6))
    W = rng.standard_normal((27, 6, 5))
    G = rng.standard_normal((km.n_out, 5))
    lhs = (oc.forward(X, W, km.M) * G).sum()
    np.testing.assert_allclose((X * oc.dgrad(G, W, km.M, km.n_in)).sum(), lhs, rtol=1e-12)
    np.testing.assert_allclose((W * oc.wgrad(X, G, km.M)).sum(), lhs, rtol=1e-12)


def test_gradients_finite_differences():
    rng = np.random.default_rng(6)
    c = gen.uniform_cloud(20, 3, 2)   # 20 of 27 cells: plenty of neighbours
    km = oc.build_kmap(c, 3, 1)
    X = rng.standard_normal((20, 3))
    W = rng.standard_normal((27, 3, 2))
    G = rng.standard_normal((20, 2))
    loss = lambda X_, W_: (oc.forward(X_, W_, km.M) * G).sum()
    dX, dW = oc.dgrad(G, W, km.M, 20), oc.wgrad(X, G, km.M)
    h = 1e-6
    for idx in [(0, 0), (7, 2), (19, 1)]:
        E = np.zeros_like(X); E[idx] = h
        np.testing.assert_allclose((loss(X + E, W) - loss(X - E, W)) / (2 * h), dX[idx], rtol=1e-7, atol=1e-8)
    for idx in [(0, 0, 0), (13, 2, 1), (26, 1, 0), (5, 0, 1)]:
        E = np.zeros_like(W); E[idx] = h
        np.testing.assert_allclose((loss(X, W + E) - loss(X, W - E)) / (2 * h), dW[idx], rtol=1e-7, atol=1e-8)


def test_gradients_match_torch_autograd_on_full_grid():
    rng = np.random.default_rng(7)
    G_, B = 5, 1
    c = gen.full_grid(G_, B, seed=3)
    X = rng.standard_normal((len(c), 3))
    W = rng.standard_normal((27, 3, 4))
    Gy = rng.standard_normal((len(c), 4))
    km = oc.build_kmap(c, 3, 1)
    xd = _dense_from_sparse(c, X, B, G_).requires_grad_(True)
    wt = _torch_weight(W, 3).requires_grad_(True)
    gd = _dense_from_sparse(c, Gy, B, G_)
    (torch.nn.functional.conv3d(xd, wt, padding=1) * gd).sum().backward()
    dX = oc.dgrad(Gy, W, km.M, km.n_in)
    dW = oc.wgrad(X, Gy, km.M)
    for (b, x, y, z), row in zip(c, dX):
        np.testing.assert_allclose(row, xd.grad[b, :, x, y, z].numpy(), rtol=1e-11, atol=1e-11)
    # wt.grad[co, ci, kx, ky, kz] -> [k, ci, co]
    np.testing.assert_allclose(dW, wt.grad.permute(2, 3, 4, 1, 0).reshape(27, 3, 4).numpy(),
                               rtol=1e-11, atol=1e-11)


# --------------------------------------------------- bitmask / redundancy
def test_bitmask_bits():
    M = np.array([[-1, 3, -1], [0, -1, 2], [-1, -1, -1]])
    np.testing.assert_array_equal(oc.bitmask(M), np.array([2, 5, 0], dtype=np.uint32))


def test_split_ranges_cover():
    for s in range(0, 6):
        r = oc.split_ranges(27, s)
        assert r[0][0] == 0 and r[-1][1] == 27
        assert all(a[1] == b[0] for a, b in zip(r, r[1:]))
    assert oc.split_ranges(27, 2) == [(0, 13), (13, 27)]
    assert oc.split_ranges(27, 3) == [(0, 9), (9, 18), (18, 27)]


def _brute_redundancy(M, tile, n_split):
    """Lock-step model written as explicit loops over groups, rows and offsets."""
    n, V = M.shape
    if n_split == 0:
        parts = [(0, V, list(range(n)))]
    else:
        parts = []
        for i in range(n_split):
            lo, hi = (i * V) // n_split, ((i + 1) * V) // n_split
            keys = []
            for r in range(n):
                v = 0
                for k in range(lo, hi):
                    if M[r, k] >= 0:
                        v += 1 << (k - lo)
                keys.append((v, r))
            parts.append((lo, hi, [r for _, r in sorted(keys)]))
    executed = 0
    for lo, hi, order in parts:
        for t in range(0, n, tile):
            rows = order[t:t + tile]
            for k in range(lo, hi):
                if any(M[r, k] >= 0 for r in rows):
                    executed += len(rows)
    return executed, int((M >= 0).sum())


@pytest.mark.parametrize("n_split", [0, 1, 2, 3])
def test_redundancy_brute(n_split):
    M = oc.build_kmap(gen.uniform_cloud(90, 6, 17), 3, 1).M
    assert oc.redundancy(M, 4, n_split) == _brute_redundancy(M, 4, n_split)


def test_redundancy_limits():
    M = oc.build_kmap(gen.uniform_cloud(64, 5, 3), 3, 1).M
    ex, eff = oc.redundancy(M, 1, 0)
    assert ex == eff                       # one row per group: nothing is wasted
    ex_all, _ = oc.redundancy(M, 64, 0)
    assert ex_all == 64 * (M >= 0).any(axis=0).sum()


# ------------------------------------------- K = 5 and dilated output sets
def test_offsets_k5():
    offs = oc.offsets(5)
    assert len(offs) == 125 and offs[0] == (-2, -2, -2) and offs[62] == (0, 0, 0) and offs[124] == (2, 2, 2)
    for k, (dx, dy, dz) in enumerate(offs):
        assert k == 25 * (dx + 2) + 5 * (dy + 2) + (dz + 2)


@pytest.mark.parametrize("seed", [6, 7])
def test_kmap_k5_bruteforce_and_symmetry(seed):
    c = gen.uniform_cloud(120, 8, seed, lo=-3)
    km = oc.build_kmap(c, 5, 1)
    np.testing.assert_array_equal(km.M, _brute_kmap(c, c, 5, 1))
    for n in range(km.n_out):
        assert km.M[n, 62] == n
        for k in range(125):
            if km.M[n, k] >= 0:
                assert km.M[km.M[n, k], 124 - k] == n


def test_forward_k5_full_grid_is_dense_conv3d_kernel5():
    """Pins the offset order and sign of K = 5 jointly, as conv3d(padding=1) does for K = 3."""
    rng = np.random.default_rng(55)
    G, B = 6, 2
    c = gen.full_grid(G, B, seed=8)
    X = rng.standard_normal((len(c), 3))
    W = rng.standard_normal((125, 3, 4))
    km = oc.build_kmap(c, 5, 1)
    Y = oc.forward(X, W, km.M)
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, B, G), _torch_weight(W, 5), padding=2)
    for (b, x, y, z), row in zip(c, Y):
        np.testing.assert_allclose(row, ref[b, :, x, y, z].numpy(), rtol=1e-12, atol=1e-12)
    # and its gradients through the adjoint identity
    G_out = rng.standard_normal(Y.shape)
    lhs = float((Y * G_out).sum())
    np.testing.assert_allclose(lhs, float((X * oc.dgrad(G_out, W, km.M, km.n_in)).sum()), rtol=1e-12)
    np.testing.assert_allclose(lhs, float((W * oc.wgrad(X, G_out, km.M)).sum()), rtol=1e-12)


def test_wide_bitmask_and_redundancy_beyond_32_offsets():
    M = oc.build_kmap(gen.uniform_cloud(70, 6, 19), 5, 1).M
    m = oc.bitmask(M)
    assert m.dtype == object
    for n in (0, 13, 69):
        assert [k for k in range(125) if (int(m[n]) >> k) & 1] == np.nonzero(M[n] >= 0)[0].tolist()
    for n_split in (0, 1, 3, 4):
        assert oc.redundancy(M, 4, n_split) == _brute_redundancy(M, 4, n_split)


def _brute_dilated(c, K):
    """Every lattice point of the bounding box (grown by the kernel radius) that has an input in
    its neighbourhood, by exhaustive search, in lexicographic order."""
    r = (K - 1) // 2
    pts = {tuple(int(v) for v in p) for p in c}
    lo, hi = c[:, 1:].min(0) - r, c[:, 1:].max(0) + r
    out = []
    for b in sorted(set(int(v) for v in c[:, 0])):
        for x, y, z in itertools.product(*(range(int(l), int(h) + 1) for l, h in zip(lo, hi))):
            if any((b, x + dx, y + dy, z + dz) in pts for dx, dy, dz in itertools.product(range(-r, r + 1), repeat=3)):
                out.append((b, x, y, z))
    return np.asarray(out, dtype=np.int64)


@pytest.mark.parametrize("seed,lo", [(31, 0), (32, -4)])
def test_dilated_output_set_bruteforce(seed, lo):
    c = gen.uniform_cloud(60, 7, seed, lo=lo)
    c[:20, 0] = 1
    km = oc.build_kmap(c, 3, 1, dilate=True)
    want = _brute_dilated(c, 3)
    np.testing.assert_array_equal(km.out_coords, want)
    np.testing.assert_array_equal(km.M, _brute_kmap(c, want, 3, 1))
    assert (km.M >= 0).any(axis=1).all()                 # no output without a neighbour (minimal)
    assert km.n_out > km.n_in and km.n_in == 60
    # every input is the centre neighbour of the output at its own coordinate
    where = {tuple(q): n for n, q in enumerate(km.out_coords.tolist())}
    for j, p in enumerate(c.tolist()):
        assert km.M[where[tuple(p)], 13] == j
    with pytest.raises(ValueError):
        oc.build_kmap(c, 3, 2, dilate=True)
    with pytest.raises(ValueError):
        oc.build_kmap(c, 3, 1, transposed=True, dilate=True)


def test_dilated_forward_is_dense_conv3d_and_zero_elsewhere():
    """A sparse cloud in a zero-filled grid: conv3d(padding=1) of the dense grid equals the
    dilated sparse convolution on the dilated set and is exactly zero everywhere else (so the set
    is complete); gradients through the adjoint identities."""
    rng = np.random.default_rng(77)
    G = 9
    c = gen.uniform_cloud(40, G - 2, 41) + np.array([0, 1, 1, 1])     # one cell of margin: the dilated set stays inside
    X = rng.standard_normal((40, 3))
    W = rng.standard_normal((27, 3, 5))
    km = oc.build_kmap(c, 3, 1, dilate=True)
    Y = oc.forward(X, W, km.M)
    ref = torch.nn.functional.conv3d(_dense_from_sparse(c, X, 1, G), _torch_weight(W, 3), padding=1)[0].numpy()
    seen = np.zeros((G, G, G), dtype=bool)
    for (b, x, y, z), row in zip(km.out_coords, Y):
        np.testing.assert_allclose(row, ref[:, x, y, z], rtol=1e-12, atol=1e-12)
        seen[x, y, z] = True
    assert np.abs(ref[:, ~seen]).max() == 0.0
    G_out = rng.standard_normal(Y.shape)
    lhs = float((Y * G_out).sum())
    np.testing.assert_allclose(lhs, float((X * oc.dgrad(G_out, W, km.M, km.n_in)).sum()), rtol=1e-12)
    np.testing.assert_allclose(lhs, float((W * oc.wgrad(X, G_out, km.M)).sum()), rtol=1e-12)
