"""Plain float64 CPU oracle for sparse 3-D convolution.

TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
measured against; it shares no code with it and is never used by the product
path.  Everything here is the *definition* written out (paper Section 2.1,
Equation 1, and the map definitions of Sections 2.2.1 and 3.1), not an
optimised algorithm: a Python dict for the coordinate look-up, Python loops
over output points and offsets for the kernel map, and one float64 matmul per
kernel offset for the features (the gather-GEMM-scatter regrouping of
Equation 1 by offset, Section 2.2.1).

Conventions fixed by this repository where the paper gives only a set or is
silent (each is pinned by a test against a dense torch convolution):

* A point is a row (b, x, y, z) of int coordinates; b is the batch index and
  is never offset or strided.
* Offsets of Delta^3(K) are enumerated with x slowest and z fastest:
  k = ((dx+r)*K + (dy+r))*K + (dz+r), r = (K-1)/2, K odd.
* Equation 1 is taken literally: output q reads the input at s*q + delta with
  W[delta] (cross-correlation, no kernel flip).
* Stride 1: P_out = P_in in input order (submanifold).  Stride s > 1:
  P_out = sorted unique floor(p / s), lexicographic in (b, x, y, z).
* dilate=True (stride-1 convolution whose output set is not the input set, the
  other reading of Equation 1's "q_k in P_out"): P_out = every q that has at
  least one input among its neighbours, { q : exists delta in Delta^3(K) with
  q + delta in P_in }, sorted lexicographically in (b, x, y, z).
* Transposed convolution with stride s: the caller supplies the fine set F
  (the outputs).  The inputs are Q = P_out(F, s) in that sorted order, and
  y_F[j] = sum over (i, delta) with F_j = s*Q_i + delta of x_Q[i] . W[delta].

Pins (tests/test_oracle_*.py): brute-force O(N^2) neighbour search, the
submanifold map symmetry, K=1 == dense linear layer, fully occupied grid ==
torch conv3d / strided conv3d / conv_transpose3d in float64 (K = 3, 5 and 2),
a sparse cloud in a zero-filled dense grid == conv3d read on the dilated set
(and exactly zero off it), adjoint identities, finite differences and
torch.autograd on the dense grid.

Parity unpinned: the paper's worked 2-D example (22 effective MACs; 34 / 26 /
22 redundant MACs for unsorted / sorted / three splits, Sections 2.2.3 and
4.1).  Its point layout is only in a figure that is not available, so
`redundancy` below is pinned by a brute-force count on tiny clouds instead of
by those printed values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def offsets(K: int) -> list[tuple[int, int, int]]:
    """Delta^3(K) (Section 2.1) as a list; position in the list is k.

    The paper defines the neighbourhood for odd K only ({-r..r}^3, r = (K-1)/2).  Reading for
    even K: {0..K-1}^3, so that K = s = 2 tiles space without overlap (every input belongs to
    exactly one output), which is what the 2x2x2 / stride-2 layers of U-Nets compute."""
    if K < 1:
        raise ValueError("K must be positive")
    lo, hi = (-((K - 1) // 2), (K - 1) // 2) if K % 2 else (0, K - 1)
    out = []
    for dx in range(lo, hi + 1):
        for dy in range(lo, hi + 1):
            for dz in range(lo, hi + 1):
                out.append((dx, dy, dz))
    return out


def _as_tuples(coords) -> list[tuple[int, int, int, int]]:
    c = np.asarray(coords)
    if c.ndim != 2 or c.shape[1] != 4:
        raise ValueError("coords must be [N, 4] = (b, x, y, z)")
    return [(int(r[0]), int(r[1]), int(r[2]), int(r[3])) for r in c]


def _table(points) -> dict:
    """coordinate -> row index; duplicates are an error (the paper applies
    Unique to the quantised coordinates before anything else, Section 2)."""
    t = {}
    for j, p in enumerate(points):
        if p in t:
            raise ValueError(f"duplicate coordinate {p} at rows {t[p]} and {j}")
        t[p] = j
    return t


def downsample_coords(coords, stride: int) -> np.ndarray:
    """P_out of a stride-s convolution: sorted unique floor(p / s)."""
    pts = _as_tuples(coords)
    if stride == 1:
        return np.asarray(pts, dtype=np.int64).reshape(-1, 4)
    # Python's // is floor division, also for negative coordinates.
    q = {(b, x // stride, y // stride, z // stride) for (b, x, y, z) in pts}
    return np.asarray(sorted(q), dtype=np.int64).reshape(-1, 4)


@dataclass
class KMap:
    """Output-stationary kernel map M[n_out, K^3] (Section 3.1): M[n, k] is the
    input row that is the k-th neighbour of output n, or -1."""
    M: np.ndarray           # int64 [n_out, K^3]
    n_in: int
    n_out: int
    in_coords: np.ndarray   # int64 [n_in, 4]
    out_coords: np.ndarray  # int64 [n_out, 4]
    K: int
    stride: int
    transposed: bool


def dilated_coords(coords, K: int) -> np.ndarray:
    """P_out of a stride-1 convolution that writes wherever it can read something: every q with
    an input at q + delta for some delta in Delta^3(K), sorted."""
    offs = offsets(K)
    q = {(b, x - dx, y - dy, z - dz) for (b, x, y, z) in _as_tuples(coords) for (dx, dy, dz) in offs}
    return np.asarray(sorted(q), dtype=np.int64).reshape(-1, 4)


def build_kmap(coords, K: int, stride: int = 1, transposed: bool = False, dilate: bool = False) -> KMap:
    """Kernel map of Equation 1.

    transposed=False: coords are P_in; M[n, k] = j with p_j = s*q_n + delta_k.
    transposed=True : coords are the fine output set F; inputs are the coarse
    set Q = downsample_coords(F, s); M[j, k] = i with F_j = s*Q_i + delta_k.
    dilate=True (stride 1, not transposed): P_out = dilated_coords(coords, K).
    """
    if stride < 1:
        raise ValueError("stride must be >= 1")
    if dilate and (stride != 1 or transposed):
        raise ValueError("dilated output sets are defined here for stride 1, not transposed")
    offs = offsets(K)
    pts = _as_tuples(coords)
    _table(pts)  # duplicate check on what the caller handed over
    if not transposed:
        tab = _table(pts)
        out = dilated_coords(coords, K) if dilate else downsample_coords(coords, stride)
        out_pts = _as_tuples(out) if len(out) else []
        M = np.full((len(out_pts), len(offs)), -1, dtype=np.int64)
        for n, (b, x, y, z) in enumerate(out_pts):
            for k, (dx, dy, dz) in enumerate(offs):
                M[n, k] = tab.get((b, stride * x + dx, stride * y + dy, stride * z + dz), -1)
        return KMap(M, len(pts), len(out_pts), np.asarray(pts, dtype=np.int64).reshape(-1, 4),
                    out, K, stride, False)
    # stride 1: Q = F in input order; F_j = Q_i + delta  <=>  Q_i = F_j - delta.
    coarse = downsample_coords(coords, stride)
    coarse_pts = _as_tuples(coarse) if len(coarse) else []
    tab = _table(coarse_pts)
    M = np.full((len(pts), len(offs)), -1, dtype=np.int64)
    for j, (b, x, y, z) in enumerate(pts):
        for k, (dx, dy, dz) in enumerate(offs):
            tx, ty, tz = x - dx, y - dy, z - dz
            if tx % stride or ty % stride or tz % stride:
                continue
            M[j, k] = tab.get((b, tx // stride, ty // stride, tz // stride), -1)
    return KMap(M, len(coarse_pts), len(pts),
                np.asarray(coarse_pts, dtype=np.int64).reshape(-1, 4),
                np.asarray(pts, dtype=np.int64).reshape(-1, 4), K, stride, True)


def forward(X, W, M, n_out: int | None = None) -> np.ndarray:
    """Equation 1 regrouped by offset: Y[rows] += X[M[rows, k]] @ W[k]."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    M = np.asarray(M)
    n_out = M.shape[0] if n_out is None else n_out
    Y = np.zeros((n_out, W.shape[2]), dtype=np.float64)
    for k in range(M.shape[1]):
        rows = np.nonzero(M[:, k] >= 0)[0]
        if rows.size:
            Y[rows] += X[M[rows, k]] @ W[k]
    return Y


def dgrad(dY, W, M, n_in: int) -> np.ndarray:
    """Gradient of Equation 1 w.r.t. the input features:
    dX[M[n, k]] += dY[n] @ W[k]^T for every present pair."""
    dY = np.asarray(dY, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    M = np.asarray(M)
    dX = np.zeros((n_in, W.shape[1]), dtype=np.float64)
    for k in range(M.shape[1]):
        rows = np.nonzero(M[:, k] >= 0)[0]
        if rows.size:
            # np.add.at: correct even if an input row occurred twice for one k
            np.add.at(dX, M[rows, k], dY[rows] @ W[k].T)
    return dX


def wgrad(X, dY, M) -> np.ndarray:
    """Gradient of Equation 1 w.r.t. the weights:
    dW[k] = X[M[rows, k]]^T @ dY[rows]."""
    X = np.asarray(X, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    M = np.asarray(M)
    dW = np.zeros((M.shape[1], X.shape[1], dY.shape[1]), dtype=np.float64)
    for k in range(M.shape[1]):
        rows = np.nonzero(M[:, k] >= 0)[0]
        if rows.size:
            dW[k] = X[M[rows, k]].T @ dY[rows]
    return dW


def bitmask(M) -> np.ndarray:
    """Neighbour bitmask of Section 2.2.3: bit k of mask[n] is set iff the
    k-th neighbour of output n is present.  uint32 up to 32 offsets; beyond (K = 5 has 125), an
    object array of Python integers, which have no width."""
    M = np.asarray(M)
    if M.shape[1] > 32:
        m = np.zeros(M.shape[0], dtype=object)
        for n in range(M.shape[0]):
            m[n] = sum(1 << k for k in np.nonzero(M[n] >= 0)[0].tolist())
        return m
    m = np.zeros(M.shape[0], dtype=np.uint64)
    for k in range(M.shape[1]):
        m |= (M[:, k] >= 0).astype(np.uint64) << np.uint64(k)
    return m.astype(np.uint32)


def split_ranges(V: int, s: int) -> list[tuple[int, int]]:
    """Partition of the V offsets into s contiguous parts (Section 4.1 splits the
    sequential loop over offsets into s parts); s <= 1 is a single part."""
    s = max(1, s)
    return [((i * V) // s, ((i + 1) * V) // s) for i in range(s)]


def redundancy(M, tile_rows: int, n_split: int):
    """Executed and effective MAC units (in units of C_in*C_out MACs) of the
    implicit-GEMM dataflow under the lock-step model of Section 2.2.3: rows are
    processed in groups of `tile_rows`; a group pays for offset k for all of
    its rows whenever any of its rows has neighbour k.

    n_split = 0: rows in their given order, one pass (unsorted).
    n_split >= 1: the offsets are cut into n_split contiguous ranges; in each
    range the rows are sorted by the numeric value of that range's bits of the
    bitmask (Sections 2.2.3 and 4.1), ascending, ties in original order.
    Returns (executed, effective); redundant = executed - effective.
    """
    M = np.asarray(M)
    n, V = M.shape
    present = M >= 0
    effective = int(present.sum())
    executed = 0
    if n_split == 0:
        parts = [(0, V, np.arange(n))]
    else:
        mask = [int(v) for v in bitmask(M)]     # Python integers: any width
        parts = []
        for lo, hi in split_ranges(V, n_split):
            key = [(v >> lo) & ((1 << (hi - lo)) - 1) for v in mask]
            # ascending by the number the bits spell, ties in original order
            parts.append((lo, hi, np.asarray(sorted(range(n), key=key.__getitem__), dtype=np.int64)))
    for lo, hi, order in parts:
        for t in range(0, n, tile_rows):
            rows = order[t:t + tile_rows]
            active = present[rows, lo:hi].any(axis=0)
            executed += int(active.sum()) * len(rows)
    return executed, effective
