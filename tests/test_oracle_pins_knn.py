"""Pins of the k-nearest-neighbour distogram oracle (oracle/knn_ref.py; Section 2.5 of the paper):
a loop-only brute force, scipy's k-d tree on random points, closed forms on a straight chain, ties on a
lattice, masks and short chains."""
import numpy as np
from scipy.spatial import cKDTree

from oracle import knn_ref


def _brute(trans, mask, k):
    """Pure-Python loops in float64 with a stable sort: for inputs whose squared distances are exact
    in float32 (small integers) this is the same decision."""
    B, L = trans.shape[:2]
    out = -np.ones((B, L, k), dtype=np.int64)
    for b in range(B):
        for i in range(L):
            if mask is not None and not mask[b, i]:
                continue
            cand = []
            for j in range(L):
                if j == i or (mask is not None and not mask[b, j]):
                    continue
                d2 = sum((float(trans[b, j, a]) - float(trans[b, i, a])) ** 2 for a in range(3))
                cand.append((d2, j))
            cand.sort()
            for s, (_, j) in enumerate(cand[:k]):
                out[b, i, s] = j
    return out


def test_brute_force_on_integer_points_with_ties():
    rng = np.random.default_rng(0)
    trans = rng.integers(-4, 5, size=(2, 23, 3)).astype(np.float32)  # many equal distances
    mask = (rng.random((2, 23)) > 0.2).astype(np.uint8)
    for m in (None, mask):
        idx, d2, bins = knn_ref.knn_distogram(trans, m, 6, 8, 1.0, 8.0)
        assert np.array_equal(idx, _brute(trans, m, 6))
        # the reported squared distances are those of the reported neighbours
        for b in range(2):
            for i in range(23):
                for s in range(6):
                    j = idx[b, i, s]
                    if j >= 0:
                        assert d2[b, i, s] == float(((trans[b, j] - trans[b, i]) ** 2).sum())
                        assert j != i


def test_against_a_kd_tree_on_random_points():
    rng = np.random.default_rng(1)
    trans = (10.0 * rng.standard_normal((1, 400, 3))).astype(np.float32)
    k = 20
    idx, d2, _ = knn_ref.knn_distogram(trans, None, k, 16, 2.0, 22.0)
    dist, nn = cKDTree(trans[0].astype(np.float64)).query(trans[0].astype(np.float64), k=k + 1)
    # (the tree returns the point itself first; distances of random points are distinct, and the float32
    # decision can differ from the float64 one only between neighbours closer than float32 resolution)
    same = idx[0] == nn[:, 1:]
    assert same.mean() > 0.999
    assert np.allclose(np.sqrt(d2[0].astype(np.float64)), dist[:, 1:], rtol=2e-6, atol=0)
    rows, slots = np.nonzero(~same)
    for i, s in zip(rows, slots):
        assert abs(dist[i, 1 + s] - np.sqrt(float(d2[0, i, s]))) <= 2e-6 * dist[i, 1 + s]


def test_straight_chain_closed_form_and_bin_edges():
    # residues on a line with unit spacing: the neighbours of i are i-1, i+1, i-2, i+2, ... (ties by index)
    L, k = 12, 4
    trans = np.zeros((1, L, 3), dtype=np.float32)
    trans[0, :, 1] = np.arange(L)
    idx, d2, bins = knn_ref.knn_distogram(trans, None, k, 5, 1.0, 3.0)  # edges 1.0, 1.5, 2.0, 2.5
    assert list(idx[0, 5]) == [4, 6, 3, 7]
    assert list(d2[0, 5]) == [1.0, 1.0, 4.0, 4.0]
    assert list(idx[0, 0]) == [1, 2, 3, 4]          # chain end: one-sided
    assert list(d2[0, 0]) == [1.0, 4.0, 9.0, 16.0]
    # d = 1 sits on the first edge (counts it), d = 2 on the third, d = 3 and 4 beyond the last
    assert list(bins[0, 0]) == [1, 3, 4, 4]
    # below the first edge: bin 0
    close = np.zeros((1, 2, 3), dtype=np.float32)
    close[0, 1, 0] = 0.5
    assert knn_ref.knn_distogram(close, None, 1, 5, 1.0, 3.0)[2][0, 0, 0] == 0


def test_masks_and_short_chains():
    rng = np.random.default_rng(2)
    trans = rng.standard_normal((1, 9, 3)).astype(np.float32)
    mask = np.array([[1, 1, 0, 1, 0, 0, 1, 1, 0]], dtype=np.uint8)  # five valid residues
    idx, d2, bins = knn_ref.knn_distogram(trans, mask, 6, 4, 0.5, 2.0)
    valid = set(np.nonzero(mask[0])[0])
    for i in range(9):
        if i not in valid:
            assert np.all(idx[0, i] == -1) and np.all(np.isinf(d2[0, i])) and np.all(bins[0, i] == -1)
            continue
        got = [j for j in idx[0, i] if j >= 0]
        assert len(got) == 4 and set(got) == valid - {i}      # every other valid residue, nothing else
        assert list(idx[0, i, 4:]) == [-1, -1] and np.all(np.isinf(d2[0, i, 4:])) and np.all(bins[0, i, 4:] == -1)
        assert np.all(np.diff(d2[0, i, :4]) >= 0)
    # moving a masked residue changes nothing
    moved = trans.copy()
    moved[0, 2] += 100.0
    again = knn_ref.knn_distogram(moved, mask, 6, 4, 0.5, 2.0)
    assert np.array_equal(again[0], idx) and np.array_equal(again[1], d2)


def test_invariance_under_rigid_motion_of_well_separated_points():
    # distances are invariant (Section 2.5 motivates the k-NN form by invariance); on points whose
    # distances are well separated the neighbour lists are too
    rng = np.random.default_rng(3)
    # points at 1, 2, 4, ..., 2048 along a skew line, in shuffled order: all pairwise distances differ by far
    base = (2.0 ** rng.permutation(12))[:, None] * np.array([[1.0, 0.37, 0.11]])
    trans = base[None].astype(np.float32)
    q, _ = np.linalg.qr(rng.standard_normal((3, 3)))
    moved = (trans[0].astype(np.float64) @ q.T + np.array([3.0, -2.0, 5.0])).astype(np.float32)[None]
    a = knn_ref.knn_distogram(trans, None, 5, 6, 1.0, 6.0)
    b = knn_ref.knn_distogram(moved, None, 5, 6, 1.0, 6.0)
    assert np.array_equal(a[0], b[0])
    assert np.allclose(a[1], b[1], rtol=1e-4)
