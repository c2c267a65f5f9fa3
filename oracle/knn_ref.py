"""k-nearest-neighbour distogram features (Section 2.5 of the paper: instead of the full
[L, L, n_bins] distogram only the distances to the k nearest neighbours are kept, [L, k, n_bins],
and the neighbours' identities are kept as indices) in plain numpy -- test infrastructure only.

Readings (the paper gives one paragraph and no formula):
  * the distance between residues i and j is the Euclidean distance of their frame origins t_i, t_j;
  * a residue is not its own neighbour; only valid (unmasked) residues are candidates; an invalid
    residue has no neighbours; when fewer than k candidates exist the remaining slots are empty
    (index -1, squared distance +inf, bin -1);
  * neighbours are listed by increasing distance, equal distances by increasing index;
  * the distogram has n_bins bins with n_bins - 1 edges e_m = d_min + m (d_max - d_min)/(n_bins - 1),
    m = 0 .. n_bins - 2, and bin(d) = number of edges e_m <= d (so bin 0 holds d < d_min and the last
    bin d >= d_max).
Every decision (order, bin) is taken on the squared distance in float32, formed as
((dx*dx + dy*dy) + dz*dz) with dx = x_j - x_i and each operation rounded to float32, and on the
squared edges e_m*e_m with e_m = d_min + m*w, w = (d_max - d_min)/(n_bins - 1), all in float32:
the precision a GPU kernel would use, so that both sides take identical decisions.
"""
import numpy as np


def bin_edges_squared(n_bins, d_min, d_max):
    f = np.float32
    w = f(f(d_max) - f(d_min)) / f(n_bins - 1)
    e = f(d_min) + np.arange(n_bins - 1, dtype=np.float32) * w
    return (e * e).astype(np.float32)


def knn_distogram(trans, mask, k, n_bins, d_min, d_max):
    """trans [B, L, 3] float32, mask [B, L] (0/1) or None ->
    idx [B, L, k] int32, d2 [B, L, k] float32, bins [B, L, k] int32."""
    t = np.ascontiguousarray(trans, dtype=np.float32)
    B, L = t.shape[:2]
    valid = np.ones((B, L), dtype=bool) if mask is None else (np.asarray(mask) != 0)
    e2 = bin_edges_squared(n_bins, d_min, d_max)
    idx = np.full((B, L, k), -1, dtype=np.int32)
    d2o = np.full((B, L, k), np.inf, dtype=np.float32)
    bins = np.full((B, L, k), -1, dtype=np.int32)
    j_all = np.arange(L)
    for b in range(B):
        for i in range(L):
            if not valid[b, i]:
                continue
            dx = t[b, :, 0] - t[b, i, 0]
            dy = t[b, :, 1] - t[b, i, 1]
            dz = t[b, :, 2] - t[b, i, 2]
            d2 = (dx * dx + dy * dy) + dz * dz  # float32 throughout, one rounding per operation
            cand = valid[b] & (j_all != i)
            js = j_all[cand]
            order = np.lexsort((js, d2[cand]))[:k]  # by squared distance, then by index
            n = len(order)
            idx[b, i, :n] = js[order]
            d2o[b, i, :n] = d2[cand][order]
            bins[b, i, :n] = np.searchsorted(e2, d2o[b, i, :n], side="right")
    return idx, d2o, bins
