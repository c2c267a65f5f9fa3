"""Pair pseudo-factors from k-nearest-neighbour features (Section 2.4 of the paper: every pair
feature is represented by two tensors of shape [B, L, r, c_z] "obtained via linear projections";
Section 2.5: the features are the distogram bins of the k nearest neighbours, whose identities
are kept through a positional encoding of their indices) in plain numpy float64 -- test
infrastructure only.

Readings (the paper names the ingredients and gives no formula):
  * the feature vector of residue i is the concatenation over its k neighbour slots s of
    [one-hot_{n_bins}(bin_is) | one-hot_{n_pos}(pos_is)]; an empty slot (index -1) is all zero;
  * the positional encoding of a neighbour is taken in its general linear form, a one-hot of a
    position code that the projection turns into a learned embedding (a fixed encoding such as
    sines and cosines followed by a linear map is the special case of a particular table):
    pos_mode 0: the code is the neighbour's own index j, clipped to n_pos - 1;
    pos_mode 1: the code is the offset j - i clipped to +-(n_pos - 1)/2, shifted to 0 .. n_pos - 1
    (n_pos odd);
  * a factor is one linear projection of that vector plus a bias: z_i = W x_i + b with
    W of shape [n_out, k (n_bins + n_pos)], n_out = r c_z, given here as the two tables
    e_bin [k, n_bins, n_out] and e_pos [k, n_pos, n_out] of W's columns.
The function below builds x explicitly and multiplies.
"""
import numpy as np


def position_codes(idx, n_pos, pos_mode):
    """idx [B, L, k] neighbour indices (-1 = empty) -> codes [B, L, k] (entries of empty slots are meaningless)."""
    idx = np.asarray(idx, dtype=np.int64)
    if pos_mode == 0:
        return np.minimum(idx, n_pos - 1)
    half = (n_pos - 1) // 2
    i = np.arange(idx.shape[1], dtype=np.int64)[None, :, None]
    return np.clip(idx - i, -half, half) + half


def features(idx, bins, n_bins, n_pos, pos_mode):
    """The explicit feature tensor x [B, L, k, n_bins + n_pos] of zeros and ones."""
    idx = np.asarray(idx, dtype=np.int64)
    bins = np.asarray(bins, dtype=np.int64)
    B, L, k = idx.shape
    x = np.zeros((B, L, k, n_bins + n_pos), dtype=np.float64)
    codes = position_codes(idx, n_pos, pos_mode)
    for b in range(B):
        for i in range(L):
            for s in range(k):
                if idx[b, i, s] < 0:
                    continue
                x[b, i, s, bins[b, i, s]] = 1.0
                if n_pos > 0:
                    x[b, i, s, n_bins + codes[b, i, s]] = 1.0
    return x


def factor_project(idx, bins, e_bin, e_pos, bias, pos_mode=1):
    """idx, bins [B, L, k]; e_bin [k, n_bins, n_out]; e_pos [k, n_pos, n_out] or None; bias [n_out] or
    None -> z [B, L, n_out] float64."""
    e_bin = np.asarray(e_bin, dtype=np.float64)
    k, n_bins, n_out = e_bin.shape
    n_pos = 0 if e_pos is None else np.asarray(e_pos).shape[1]
    x = features(idx, bins, n_bins, n_pos, pos_mode)
    w = e_bin if e_pos is None else np.concatenate([e_bin, np.asarray(e_pos, dtype=np.float64)], axis=1)
    B, L = x.shape[:2]
    z = x.reshape(B, L, k * (n_bins + n_pos)) @ w.reshape(k * (n_bins + n_pos), n_out)
    return z if bias is None else z + np.asarray(bias, dtype=np.float64)


def factor_project_backward(idx, bins, d_z, n_bins, n_pos, pos_mode=1, mask=None):
    """Gradient of a loss through factor_project with respect to its tables and bias, given d_z
    [B, L, n_out] = d loss / d z: the projection is linear, z = x W + b, so d W = x^T d_z and
    d b = sum of d_z over the residues (residues with mask 0 contribute nothing).
    Returns d_e_bin [k, n_bins, n_out], d_e_pos [k, n_pos, n_out] (None when n_pos = 0), d_bias [n_out]."""
    d_z = np.asarray(d_z, dtype=np.float64)
    B, L, n_out = d_z.shape
    k = np.asarray(idx).shape[2]
    if mask is not None:
        d_z = d_z * (np.asarray(mask) != 0)[:, :, None]
    x = features(idx, bins, n_bins, n_pos, pos_mode)
    dw = x.reshape(B * L, k * (n_bins + n_pos)).T @ d_z.reshape(B * L, n_out)
    dw = dw.reshape(k, n_bins + n_pos, n_out)
    return dw[:, :n_bins], (dw[:, n_bins:] if n_pos > 0 else None), d_z.reshape(B * L, n_out).sum(axis=0)
