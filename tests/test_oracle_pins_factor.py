"""Pins of oracle/factor_ref.py (pair pseudo-factors as linear projections of k-nearest-neighbour
features, Sections 2.4 and 2.5 of the paper) against things fixed outside it: a case worked by hand,
a direct sum written with loops, and properties every linear projection of one-hot features has."""
import numpy as np

from oracle import factor_ref as fr


def _random_case(rng, B=2, L=9, k=4, n_bins=5, n_pos=7, n_out=6, empty=0.2):
    idx = rng.integers(0, L, size=(B, L, k))
    idx[rng.random((B, L, k)) < empty] = -1
    bins = rng.integers(0, n_bins, size=(B, L, k))
    bins[idx < 0] = -1
    return idx, bins, rng.standard_normal((k, n_bins, n_out)), rng.standard_normal((k, n_pos, n_out)), rng.standard_normal(n_out)


def test_worked_example():
    # one chain of three residues, two slots, three bins, offsets -1, 0, +1, two outputs; the tables
    # hold distinct powers of ten so that every term of the sum is visible in the result
    idx = np.array([[[1, 2], [0, -1], [1, 0]]])
    bins = np.array([[[0, 2], [1, -1], [2, 2]]])
    e_bin = np.array([[[1, 2], [10, 20], [100, 200]], [[1000, 2000], [1e4, 2e4], [1e5, 2e5]]], dtype=np.float64)
    e_pos = np.array([[[0.1, 0.2], [0.3, 0.4], [0.5, 0.6]], [[0.01, 0.02], [0.03, 0.04], [0.05, 0.06]]])
    bias = np.array([7e6, 8e6])
    z = fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode=1)
    # residue 0: slot 0 -> bin 0, offset +1 (row 2); slot 1 -> bin 2, offset +2 clipped to +1 (row 2)
    assert np.allclose(z[0, 0], [7e6 + 1 + 0.5 + 1e5 + 0.05, 8e6 + 2 + 0.6 + 2e5 + 0.06], rtol=0, atol=1e-9)
    # residue 1: slot 0 -> bin 1, offset -1 (row 0); slot 1 empty
    assert np.allclose(z[0, 1], [7e6 + 10 + 0.1, 8e6 + 20 + 0.2], rtol=0, atol=1e-9)
    # residue 2: slot 0 -> bin 2, offset -1 (row 0); slot 1 -> bin 2, offset -2 clipped to -1 (row 0)
    assert np.allclose(z[0, 2], [7e6 + 100 + 0.1 + 1e5 + 0.01, 8e6 + 200 + 0.2 + 2e5 + 0.02], rtol=0, atol=1e-9)
    # absolute codes: the neighbour's own index selects the row
    za = fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode=0)
    assert np.allclose(za[0, 0], [7e6 + 1 + 0.3 + 1e5 + 0.05, 8e6 + 2 + 0.4 + 2e5 + 0.06], rtol=0, atol=1e-9)


def test_direct_sum_with_loops():
    rng = np.random.default_rng(11)
    for pos_mode in (0, 1):
        idx, bins, e_bin, e_pos, bias = _random_case(rng)
        z = fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode)
        B, L, k = idx.shape
        n_pos = e_pos.shape[1]
        for b in range(B):
            for i in range(L):
                want = bias.copy()
                for s in range(k):
                    j = idx[b, i, s]
                    if j < 0:
                        continue
                    code = min(j, n_pos - 1) if pos_mode == 0 else min(max(j - i, -(n_pos // 2)), n_pos // 2) + n_pos // 2
                    want = want + e_bin[s, bins[b, i, s]] + e_pos[s, code]
                assert np.allclose(z[b, i], want, rtol=0, atol=1e-12), (pos_mode, b, i)


def test_properties_of_a_linear_projection():
    rng = np.random.default_rng(12)
    idx, bins, e_bin, e_pos, bias = _random_case(rng)
    z = fr.factor_project(idx, bins, e_bin, e_pos, bias)
    # no neighbours at all: the bias alone
    none = np.full_like(idx, -1)
    assert np.array_equal(fr.factor_project(none, none, e_bin, e_pos, bias), np.broadcast_to(bias, z.shape))
    # linear in the tables
    e2, p2 = rng.standard_normal(e_bin.shape), rng.standard_normal(e_pos.shape)
    z2 = fr.factor_project(idx, bins, e2, p2, None)
    assert np.allclose(fr.factor_project(idx, bins, e_bin + 2 * e2, e_pos + 2 * p2, bias), z + 2 * z2, atol=1e-12)
    # exchanging two slots together with their tables changes nothing
    perm = [2, 1, 0, 3]
    assert np.allclose(fr.factor_project(idx[..., perm], bins[..., perm], e_bin[perm], e_pos[perm], bias), z, atol=1e-12)
    # without a position table only the bins count
    zb = fr.factor_project(idx, bins, e_bin, None, bias)
    assert np.allclose(zb, fr.factor_project(idx, bins, e_bin, np.zeros_like(e_pos), bias), atol=1e-12)
    # every feature vector has one 1 per filled slot and table, none in an empty slot
    x = fr.features(idx, bins, e_bin.shape[1], e_pos.shape[1], 1)
    assert np.array_equal(x.sum(axis=-1), 2.0 * (idx >= 0))


def test_relative_codes_do_not_see_a_shift_of_the_chain():
    # the same neighbourhood pattern placed 5 residues further along a longer chain
    rng = np.random.default_rng(13)
    idx, bins, e_bin, e_pos, bias = _random_case(rng, B=1, L=8, empty=0.0)
    z = fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode=1)
    big_idx = np.full((1, 13, idx.shape[2]), -1)
    big_bins = np.full_like(big_idx, -1)
    big_idx[0, 5:] = idx[0] + 5
    big_bins[0, 5:] = bins[0]
    zs = fr.factor_project(big_idx, big_bins, e_bin, e_pos, bias, pos_mode=1)
    assert np.allclose(zs[0, 5:], z[0], atol=1e-12)
    assert not np.allclose(fr.factor_project(big_idx, big_bins, e_bin, e_pos, bias, pos_mode=0)[0, 5:],
                           fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode=0)[0])


def test_backward_is_the_adjoint_of_the_projection_and_a_direct_scatter():
    rng = np.random.default_rng(14)
    for pos_mode in (0, 1):
        idx, bins, e_bin, e_pos, bias = _random_case(rng)
        B, L, k = idx.shape
        d_z = rng.standard_normal((B, L, e_bin.shape[2]))
        mask = (rng.random((B, L)) > 0.25).astype(np.uint8)
        g_bin, g_pos, g_bias = fr.factor_project_backward(idx, bins, d_z, e_bin.shape[1], e_pos.shape[1], pos_mode, mask)
        # adjoint identity of a linear map: <d_z, z(E, b)> = <dE, E> + <db, b> (masked residues left out of the loss)
        z = fr.factor_project(idx, bins, e_bin, e_pos, bias, pos_mode)
        lhs = float((z * d_z * mask[:, :, None]).sum())
        rhs = float((g_bin * e_bin).sum() + (g_pos * e_pos).sum() + (g_bias * bias).sum())
        assert abs(lhs - rhs) <= 1e-9 * max(1.0, abs(lhs))
        # direct scatter with loops
        want_bin, want_pos = np.zeros_like(e_bin), np.zeros_like(e_pos)
        n_pos = e_pos.shape[1]
        for b in range(B):
            for i in range(L):
                if not mask[b, i]:
                    continue
                for s in range(k):
                    j = idx[b, i, s]
                    if j < 0:
                        continue
                    code = min(j, n_pos - 1) if pos_mode == 0 else min(max(j - i, -(n_pos // 2)), n_pos // 2) + n_pos // 2
                    want_bin[s, bins[b, i, s]] += d_z[b, i]
                    want_pos[s, code] += d_z[b, i]
        assert np.allclose(g_bin, want_bin, atol=1e-12) and np.allclose(g_pos, want_pos, atol=1e-12)
        assert np.allclose(g_bias, (d_z * mask[:, :, None]).sum(axis=(0, 1)), atol=1e-12)
    # a table row that no residue selects gets no gradient
    idx1 = np.array([[[1], [0]]])
    bins1 = np.array([[[2], [2]]])
    g_bin, g_pos, _ = fr.factor_project_backward(idx1, bins1, np.ones((1, 2, 3)), 4, 0)
    assert g_pos is None and np.array_equal(g_bin[0, 2], [2.0, 2.0, 2.0]) and not g_bin[0, [0, 1, 3]].any()
