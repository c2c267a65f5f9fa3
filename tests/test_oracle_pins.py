"""Pins of the CPU oracle to things other than itself (no GPU needed).

The oracle is standard IPA (paper Eqs. 2-4) in float64.  It is checked against
  * a loop-only evaluation of Eqs. 2-4 on tiny inputs with an arbitrary dense z,
  * the factorized update rule (Algorithm 1) on rank-r pair tensors (Section 2.4's
    equivalence claim),
  * SE(3) invariance (Section 3.1),
  * closed forms and special cases (one residue, two residues, identical keys,
    gamma = 0 and w_b = 0 -> library softmax attention, constant pair tensor),
  * mask semantics, the row-subset form, and
  * central finite differences of the forward for every gradient of the backward.
"""
import math

import numpy as np
import pytest
import torch

from oracle import factorized_ref, ipa_oracle
from paper_2505_11580_amd import workloads as wl


def small(seed=0, B=1, L=6, H=2, c=3, Pq=2, Pv=3, cz=4, r=2, dense=False, mask=None):
    rng = np.random.default_rng(seed)
    inp = dict(
        q=rng.standard_normal((B, L, H, c)), k=rng.standard_normal((B, L, H, c)),
        v=rng.standard_normal((B, L, H, c)),
        q_pts=rng.standard_normal((B, L, H, Pq, 3)), k_pts=rng.standard_normal((B, L, H, Pq, 3)),
        v_pts=rng.standard_normal((B, L, H, Pv, 3)),
        rot=wl.random_rotations(rng, (B, L)), trans=2.0 * rng.standard_normal((B, L, 3)),
        w_b=rng.standard_normal((H, cz)) / math.sqrt(cz),
        gamma=np.log1p(np.exp(rng.standard_normal(H))),
        w_L=math.sqrt(1 / 3), w_C=math.sqrt(2 / (9 * Pq)), mask=mask)
    if dense:
        inp["z"] = rng.standard_normal((B, L, L, cz))
    else:
        inp["z1"] = rng.standard_normal((B, L, r, cz))
        inp["z2"] = rng.standard_normal((B, L, r, cz))
    return inp


def brute_force(inp):
    """Eqs. 2-4 with Python loops over every index; dense z."""
    B, L, H, c = inp["q"].shape
    Pq, Pv, cz = inp["q_pts"].shape[3], inp["v_pts"].shape[3], inp["w_b"].shape[1]
    o = np.zeros((B, L, H, c)); o_pts = np.zeros((B, L, H, Pv, 3)); o_pair = np.zeros((B, L, H, cz))
    attn = np.zeros((B, L, H, L))
    for b in range(B):
        R, t = inp["rot"][b], inp["trans"][b]
        for h in range(H):
            for i in range(L):
                s = []
                for j in range(L):
                    qk = sum(inp["q"][b, i, h, d] * inp["k"][b, j, h, d] for d in range(c))
                    bias = sum(inp["w_b"][h, d] * inp["z"][b, i, j, d] for d in range(cz))
                    dist = 0.0
                    for p in range(Pq):
                        Qg = R[i] @ inp["q_pts"][b, i, h, p] + t[i]
                        Kg = R[j] @ inp["k_pts"][b, j, h, p] + t[j]
                        dist += float(np.sum((Qg - Kg) ** 2))
                    s.append(inp["w_L"] * (qk / math.sqrt(c) + bias
                                           - inp["gamma"][h] * inp["w_C"] / 2 * dist))
                e = [math.exp(x - max(s)) for x in s]
                a = [x / sum(e) for x in e]
                attn[b, i, h] = a
                for j in range(L):
                    o[b, i, h] += a[j] * inp["v"][b, j, h]
                    o_pair[b, i, h] += a[j] * inp["z"][b, i, j]
                for p in range(Pv):
                    G = sum(a[j] * (R[j] @ inp["v_pts"][b, j, h, p] + t[j]) for j in range(L))
                    o_pts[b, i, h, p] = R[i].T @ (G - t[i])
    return dict(o=o, o_pts=o_pts, o_pair=o_pair, attn=attn)


def assert_close(got, want, tol, names=("o", "o_pts", "o_pair")):
    for n in names:
        scale = max(np.abs(want[n]).max(), 1e-30)
        err = np.abs(got[n] - want[n]).max() / scale
        assert err <= tol, (n, err)


def test_brute_force_dense_z():
    for seed in (1, 2):
        inp = small(seed=seed, B=2, L=5, dense=True)
        assert_close(ipa_oracle.forward(inp, want_attn=True), brute_force(inp), 1e-12,
                     ("o", "o_pts", "o_pair", "attn"))


def test_equals_factorized_update_rule_on_rank_r():
    # Section 2.4: with z_ij = z1_i^T z2_j the lifted attention is an equivalent update rule
    inp = wl.make_inputs(0)
    got = ipa_oracle.forward(inp, want_attn=True)
    ref = factorized_ref.forward(inp)
    assert_close(got, ref, 1e-9, ("o", "o_pts", "o_pair", "attn"))
    for seed, r in ((3, 1), (4, 3)):
        inp = small(seed=seed, B=2, L=8, r=r)
        assert_close(ipa_oracle.forward(inp, want_attn=True), factorized_ref.forward(inp), 1e-11,
                     ("o", "o_pts", "o_pair", "attn"))


def test_factorized_with_mask():
    mask = np.array([[1, 1, 0, 1, 1, 0, 0, 1]], dtype=np.uint8)
    inp = small(seed=5, L=8, mask=mask)
    assert_close(ipa_oracle.forward(inp), factorized_ref.forward(inp), 1e-11)


def global_move(inp, seed):
    rng = np.random.default_rng(seed)
    Rg = wl.random_rotations(rng, ())
    tg = 50.0 * rng.standard_normal(3)
    out = dict(inp)
    out["rot"] = np.einsum("xy,blyz->blxz", Rg, inp["rot"])
    out["trans"] = np.einsum("xy,bly->blx", Rg, inp["trans"]) + tg
    return out


def test_se3_invariance():
    # Section 3.1: outputs do not change under a global rotation + translation of all frames
    inp = wl.make_inputs(0, L=32)
    base = ipa_oracle.forward(inp)
    moved = ipa_oracle.forward(global_move(inp, 7))
    assert_close(moved, base, 1e-10)
    # ... and do change when a single frame moves
    one = dict(inp)
    one["trans"] = inp["trans"].copy()
    one["trans"][0, 3] += 1.0
    changed = ipa_oracle.forward(one)
    assert np.abs(changed["o_pts"] - base["o_pts"]).max() > 1e-3


def test_reduces_to_library_softmax_attention():
    # gamma = 0 and w_b = 0 leave softmax(w_L q.k / sqrt(c)) v
    inp = small(seed=8, B=2, L=7, H=3, c=5)
    inp["gamma"] = np.zeros(3)
    inp["w_b"] = np.zeros_like(inp["w_b"])
    got = ipa_oracle.forward(inp)
    tq, tk, tv = (torch.from_numpy(inp[n]).permute(0, 2, 1, 3) for n in ("q", "k", "v"))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, scale=inp["w_L"] / math.sqrt(5)).permute(0, 2, 1, 3).numpy()
    assert np.abs(got["o"] - ref).max() <= 1e-12


def test_single_residue_is_identity():
    inp = small(seed=9, L=1, dense=True)
    got = ipa_oracle.forward(inp)
    assert np.allclose(got["o"], inp["v"], atol=1e-14)
    assert np.allclose(got["o_pts"], inp["v_pts"], atol=1e-13)
    assert np.allclose(got["o_pair"][0, 0], np.broadcast_to(inp["z"][0, 0, 0], got["o_pair"][0, 0].shape),
                       atol=1e-14)


def test_two_residue_closed_form():
    # zero scalars and bias: a_12 / a_11 = exp(-gamma w_L w_C / 2 * (D_12 - D_11))
    inp = small(seed=10, L=2, H=1, Pq=1)
    inp["q"][:] = 0; inp["w_b"][:] = 0
    a = ipa_oracle.forward(inp, want_attn=True)["attn"][0, 0, 0]
    R, t = inp["rot"][0], inp["trans"][0]
    Q1 = R[0] @ inp["q_pts"][0, 0, 0, 0] + t[0]
    K = [R[j] @ inp["k_pts"][0, j, 0, 0] + t[j] for j in range(2)]
    d11, d12 = np.sum((Q1 - K[0]) ** 2), np.sum((Q1 - K[1]) ** 2)
    want = math.exp(-inp["gamma"][0] * inp["w_L"] * inp["w_C"] / 2 * (d12 - d11))
    assert abs(a[1] / a[0] - want) <= 1e-12 * want
    # the printed constants for N_query = 4 (w_L = sqrt(1/3), w_C = sqrt(2/(9*4)))
    assert abs(math.sqrt(1 / 3) * math.sqrt(2 / 36) / 2 - 0.0680414) < 1e-6


def test_identical_keys_give_uniform_weights():
    inp = small(seed=11, L=6)
    for n in ("k", "k_pts", "z2"):
        inp[n][:] = inp[n][:, :1]
    inp["rot"][:] = inp["rot"][:, :1]
    inp["trans"][:] = inp["trans"][:, :1]
    got = ipa_oracle.forward(inp, want_attn=True)
    assert np.allclose(got["attn"], 1 / 6, atol=1e-13)
    assert np.allclose(got["o"], inp["v"].mean(axis=1, keepdims=True), atol=1e-13)


def test_convex_combination_invariants():
    inp = small(seed=12, B=2, L=7)
    inp["v_pts"][:] = 0
    got = ipa_oracle.forward(inp, want_attn=True)
    assert np.allclose(got["attn"].sum(-1), 1.0, atol=1e-13)
    # zero local value points: o_pts = R_i^T (sum_j a_ij t_j - t_i)
    centre = np.einsum("bihj,bjx->bihx", got["attn"], inp["trans"]) - inp["trans"][:, :, None, :]
    want = np.einsum("biyx,bihy->bihx", inp["rot"], centre)
    assert np.allclose(got["o_pts"], want[:, :, :, None, :], atol=1e-12)
    # rank-1 all-ones factors: z_ij = 1, bias constant in j => same weights as no bias, o_pair = 1
    ones = small(seed=12, B=2, L=7, r=1)
    ones["z1"][:] = 1; ones["z2"][:] = 1
    nob = dict(ones); nob["w_b"] = np.zeros_like(ones["w_b"])
    g1 = ipa_oracle.forward(ones, want_attn=True)
    g0 = ipa_oracle.forward(nob, want_attn=True)
    assert np.allclose(g1["attn"], g0["attn"], atol=1e-13)
    assert np.allclose(g1["o_pair"], 1.0, atol=1e-13)


def test_mask_semantics():
    L, keep = 8, [0, 1, 3, 4, 7]
    mask = np.zeros((1, L), dtype=np.uint8); mask[0, keep] = 1
    inp = small(seed=13, L=L, mask=mask)
    got = ipa_oracle.forward(inp, want_attn=True)
    drop = [j for j in range(L) if j not in keep]
    assert np.all(got["attn"][0, :, :, drop] == 0)
    for n in ("o", "o_pts", "o_pair"):
        assert np.all(got[n][0, drop] == 0)
    # same as running on the valid residues alone
    sub = {n: (a[:, keep] if isinstance(a, np.ndarray) and a.ndim >= 2 and a.shape[1] == L else a)
           for n, a in inp.items()}
    sub["mask"] = None
    ref = ipa_oracle.forward(sub)
    for n in ("o", "o_pts", "o_pair"):
        assert np.allclose(got[n][0, keep], ref[n][0], atol=1e-12)
    # junk in padded slots is ignored
    junk = {n: (a.copy() if isinstance(a, np.ndarray) else a) for n, a in inp.items()}
    for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts", "trans", "z1", "z2"):
        junk[n][0, drop] = wl.PAD_GARBAGE
    again = ipa_oracle.forward(junk)
    for n in ("o", "o_pts", "o_pair"):
        assert np.array_equal(got[n], again[n])
    with pytest.raises(ValueError):
        bad = dict(inp); bad["mask"] = np.zeros((1, L), dtype=np.uint8)
        ipa_oracle.forward(bad)


def test_row_subset_form():
    inp = wl.make_inputs(0, L=24)
    full = ipa_oracle.forward(inp)
    rows = [np.array([23, 0, 7, 11], dtype=np.int32)]
    part = ipa_oracle.forward(inp, rows=rows)
    for n in ("o", "o_pts", "o_pair"):
        assert np.array_equal(part[n][0], full[n][0, rows[0]])


def loss(inp, ups):
    out = ipa_oracle.forward(inp)
    return sum(float(np.sum(out[n] * ups[n])) for n in ("o", "o_pts", "o_pair"))


@pytest.mark.parametrize("dense,masked", [(False, False), (True, False), (False, True)])
def test_backward_matches_central_differences(dense, masked):
    mask = np.array([[1, 1, 0, 1, 1]], dtype=np.uint8) if masked else None
    inp = small(seed=20 + dense, L=5, H=2, c=3, Pq=2, Pv=2, cz=3, r=2, dense=dense, mask=mask)
    rng = np.random.default_rng(99)
    ups = {n: rng.standard_normal(s) for n, s in
           (("o", (1, 5, 2, 3)), ("o_pts", (1, 5, 2, 2, 3)), ("o_pair", (1, 5, 2, 3)))}
    g = ipa_oracle.backward(inp, ups["o"], ups["o_pts"], ups["o_pair"])
    names = [("q", "dq"), ("k", "dk"), ("v", "dv"), ("q_pts", "dq_pts"), ("k_pts", "dk_pts"),
             ("v_pts", "dv_pts"), ("gamma", "dgamma"), ("w_b", "dw_b"), ("rot", "drot"), ("trans", "dtrans")]
    names += [("z", "dz")] if dense else [("z1", "dz1"), ("z2", "dz2")]
    h = 1e-5
    for src, dst in names:
        base = np.array(inp[src], dtype=np.float64)
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            vals = []
            for sgn in (+1, -1):
                pert = base.copy(); pert[idx] += sgn * h
                trial = dict(inp); trial[src] = pert
                vals.append(loss(trial, ups))
            fd[idx] = (vals[0] - vals[1]) / (2 * h)
        scale = max(np.abs(fd).max(), 1e-12)
        err = np.abs(g[dst] - fd).max() / scale
        assert err < 2e-7, (src, err)
        if masked and src not in ("gamma", "w_b"):
            assert np.all(g[dst][0, 2] == 0), src


def test_translation_gradients_sum_to_zero_and_rotation_gradient_has_no_net_torque():
    """A common shift of all frames leaves the loss unchanged, so the translation gradients sum to
    zero; so does a common rotation G, whose generator gives sum_i (dR_i R_i^T + dt_i t_i^T) with
    no antisymmetric part."""
    inp = small(seed=41, L=6)
    rng = np.random.default_rng(42)
    ups = [rng.standard_normal(inp[n].shape) for n in ("v", "v_pts")] + \
          [rng.standard_normal(inp["q"].shape[:3] + (4,))]
    g = ipa_oracle.backward(inp, *ups)
    assert np.abs(g["dtrans"].sum(axis=1)).max() <= 1e-10 * max(1.0, np.abs(g["dtrans"]).max())
    R, t = np.asarray(inp["rot"], dtype=np.float64), np.asarray(inp["trans"], dtype=np.float64)
    M = np.einsum("blxy,blzy->xz", g["drot"], R) + np.einsum("blx,blz->xz", g["dtrans"], t)
    assert np.abs(M - M.T).max() <= 1e-9 * max(1.0, np.abs(M).max())


def test_gradients_are_se3_invariant():
    # local-frame gradients do not change under a global move (sum_j dS_ij = 0)
    inp = small(seed=30, L=6)
    rng = np.random.default_rng(31)
    ups = [rng.standard_normal(inp[n].shape) for n in ("v", "v_pts")] + \
          [rng.standard_normal(inp["q"].shape[:3] + (4,))]
    g0 = ipa_oracle.backward(inp, *ups)
    g1 = ipa_oracle.backward(global_move(inp, 32), *ups)
    for n in ("dq", "dk", "dv", "dq_pts", "dk_pts", "dv_pts", "dz1", "dz2", "dgamma"):
        assert np.abs(g0[n] - g1[n]).max() <= 1e-9 * max(1.0, np.abs(g0[n]).max()), n


@pytest.mark.parametrize("masked", [False, True])
def test_sampled_backward_equals_dense_backward(masked):
    """The row-walking backward (for sizes where the dense pair tensor does not fit) must give, for
    any sampled residues, exactly the entries of the dense backward (itself pinned by central
    differences above) -- all residues sampled, a shuffled subset, and a single one."""
    L = 8
    mask = np.array([[1, 1, 0, 1, 1, 1, 0, 1], [1] * 8], dtype=np.uint8) if masked else None
    inp = small(seed=50, B=2, L=L, H=2, c=3, Pq=2, Pv=3, cz=4, r=2, mask=mask)
    rng = np.random.default_rng(51)
    ups = [rng.standard_normal(inp[n].shape) for n in ("v", "v_pts")] + \
          [rng.standard_normal(inp["q"].shape[:3] + (4,))]
    dense = ipa_oracle.backward(inp, *ups)
    for samples in ([np.arange(L)] * 2, [np.array([5, 0, 3]), np.array([7, 2, 6])], [np.array([4]), np.array([1])]):
        got = ipa_oracle.backward_sampled(inp, *ups, samples)
        for n in ("dq", "dk", "dv", "dq_pts", "dk_pts", "dv_pts", "dz1", "dz2", "drot", "dtrans"):
            for b in range(2):
                want = dense[n][b][samples[b]]
                assert np.abs(got[n][b] - want).max() <= 1e-12 * max(1.0, np.abs(dense[n]).max()), (n, b)
        for n in ("dgamma", "dw_b"):
            assert np.abs(got[n] - dense[n]).max() <= 1e-12 * max(1.0, np.abs(dense[n]).max()), n


def test_sampled_backward_on_a_workload_slice():
    # the generators of the forward+backward workload at a size both routines can sweep (several
    # threads share the rows here: the per-thread copies must add up)
    inp = wl.make_inputs(4, B=1, L=40, H=3, cz=8, r=2)
    ups = (inp["d_o"], inp["d_o_pts"], inp["d_o_pair"])
    dense = ipa_oracle.backward(inp, *ups)
    samples = [np.array([39, 0, 17, 18, 5])]
    got = ipa_oracle.backward_sampled(inp, *ups, samples)
    for n in ("dq", "dk", "dv", "dq_pts", "dk_pts", "dv_pts", "dz1", "dz2", "drot", "dtrans"):
        assert np.abs(got[n][0] - dense[n][0][samples[0]]).max() <= 1e-11 * np.abs(dense[n]).max(), n
    for n in ("dgamma", "dw_b"):
        assert np.abs(got[n] - dense[n]).max() <= 1e-11 * np.abs(dense[n]).max(), n


# ---- the module around the core (Eq. 1, Eq. 5) -----------------------------------------------------
def _tiny_module(seed=3, B=1, L=6, H=2, cz=8, r=2, d_s=None, varlen=False):
    from paper_2505_11580_amd import workloads as wl
    dims = dict(B=B, L=L, H=H, cz=cz, r=r, varlen=varlen, min_len=3, dtype="bf16")
    n_in, _ = wl.module_widths(dict(H=H, c=16, Pq=4, Pv=8, cz=cz))
    return wl.make_module_inputs(1, d_s=d_s or 24, seed=seed, **dims)


def test_module_identity_projections_reduce_to_core():
    """With identity weights and no bias the module is the core applied to slices of s, followed
    by the concatenation with norms, written here with plain loops."""
    from oracle import module_ref
    from paper_2505_11580_amd import workloads as wl
    m = _tiny_module()
    d = m["dims"]
    n_in, n_cat = wl.module_widths(d)
    rng = np.random.default_rng(0)
    m["s"] = wl.round_to_bf16(rng.standard_normal((d["B"], d["L"], n_in)).astype(np.float32))
    m["w_in"], m["b_in"] = np.eye(n_in), None
    m["w_out"], m["b_out"] = np.eye(n_cat), None
    got = module_ref.module_forward(m)
    H, c, Pq, Pv, cz = d["H"], d["c"], d["Pq"], d["Pv"], d["cz"]
    s = m["s"].astype(np.float64)
    inp = dict(m)
    at = 0
    for name, shp in (("q", (H, c)), ("k", (H, c)), ("v", (H, c)), ("q_pts", (H, Pq, 3)), ("k_pts", (H, Pq, 3)),
                      ("v_pts", (H, Pv, 3))):
        w = int(np.prod(shp))
        inp[name] = s[..., at:at + w].reshape((d["B"], d["L"]) + shp)
        at += w
    core = ipa_oracle.forward(inp)
    for b in range(d["B"]):
        for i in range(d["L"]):
            row = []
            for h in range(H):
                row += list(core["o_pair"][b, i, h])
            for h in range(H):
                row += list(core["o"][b, i, h])
            for h in range(H):
                for p in range(Pv):
                    row += list(core["o_pts"][b, i, h, p])
            for h in range(H):
                for p in range(Pv):
                    x, y, z = core["o_pts"][b, i, h, p]
                    row.append(math.sqrt(x * x + y * y + z * z))
            assert np.allclose(got[b, i], row, rtol=1e-12, atol=1e-12)


def test_module_is_invariant_under_global_rigid_motion():
    """Section 2.2: the IPA update is SE(3) invariant -- also through the norms of Eq. 5."""
    from oracle import module_ref
    m = _tiny_module(seed=5, L=7, varlen=True)
    base = module_ref.module_forward(m)
    rng = np.random.default_rng(1)
    qn = rng.standard_normal(4)
    qn /= np.linalg.norm(qn)
    w, x, y, z = qn
    G = np.array([[1 - 2 * (y * y + z * z), 2 * (x * y - z * w), 2 * (x * z + y * w)],
                  [2 * (x * y + z * w), 1 - 2 * (x * x + z * z), 2 * (y * z - x * w)],
                  [2 * (x * z - y * w), 2 * (y * z + x * w), 1 - 2 * (x * x + y * y)]])
    shift = np.array([30.0, -20.0, 5.0])
    moved = dict(m)
    moved["rot"] = np.einsum("xy,blyz->blxz", G, m["rot"].astype(np.float64))
    moved["trans"] = np.einsum("xy,bly->blx", G, m["trans"].astype(np.float64)) + shift
    assert np.allclose(module_ref.module_forward(moved), base, rtol=1e-9, atol=1e-9)
    # and it does depend on the frames: moving one residue alone changes the result
    one = dict(m)
    one["trans"] = m["trans"].astype(np.float64).copy()
    one["trans"][0, 1] += np.array([3.0, 0.0, 0.0])
    assert np.abs(module_ref.module_forward(one) - base).max() > 1e-6


def test_module_output_projection_is_affine_and_masked_rows_give_the_bias():
    from oracle import module_ref
    m = _tiny_module(seed=7, B=2, L=6, varlen=True)
    base = module_ref.module_forward(m)
    shifted = dict(m)
    delta = np.linspace(-1, 1, m["d_s"])
    shifted["b_out"] = m["b_out"].astype(np.float64) + delta
    assert np.allclose(module_ref.module_forward(shifted) - base, delta, atol=1e-12)
    doubled = dict(m)
    doubled["w_out"] = 2.0 * m["w_out"].astype(np.float64)
    b = m["b_out"].astype(np.float64)
    assert np.allclose(module_ref.module_forward(doubled) - b, 2.0 * (base - b), rtol=1e-12, atol=1e-12)
    for bi, ln in enumerate(m["lengths"]):
        assert np.allclose(base[bi, int(ln):], b, atol=1e-12)   # masked rows: zero core output
    # rows argument: a subset equals the full result at those rows
    rows = [np.array([0, 2], dtype=np.int32)] * 2
    assert np.allclose(module_ref.module_forward(m, rows=rows), base[:, [0, 2]], atol=1e-12)


def test_module_input_projection_orientation_and_rounding():
    """Eq. 1 with weights [out, in]: a single non-zero weight copies one input feature into one
    output feature; outputs are bfloat16 values; torch's Linear agrees before the rounding."""
    from oracle import module_ref
    m = _tiny_module(seed=9)
    d = m["dims"]
    n_in = m["w_in"].shape[0]
    w = np.zeros_like(m["w_in"], dtype=np.float64)
    w[5, 2] = 0.5           # output feature 5 (= q[h=0, channel 5]) <- 0.5 * s[..., 2]
    w[n_in - 1, 0] = -2.0   # last output feature (= v_pts[h=H-1, p=Pv-1, z]) <- -2 * s[..., 0]
    one = dict(m, w_in=w, b_in=None)
    got = module_ref.project_in(one)
    s = m["s"].astype(np.float64)
    assert np.array_equal(got["q"][..., 0, 5], 0.5 * s[..., 2])
    assert np.array_equal(got["v_pts"][..., d["H"] - 1, d["Pv"] - 1, 2], -2.0 * s[..., 0])
    assert np.count_nonzero(got["k"]) == 0 and np.count_nonzero(got["q_pts"]) == 0
    full = module_ref.project_in(m)
    ref = torch.nn.functional.linear(torch.tensor(s), torch.tensor(m["w_in"].astype(np.float64)),
                                     torch.tensor(m["b_in"].astype(np.float64))).numpy()
    flat = np.concatenate([full[n].reshape(d["B"], d["L"], -1) for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts")], -1)
    assert np.abs(flat - ref).max() <= 2.0 ** -8 * np.abs(ref).max()      # half an ulp of bf16
    assert np.array_equal(flat.astype(np.float32).view(np.uint32) & 0xFFFF, np.zeros(flat.shape, np.uint32))


def test_module_backward_matches_central_differences():
    """Every gradient of the module against central differences of its (unrounded) forward."""
    from oracle import module_ref
    from paper_2505_11580_amd import workloads as wl
    m = wl.make_module_inputs(1, d_s=8, seed=11, B=1, L=4, H=1, cz=8, r=2, varlen=False, dtype="bf16")
    m["mask"] = np.array([[1, 1, 0, 1]], dtype=np.uint8)
    for n in ("s", "w_in", "b_in", "w_out", "b_out"):
        m[n] = np.asarray(m[n], dtype=np.float64)
    rng = np.random.default_rng(12)
    up = rng.standard_normal((1, 4, 8))

    def loss(mm):
        return float(np.sum(module_ref.module_forward(mm, rounded=False) * up))

    g = module_ref.module_backward(m, up, rounded=False)
    h = 1e-5
    for src, dst in (("s", "ds"), ("b_in", "db_in"), ("w_out", "dw_out"), ("b_out", "db_out"), ("w_in", "dw_in")):
        base = m[src]
        fd = np.zeros_like(base)
        idxs = list(np.ndindex(base.shape))
        if len(idxs) > 150:                      # w_in, w_out: a fixed sample of entries
            idxs = [idxs[i] for i in np.random.default_rng(13).choice(len(idxs), 150, replace=False)]
        for idx in idxs:
            vals = []
            for sgn in (+1, -1):
                pert = base.copy(); pert[idx] += sgn * h
                vals.append(loss(dict(m, **{src: pert})))
            fd[idx] = (vals[0] - vals[1]) / (2 * h)
        sel = tuple(np.array(idxs).T)
        scale = max(np.abs(fd[sel]).max(), 1e-12)
        assert np.abs(g[dst][sel] - fd[sel]).max() / scale < 1e-6, (src, np.abs(g[dst][sel] - fd[sel]).max() / scale)
    assert np.all(g["ds"][0, 2] == 0)            # a masked residue receives no gradient
