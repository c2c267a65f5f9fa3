"""Algorithm 1 of the paper (the factorized update rule) in float64 numpy -- test infrastructure.

This is the second, independent statement of the method: the squared distance of
Eq. 3 expanded into |Q|^2 - 2 Q.K + |K|^2 and folded, with the factor bias
vectors, into lifted q^, k^ of width c + 5*N_query + r*d_z and v^ of width
c + 3*N_value + r*d_z, followed by ordinary softmax attention on the lifted
features, the split, and the z1 contraction (Algorithm 1, steps 2-9).  The C
oracle (standard IPA on the dense pair tensor) must agree with it to float64
round-off whenever z_ij is exactly z1_i^T z2_j (Section 2.4).

Readings taken where the printed algorithm is silent or inconsistent with Eq. 3/4:
  * w_L multiplies the pair bias (Eq. 3), so it is folded into b^{h1};
  * Linear(z1), Linear(z2) of steps 2-3 are the diagonal maps that make
    b^{h1}.b^{h2} equal Linear(z_ij) of Eq. 2: b^{h1} = w_L * w_b[h] * z1, b^{h2} = z2;
  * the point output gets T_i^{-1} (Eq. 4), which step 8 leaves implicit.
"""
import numpy as np


def forward(inp):
    """Same inputs as oracle.ipa_oracle.forward with factors z1, z2; returns o, o_pts, o_pair, attn."""
    q, k, v = (np.asarray(inp[n], dtype=np.float64) for n in ("q", "k", "v"))
    q_pts, k_pts, v_pts = (np.asarray(inp[n], dtype=np.float64) for n in ("q_pts", "k_pts", "v_pts"))
    R = np.asarray(inp["rot"], dtype=np.float64)
    t = np.asarray(inp["trans"], dtype=np.float64)
    z1 = np.asarray(inp["z1"], dtype=np.float64)
    z2 = np.asarray(inp["z2"], dtype=np.float64)
    w_b = np.asarray(inp["w_b"], dtype=np.float64)
    gamma = np.asarray(inp["gamma"], dtype=np.float64)
    w_L, w_C = float(inp["w_L"]), float(inp["w_C"])
    mask = inp.get("mask")
    B, L, H, c = q.shape
    Pq, Pv = q_pts.shape[3], v_pts.shape[3]
    r, cz = z1.shape[2], z1.shape[3]

    # T_i o x for every point (steps 4-6)
    def to_global(p):  # [B,L,H,P,3]
        return np.einsum("blxy,blhpy->blhpx", R, p) + t[:, :, None, None, :]

    Q, K, V = to_global(q_pts), to_global(k_pts), to_global(v_pts)
    ones = np.ones((B, L, H, Pq))
    g = gamma[None, None, :, None]
    # steps 2-3: factor bias vectors
    b1 = w_L * w_b[None, None, :, None, :] * z1[:, :, None, :, :]            # [B,L,H,r,cz]
    b2 = np.broadcast_to(z2[:, :, None, :, :], (B, L, H, r, cz))
    # step 4: q^ = (q, T o q_pts, |T o q_pts|^2, 1, b1)
    q_hat = np.concatenate([q, Q.reshape(B, L, H, 3 * Pq), (Q ** 2).sum(-1), ones,
                            b1.reshape(B, L, H, r * cz)], axis=-1)
    # step 5: k^ = (w_L/sqrt(c) k, gamma w_L w_C T o k_pts, -gamma w_L w_C/2 * 1,
    #               -gamma w_L w_C/2 |T o k_pts|^2, b2)
    k_hat = np.concatenate([w_L / np.sqrt(c) * k,
                            (g[..., None] * w_L * w_C * K).reshape(B, L, H, 3 * Pq),
                            -g * w_L * w_C / 2 * ones,
                            -g * w_L * w_C / 2 * (K ** 2).sum(-1),
                            b2.reshape(B, L, H, r * cz)], axis=-1)
    # step 6: v^ = (v, T o v_pts, z2)
    v_hat = np.concatenate([v, V.reshape(B, L, H, 3 * Pv), b2.reshape(B, L, H, r * cz)], axis=-1)
    assert q_hat.shape[-1] == c + 5 * Pq + r * cz and v_hat.shape[-1] == c + 3 * Pv + r * cz

    # step 7: ordinary attention on the lifted features
    S = np.einsum("bihd,bjhd->bhij", q_hat, k_hat)
    if mask is not None:
        keym = np.asarray(mask) != 0
        S = np.where(keym[:, None, None, :], S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    A = np.exp(S)
    A = A / A.sum(axis=-1, keepdims=True)
    o_hat = np.einsum("bhij,bjhd->bihd", A, v_hat)

    # step 8: split; Eq. 4: inverse frame on the point part
    o = o_hat[..., :c]
    G = o_hat[..., c:c + 3 * Pv].reshape(B, L, H, Pv, 3)
    U = o_hat[..., c + 3 * Pv:].reshape(B, L, H, r, cz)
    o_pts = np.einsum("blyx,blhpy->blhpx", R, G - t[:, :, None, None, :])
    # step 9: o~ = z1^T (sum_j a_ij z2_j)
    o_pair = (z1[:, :, None, :, :] * U).sum(axis=3)
    if mask is not None:
        qm = (np.asarray(mask) != 0)[:, :, None]
        o = o * qm[..., None]
        o_pts = o_pts * qm[..., None, None]
        o_pair = o_pair * qm[..., None]
        A = A * (np.asarray(mask) != 0)[:, None, :, None]
    return {"o": o, "o_pts": o_pts, "o_pair": o_pair, "attn": np.transpose(A, (0, 2, 1, 3))}
