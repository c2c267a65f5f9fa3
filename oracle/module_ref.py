"""IPA module around the attention core (Eq. 1 and Eq. 5 of the paper; Algorithm 1 steps 1 and
10) in numpy float64 -- test infrastructure only.

    q, k, v, q_pts, k_pts, v_pts = Linear(s)                         (Eq. 1)
    o, o_pts, o_pair            = IPA core (Eqs. 2-4, oracle/ipa_oracle)
    s_out = Linear(concat_{h,p}(o_pair, o, o_pts, |o_pts|_2))        (Eq. 5)

Readings: weights are stored as [out_features, in_features]; the first Linear produces, in this
order, q | k | v [H, c] each, q_pts | k_pts [H, Pq, 3], v_pts [H, Pv, 3]; its results are
rounded to bfloat16, the type in which the core takes them (a bf16 model's Linear returns bf16);
the concatenation order is o_pair [H, cz] | o [H, c] | o_pts [H, Pv, 3] | norms [H, Pv]; the norm
is the plain Euclidean norm (its regulariser at zero only matters for gradients).
"""
import numpy as np

from . import ipa_oracle


def _bf16(a):
    """Round float64/float32 values to the nearest bfloat16 (ties to even), as float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16).astype(np.uint32)
    return r.view(np.float32).reshape(f.shape).astype(np.float64)


_NAMES = ("q", "k", "v", "q_pts", "k_pts", "v_pts")


def _in_shapes(d):
    B, L, H, c, Pq, Pv = d["B"], d["L"], d["H"], d["c"], d["Pq"], d["Pv"]
    widths = [H * c, H * c, H * c, H * Pq * 3, H * Pq * 3, H * Pv * 3]
    shapes = [(B, L, H, c)] * 3 + [(B, L, H, Pq, 3)] * 2 + [(B, L, H, Pv, 3)]
    return widths, shapes


def project_in(m, rounded=True):
    """Eq. 1: the six inputs of the core from the single representation s [B, L, d_s].
    rounded=False leaves out the bfloat16 rounding of the results (for derivative checks)."""
    d = m["dims"]
    B, L, H, c, Pq, Pv = d["B"], d["L"], d["H"], d["c"], d["Pq"], d["Pv"]
    x = np.asarray(m["s"], dtype=np.float64) @ np.asarray(m["w_in"], dtype=np.float64).T
    if m.get("b_in") is not None:
        x = x + np.asarray(m["b_in"], dtype=np.float64)
    if rounded:
        x = _bf16(x)
    widths, shapes = _in_shapes(d)
    out, at = {}, 0
    for name, w, shp in zip(_NAMES, widths, shapes):
        out[name] = x[..., at:at + w].reshape(shp)
        at += w
    assert at == x.shape[-1]
    return out


def concat_out(core, dims):
    """The argument of Eq. 5's Linear: [B, n, H*cz + H*c + H*Pv*3 + H*Pv]."""
    B, n = core["o"].shape[:2]
    norms = np.sqrt((core["o_pts"] ** 2).sum(-1))
    return np.concatenate([core["o_pair"].reshape(B, n, -1), core["o"].reshape(B, n, -1),
                           core["o_pts"].reshape(B, n, -1), norms.reshape(B, n, -1)], axis=-1)


def module_forward(m, rows=None, rounded=True):
    """m: dict with s, w_in, b_in, w_out, b_out and the core's frame / pair / parameter entries
    (rot, trans, z1, z2 or z, w_b, gamma, w_L, w_C, mask, dims).  Returns s_out [B, n, d_s]."""
    inp = dict(m)
    inp.update(project_in(m, rounded))
    core = ipa_oracle.forward(inp, rows=rows)
    cat = concat_out(core, m["dims"])
    out = cat @ np.asarray(m["w_out"], dtype=np.float64).T
    if m.get("b_out") is not None:
        out = out + np.asarray(m["b_out"], dtype=np.float64)
    return out


def module_backward(m, d_s_out, rounded=True):
    """Gradients of sum(s_out * d_s_out) with respect to s, w_in, b_in, w_out, b_out, plus the
    core's own parameter gradients (dz1, dz2, dgamma, dw_b, drot, dtrans) passed through.
    Readings: the bfloat16 rounding of Eq. 1's results is transparent to the gradient
    (straight-through); the derivative of the norm at a zero vector is taken as zero."""
    d = m["dims"]
    B, L = d["B"], d["L"]
    inp = dict(m)
    inp.update(project_in(m, rounded))
    core = ipa_oracle.forward(inp)
    cat = concat_out(core, d)
    g = np.asarray(d_s_out, dtype=np.float64)
    w_out = np.asarray(m["w_out"], dtype=np.float64)
    out = {"dw_out": np.einsum("blo,bli->oi", g, cat), "db_out": g.sum(axis=(0, 1))}
    dcat = g @ w_out                                         # [B, L, N_cat]
    H, c, Pv, cz = d["H"], d["c"], d["Pv"], d["cz"]
    e1, e2, e3 = H * cz, H * cz + H * c, H * cz + H * c + H * Pv * 3
    d_o_pair = dcat[..., :e1].reshape(B, L, H, cz)
    d_o = dcat[..., e1:e2].reshape(B, L, H, c)
    d_o_pts = dcat[..., e2:e3].reshape(B, L, H, Pv, 3).copy()
    d_norm = dcat[..., e3:].reshape(B, L, H, Pv)
    norms = np.sqrt((core["o_pts"] ** 2).sum(-1))
    unit = np.divide(core["o_pts"], norms[..., None], out=np.zeros_like(core["o_pts"]), where=norms[..., None] > 0)
    d_o_pts += d_norm[..., None] * unit
    gc = ipa_oracle.backward(inp, d_o, d_o_pts, d_o_pair)
    dx = np.concatenate([gc["d" + n].reshape(B, L, -1) for n in _NAMES], axis=-1)   # [B, L, N_in]
    out["ds"] = dx @ np.asarray(m["w_in"], dtype=np.float64)
    out["dw_in"] = np.einsum("blo,bli->oi", dx, np.asarray(m["s"], dtype=np.float64))
    out["db_in"] = dx.sum(axis=(0, 1))
    for n in ("dz1", "dz2", "dgamma", "dw_b", "drot", "dtrans"):
        if n in gc:
            out[n] = gc[n]
    return out
