"""ctypes front end of the C oracle (oracle/ipa_oracle.c) -- test infrastructure only.

Standard IPA, Eqs. 2-4 of the paper, in float64 with a dense pair tensor.  The
functions here only marshal numpy arrays, loop over the batch and, when the
caller hands over factors (z1, z2), materialise z_ij = z1_i^T z2_j (Section
2.4) before calling the dense routine.  No method arithmetic lives in Python.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        bp = ctypes.POINTER(ctypes.c_uint8)
        i, d = ctypes.c_int, ctypes.c_double
        L.ipa_oracle_num_threads.restype = ctypes.c_int
        L.ipa_oracle_set_num_threads.restype = None
        L.ipa_oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.ipa_oracle_pair_rows.restype = None
        L.ipa_oracle_pair_rows.argtypes = [i, i, i, dp, dp, i, ip, dp]
        L.ipa_oracle_forward_rows.restype = ctypes.c_int
        L.ipa_oracle_forward_rows.argtypes = [i] * 6 + [dp] * 11 + [d, d, bp, i, ip] + [dp] * 4
        L.ipa_oracle_backward.restype = ctypes.c_int
        L.ipa_oracle_backward.argtypes = [i] * 6 + [dp] * 11 + [d, d, bp] + [dp] * 3 + [dp] * 11
        L.ipa_oracle_pair_backward.restype = None
        L.ipa_oracle_pair_backward.argtypes = [i, i, i, dp, dp, dp, dp, dp]
        L.ipa_oracle_backward_sampled.restype = ctypes.c_int
        L.ipa_oracle_backward_sampled.argtypes = [i] * 7 + [dp] * 12 + [d, d, bp] + [dp] * 3 + [i, ip] + [dp] * 12
        _LIB = L
    return _LIB


def num_threads():
    return int(lib().ipa_oracle_num_threads())


def set_num_threads(n):
    """Threads the oracle's row loops use from now on (marshalling only: omp_set_num_threads)."""
    lib().ipa_oracle_set_num_threads(int(n))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dims(inp):
    B, L, H, c = inp["q"].shape
    Pq = inp["q_pts"].shape[3]
    Pv = inp["v_pts"].shape[3]
    cz = inp["w_b"].shape[1]
    return B, L, H, c, Pq, Pv, cz


def pair_rows(z1_b, z2_b, rows):
    """z[rows, :, :] for one batch element from its factors [L, r, cz]."""
    z1_b, z2_b = _f64(z1_b), _f64(z2_b)
    L, r, cz = z1_b.shape
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((len(rows), L, cz), dtype=np.float64)
    lib().ipa_oracle_pair_rows(L, r, cz, _p(z1_b), _p(z2_b), len(rows),
                               rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _p(out))
    return out


def forward(inp, rows=None, want_attn=False):
    """Standard IPA forward (Eqs. 2-4).

    inp: dict with q,k,v [B,L,H,c]; q_pts,k_pts [B,L,H,Pq,3]; v_pts [B,L,H,Pv,3];
    rot [B,L,3,3]; trans [B,L,3]; w_b [H,cz]; gamma [H]; w_L, w_C (floats);
    mask [B,L] (1 = valid) or None; and EITHER z [B,L,L,cz] (dense) OR z1,z2 [B,L,r,cz].
    rows: None (every query row) or one index array per batch element.
    Returns dict o [B,n,H,c], o_pts [B,n,H,Pv,3], o_pair [B,n,H,cz] (+ attn [B,n,H,L]);
    n = L or the common length of the row lists.
    """
    B, L, H, c, Pq, Pv, cz = _dims(inp)
    if rows is None:
        rows = [np.arange(L, dtype=np.int32)] * B
    rows = [np.ascontiguousarray(r, dtype=np.int32) for r in rows]
    n = len(rows[0])
    assert all(len(r) == n for r in rows)
    o = np.zeros((B, n, H, c))
    o_pts = np.zeros((B, n, H, Pv, 3))
    o_pair = np.zeros((B, n, H, cz))
    attn = np.zeros((B, n, H, L)) if want_attn else None
    w_b, gamma = _f64(inp["w_b"]), _f64(inp["gamma"])
    mask = inp.get("mask")
    for b in range(B):
        if "z" in inp and inp["z"] is not None:
            z_rows = _f64(np.asarray(inp["z"][b])[rows[b]])
        else:
            z_rows = pair_rows(inp["z1"][b], inp["z2"][b], rows[b])
        arrs = [_f64(inp[key][b]) for key in
                ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans")]
        m = None
        mp = ctypes.POINTER(ctypes.c_uint8)()
        if mask is not None:
            m = np.ascontiguousarray(np.asarray(mask[b]) != 0, dtype=np.uint8)
            mp = m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
        ob, opb, ozb = np.zeros((n, H, c)), np.zeros((n, H, Pv, 3)), np.zeros((n, H, cz))
        ab = np.zeros((n, H, L)) if want_attn else None
        rc = lib().ipa_oracle_forward_rows(
            L, H, c, Pq, Pv, cz, *[_p(a) for a in arrs], _p(z_rows), _p(w_b), _p(gamma),
            float(inp["w_L"]), float(inp["w_C"]), mp, n,
            rows[b].ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
            _p(ob), _p(opb), _p(ozb), _p(ab) if want_attn else ctypes.POINTER(ctypes.c_double)())
        if rc != 0:
            raise ValueError("oracle: batch element %d has no valid key" % b)
        o[b], o_pts[b], o_pair[b] = ob, opb, ozb
        if want_attn:
            attn[b] = ab
    out = {"o": o, "o_pts": o_pts, "o_pair": o_pair}
    if want_attn:
        out["attn"] = attn
    return out


def backward(inp, d_o, d_o_pts, d_o_pair):
    """Gradients of sum(o*d_o) + sum(o_pts*d_o_pts) + sum(o_pair*d_o_pair).

    Same inp as forward().  Returns dq, dk, dv, dq_pts, dk_pts, dv_pts, dgamma [H],
    dw_b [H,cz], dz [B,L,L,cz], drot [B,L,3,3] (every entry of R_i taken as a free variable),
    dtrans [B,L,3] and, when inp holds factors, dz1, dz2 [B,L,r,cz].
    """
    B, L, H, c, Pq, Pv, cz = _dims(inp)
    w_b, gamma = _f64(inp["w_b"]), _f64(inp["gamma"])
    mask = inp.get("mask")
    factored = not ("z" in inp and inp["z"] is not None)
    g = {key: np.zeros(np.asarray(inp[src]).shape) for key, src in
         (("dq", "q"), ("dk", "k"), ("dv", "v"), ("dq_pts", "q_pts"), ("dk_pts", "k_pts"),
          ("dv_pts", "v_pts"))}
    g["dz"] = np.zeros((B, L, L, cz))
    g["dgamma"] = np.zeros(H)
    g["dw_b"] = np.zeros((H, cz))
    g["drot"] = np.zeros((B, L, 3, 3))
    g["dtrans"] = np.zeros((B, L, 3))
    if factored:
        g["dz1"] = np.zeros(np.asarray(inp["z1"]).shape)
        g["dz2"] = np.zeros(np.asarray(inp["z2"]).shape)
    all_rows = np.arange(L, dtype=np.int32)
    for b in range(B):
        z = pair_rows(inp["z1"][b], inp["z2"][b], all_rows) if factored else _f64(inp["z"][b])
        arrs = [_f64(inp[key][b]) for key in
                ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans")]
        mp = ctypes.POINTER(ctypes.c_uint8)()
        if mask is not None:
            m = np.ascontiguousarray(np.asarray(mask[b]) != 0, dtype=np.uint8)
            mp = m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
        ups = [_f64(d_o[b]), _f64(d_o_pts[b]), _f64(d_o_pair[b])]
        outs = [np.zeros((L, H, c)), np.zeros((L, H, c)), np.zeros((L, H, c)),
                np.zeros((L, H, Pq, 3)), np.zeros((L, H, Pq, 3)), np.zeros((L, H, Pv, 3)),
                np.zeros((L, L, cz)), np.zeros(H), np.zeros((H, cz)), np.zeros((L, 3, 3)), np.zeros((L, 3))]
        lib().ipa_oracle_backward(
            L, H, c, Pq, Pv, cz, *[_p(a) for a in arrs], _p(z), _p(w_b), _p(gamma),
            float(inp["w_L"]), float(inp["w_C"]), mp, *[_p(a) for a in ups],
            *[_p(a) for a in outs])
        for key, arr in zip(("dq", "dk", "dv", "dq_pts", "dk_pts", "dv_pts", "dz"), outs[:7]):
            g[key][b] = arr
        g["dgamma"] += outs[7]
        g["dw_b"] += outs[8]
        g["drot"][b], g["dtrans"][b] = outs[9], outs[10]
        if factored:
            z1b, z2b = _f64(inp["z1"][b]), _f64(inp["z2"][b])
            r = z1b.shape[1]
            d1, d2 = np.zeros_like(z1b), np.zeros_like(z2b)
            lib().ipa_oracle_pair_backward(L, r, cz, _p(z1b), _p(z2b), _p(outs[6]), _p(d1), _p(d2))
            g["dz1"][b], g["dz2"][b] = d1, d2
    return g


def backward_sampled(inp, d_o, d_o_pts, d_o_pair, samples):
    """The gradients of backward() at sizes where the dense pair tensor does not fit: inp must hold
    factors z1, z2; samples is one index array per batch element (equal lengths n).  Returns dq, dk,
    dv [B,n,H,c], dq_pts, dk_pts [B,n,H,Pq,3], dv_pts [B,n,H,Pv,3], dz1, dz2 [B,n,r,cz], drot [B,n,3,3],
    dtrans [B,n,3] for the sampled residues (entry a <-> residue samples[b][a]) and the full dgamma [H],
    dw_b [H,cz]."""
    B, L, H, c, Pq, Pv, cz = _dims(inp)
    r = np.asarray(inp["z1"]).shape[2]
    samples = [np.ascontiguousarray(x, dtype=np.int32) for x in samples]
    n = len(samples[0])
    assert all(len(x) == n and len(set(x.tolist())) == n for x in samples)
    w_b, gamma = _f64(inp["w_b"]), _f64(inp["gamma"])
    mask = inp.get("mask")
    shapes = (("dq", (n, H, c)), ("dk", (n, H, c)), ("dv", (n, H, c)), ("dq_pts", (n, H, Pq, 3)),
              ("dk_pts", (n, H, Pq, 3)), ("dv_pts", (n, H, Pv, 3)), ("dz1", (n, r, cz)), ("dz2", (n, r, cz)),
              ("drot", (n, 3, 3)), ("dtrans", (n, 3)))
    g = {key: np.zeros((B,) + shp) for key, shp in shapes}
    g["dgamma"] = np.zeros(H)
    g["dw_b"] = np.zeros((H, cz))
    for b in range(B):
        arrs = [_f64(inp[key][b]) for key in
                ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans", "z1", "z2")]
        mp = ctypes.POINTER(ctypes.c_uint8)()
        if mask is not None:
            m = np.ascontiguousarray(np.asarray(mask[b]) != 0, dtype=np.uint8)
            mp = m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
        ups = [_f64(d_o[b]), _f64(d_o_pts[b]), _f64(d_o_pair[b])]
        outs = [np.zeros(shp) for _, shp in shapes] + [np.zeros(H), np.zeros((H, cz))]
        lib().ipa_oracle_backward_sampled(
            L, H, c, Pq, Pv, cz, r, *[_p(a) for a in arrs], _p(w_b), _p(gamma),
            float(inp["w_L"]), float(inp["w_C"]), mp, *[_p(a) for a in ups], n,
            samples[b].ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), *[_p(a) for a in outs])
        for (key, _), arr in zip(shapes, outs[:10]):
            g[key][b] = arr
        g["dgamma"] += outs[10]
        g["dw_b"] += outs[11]
    return g
