"""Seeded synthetic inputs shaped like the paper's protein / RNA workloads.

Only input generation lives here (random draws, frame construction, rounding to
bf16, padding) -- none of the method's arithmetic -- so that both the CPU oracle
tests and the GPU path can be fed from the same arrays.  numpy only.

The five named workloads follow the benchmark definition of this project:
  0  tiny fp32          B=1 L=64   c_z=16  r=2  translations N(0, 10 A) i.i.d.
  1  AF2-sized bf16     B=8 L=512  c_z=128 r=2  random-walk chain, 3.8 A steps
  2  long chain bf16    B=2 L=2048 c_z=128 r=2  random-walk chain
  3  var-len bf16       B=4 L<=8192 (lengths U[1024,8192], padded) r=4, key/query mask
  4  fwd+bwd bf16       B=2 L=4096 c_z=128 r=2  plus upstream gradients N(0,1)
All have H=12 heads (4 for workload 0), c=16, N_query=4, N_value=8, the head/point
counts of the AlphaFold2-style IPA module the paper matches (Section 3.2), and rank
2 (4 for workload 3) as in Section 3.2.  Lengths span the 512 crop that Table 2
lists up to the multi-thousand-residue chains of Sections 3.3-3.4.
"""
import math

import numpy as np

BASE_SEED = 20250511

CONFIGS = {
    0: dict(B=1, L=64, H=4, c=16, Pq=4, Pv=8, cz=16, r=2, dtype="fp32", chain=False, varlen=False),
    1: dict(B=8, L=512, H=12, c=16, Pq=4, Pv=8, cz=128, r=2, dtype="bf16", chain=True, varlen=False),
    2: dict(B=2, L=2048, H=12, c=16, Pq=4, Pv=8, cz=128, r=2, dtype="bf16", chain=True, varlen=False),
    3: dict(B=4, L=8192, H=12, c=16, Pq=4, Pv=8, cz=128, r=4, dtype="bf16", chain=True, varlen=True),
    4: dict(B=2, L=4096, H=12, c=16, Pq=4, Pv=8, cz=128, r=2, dtype="bf16", chain=True, varlen=False),
}

PAD_GARBAGE = 1.0e3  # finite junk written into padded slots; results must not depend on it


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32).reshape(a.shape)
    return np.where(np.isfinite(a), out, a)


def bf16_bits(a):
    """uint16 bit patterns of values that are already bf16-representable float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def quat_to_rot(qt):
    """Unit quaternions [..., 4] (w, x, y, z) -> rotation matrices [..., 3, 3]."""
    w, x, y, z = (qt[..., i] for i in range(4))
    R = np.stack([
        1 - 2 * (y * y + z * z), 2 * (x * y - w * z), 2 * (x * z + w * y),
        2 * (x * y + w * z), 1 - 2 * (x * x + z * z), 2 * (y * z - w * x),
        2 * (x * z - w * y), 2 * (y * z + w * x), 1 - 2 * (x * x + y * y)], axis=-1)
    return R.reshape(qt.shape[:-1] + (3, 3))


def random_rotations(rng, shape):
    qt = rng.standard_normal(shape + (4,))
    qt /= np.linalg.norm(qt, axis=-1, keepdims=True)
    return quat_to_rot(qt)


def make_inputs(cfg, seed=None, with_grads=None, trans_scale=1.0, **override):
    """Build one workload.  `override` replaces shape entries (B, L, H, cz, r, dtype, chain,
    varlen, min_len) so the same generators give oracle-sized cases.  trans_scale < 1
    shrinks the geometry so attention spreads over many keys.  Returns a dict of numpy
    arrays: q,k,v,q_pts,k_pts,v_pts,z1,z2 float32 (already bf16-representable when
    dtype == 'bf16'), rot, trans, w_b, gamma float32, mask uint8 [B,L] or None, lengths,
    w_L, w_C, dims, and d_o, d_o_pts, d_o_pair when gradients are requested."""
    p = dict(CONFIGS[cfg])
    p.update(override)
    if with_grads is None:
        with_grads = cfg == 4
    rng = np.random.default_rng(BASE_SEED + cfg if seed is None else seed)
    B, L, H, c, Pq, Pv, cz, r = (p[n] for n in ("B", "L", "H", "c", "Pq", "Pv", "cz", "r"))
    f32 = np.float32
    q = rng.standard_normal((B, L, H, c)).astype(f32)
    k = rng.standard_normal((B, L, H, c)).astype(f32)
    v = rng.standard_normal((B, L, H, c)).astype(f32)
    q_pts = rng.standard_normal((B, L, H, Pq, 3)).astype(f32)
    k_pts = rng.standard_normal((B, L, H, Pq, 3)).astype(f32)
    v_pts = rng.standard_normal((B, L, H, Pv, 3)).astype(f32)
    rot = random_rotations(rng, (B, L)).astype(f32)
    if p["chain"]:
        steps = rng.standard_normal((B, L, 3))
        steps /= np.linalg.norm(steps, axis=-1, keepdims=True)
        steps[:, 0, :] = 0.0
        trans = np.cumsum(3.8 * steps, axis=1)
    else:
        trans = 10.0 * rng.standard_normal((B, L, 3))
    trans = (trans * trans_scale).astype(f32)
    sigma = math.sqrt(1.0 / math.sqrt(r))  # variance 1/sqrt(r): z_ij[d] has unit variance
    z1 = (sigma * rng.standard_normal((B, L, r, cz))).astype(f32)
    z2 = (sigma * rng.standard_normal((B, L, r, cz))).astype(f32)
    gamma_raw = rng.standard_normal(H)
    gamma = np.log1p(np.exp(gamma_raw)).astype(f32)  # softplus
    w_b = (rng.standard_normal((H, cz)) / math.sqrt(cz)).astype(f32)
    mask, lengths = None, np.full(B, L, dtype=np.int64)
    if p["varlen"]:
        lo = p.get("min_len", max(1, L // 8))
        lengths = rng.integers(lo, L + 1, size=B)
        mask = (np.arange(L)[None, :] < lengths[:, None]).astype(np.uint8)
        pad = mask == 0
        for a in (q, k, v, q_pts, k_pts, v_pts, trans, z1, z2):
            a[pad] = PAD_GARBAGE
    out = dict(q=q, k=k, v=v, q_pts=q_pts, k_pts=k_pts, v_pts=v_pts, rot=rot, trans=trans,
               z1=z1, z2=z2, w_b=w_b, gamma=gamma, mask=mask, lengths=lengths,
               w_L=math.sqrt(1.0 / 3.0), w_C=math.sqrt(2.0 / (9.0 * Pq)),
               dims=dict(B=B, L=L, H=H, c=c, Pq=Pq, Pv=Pv, cz=cz, r=r), dtype=p["dtype"])
    if with_grads:
        out["d_o"] = rng.standard_normal((B, L, H, c)).astype(f32)
        out["d_o_pts"] = rng.standard_normal((B, L, H, Pv, 3)).astype(f32)
        out["d_o_pair"] = rng.standard_normal((B, L, H, cz)).astype(f32)
    if p["dtype"] == "bf16":
        for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts", "z1", "z2"):
            out[n] = round_to_bf16(out[n])
    return out


def module_widths(dims):
    """(N_in, N_cat): output width of the input projection (Eq. 1) and input width of the output
    projection (Eq. 5)."""
    H, c, Pq, Pv, cz = (dims[n] for n in ("H", "c", "Pq", "Pv", "cz"))
    return H * (3 * c + 3 * (2 * Pq + Pv)), H * (cz + c + 4 * Pv)


def make_module_inputs(cfg, d_s=256, seed=None, **override):
    """Inputs of the whole IPA module: the frames, pair factors and parameters of
    make_inputs(cfg, ...) plus the single representation s [B, L, d_s] (bf16 values) and the
    two Linear layers, weights [out, in] as bf16 values with variance 1/in, biases float32."""
    m = make_inputs(cfg, seed=seed, with_grads=False, **override)
    for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts"):
        del m[n]
    d = m["dims"]
    n_in, n_cat = module_widths(d)
    rng = np.random.default_rng(BASE_SEED + 100 + cfg if seed is None else seed + 100)
    m["s"] = round_to_bf16(rng.standard_normal((d["B"], d["L"], d_s)).astype(np.float32))
    m["w_in"] = round_to_bf16((rng.standard_normal((n_in, d_s)) / math.sqrt(d_s)).astype(np.float32))
    m["b_in"] = (0.1 * rng.standard_normal(n_in)).astype(np.float32)
    m["w_out"] = round_to_bf16((rng.standard_normal((d_s, n_cat)) / math.sqrt(n_cat)).astype(np.float32))
    m["b_out"] = (0.1 * rng.standard_normal(d_s)).astype(np.float32)
    if m["mask"] is not None:
        m["s"][m["mask"] == 0] = PAD_GARBAGE
    m["d_s"] = d_s
    return m


def select_rows(inp, n_rows, seed=0, tile=128):
    """Query rows for sampled parity at sizes the oracle cannot sweep: per batch element the
    first row, the last valid row, the first padded row (if any), one row at a random position
    inside every `tile`-row query tile that holds valid rows, and random valid rows up to n_rows
    (all distinct; every batch element gets the same count)."""
    rng = np.random.default_rng(seed)
    L = inp["dims"]["L"]
    rows = []
    for b, ln in enumerate(inp["lengths"]):
        ln = int(ln)
        picked = [0, ln - 1] + ([ln] if ln < L else [])
        for t0 in range(0, ln, tile):
            picked.append(int(rng.integers(t0, min(t0 + tile, ln))))
        picked = list(dict.fromkeys(picked))  # distinct, order kept
        if len(picked) < n_rows and ln > len(picked):
            rest = [int(x) for x in rng.permutation(ln) if int(x) not in set(picked)]
            picked += rest[:n_rows - len(picked)]
        rows.append(np.array(picked, dtype=np.int32))
    n = min(len(r) for r in rows)
    # (a short chain may offer fewer rows than a long one: drop from the random tail, never the fixed rows)
    return [r[:n] for r in rows]


def valid_pairs(inp):
    """Number of (b, h, i, j) pairs with both residues valid."""
    H = inp["dims"]["H"]
    return int(H * np.sum(inp["lengths"].astype(np.int64) ** 2))


def fwd_flops_per_pair(dims):
    """Algorithmic forward flops per valid pair: 2*(c+3Pq+1+r*cz) for the logit and
    2*(c+3Pv+r*cz) for the values (minimal exact widths; no padding, no split columns)."""
    return 2 * (dims["c"] + 3 * dims["Pq"] + 1 + dims["r"] * dims["cz"]) + \
        2 * (dims["c"] + 3 * dims["Pv"] + dims["r"] * dims["cz"])


def bwd_flops_per_pair(dims):
    dqk = dims["c"] + 3 * dims["Pq"] + 1 + dims["r"] * dims["cz"]
    dv = dims["c"] + 3 * dims["Pv"] + dims["r"] * dims["cz"]
    return 2 * (3 * dqk + 2 * dv)
