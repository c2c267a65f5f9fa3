"""Thin ctypes binding of libfipa.so (include/fipa.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for device memory
and the current stream.  Loading fails loudly when the library has not been built -- there
is no fallback.
"""
import ctypes
import math
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FIPA_LIB selects another build of the same library (e.g. one compiled with different flags)
LIB_PATH = os.environ.get("FIPA_LIB") or os.path.join(_HERE, "libfipa.so")

FIPA_OK = 0
FIPA_ERR_INVALID_ARG = -1
FIPA_ERR_UNSUPPORTED = -2
FIPA_ERR_WORKSPACE = -3
FIPA_ERR_ALIGNMENT = -4
FIPA_ERR_LAUNCH = -5
FIPA_DTYPE_F32 = 0
FIPA_DTYPE_BF16 = 1
FIPA_FLAG_WAVE_SPECIALISED = 1  # desc.flags bit: opt-in attention kernel with two waves per SIMD
FIPA_FLAG_PACKED_PER_CHAIN = 2  # desc.flags bit: packed batches run chain after chain (smallest workspace)
FIPA_FLAG_KEEP_FORWARD = 4  # desc.flags bit: forward fills a backward-sized workspace, backward skips the recomputation

EXPORTS = ("fipa_version", "fipa_status_string", "fipa_workspace_bytes", "fipa_forward",
           "fipa_packed_workspace_bytes", "fipa_forward_packed", "fipa_backward_packed", "fipa_forward_static", "fipa_backward", "fipa_module_workspace_bytes", "fipa_module_forward",
           "fipa_module_backward_workspace_bytes", "fipa_module_backward",
           "fipa_knn_distogram", "fipa_factor_project", "fipa_factor_project_backward",
           "fipa_profile_begin", "fipa_profile_begin_every", "fipa_profile_end", "fipa_probe_mfma")
PROFILE_STAGES = 3


class FipaDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "L", "H", "c", "Pq", "Pv", "cz", "r", "dtype")] + \
               [("w_L", ctypes.c_float), ("w_C", ctypes.c_float), ("qk_scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


class FipaError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, status_string(code)))


_LIB = None


def lib():
    """Load libfipa.so once; raise if it is missing (build it with paper_2505_11580_amd/build.py)."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libfipa.so not built: run `python -m paper_2505_11580_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.fipa_version.restype = ctypes.c_int
        L.fipa_status_string.restype = ctypes.c_char_p
        L.fipa_status_string.argtypes = [ctypes.c_int]
        L.fipa_workspace_bytes.restype = ctypes.c_int
        L.fipa_workspace_bytes.argtypes = [ctypes.POINTER(FipaDesc), ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.fipa_forward.restype = ctypes.c_int
        L.fipa_forward.argtypes = [ctypes.POINTER(FipaDesc)] + [vp] * 17 + [vp, sz, vp]
        L.fipa_forward_static.restype = ctypes.c_int
        L.fipa_forward_static.argtypes = [ctypes.POINTER(FipaDesc)] + [vp] * 17 + [vp]
        L.fipa_forward_packed.restype = ctypes.c_int
        L.fipa_forward_packed.argtypes = [ctypes.POINTER(FipaDesc), ctypes.POINTER(ctypes.c_int32)] + [vp] * 17 + [vp, sz, vp]
        L.fipa_packed_workspace_bytes.restype = ctypes.c_int
        L.fipa_packed_workspace_bytes.argtypes = [ctypes.POINTER(FipaDesc), ctypes.POINTER(ctypes.c_int32),
                                                  ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.fipa_backward_packed.restype = ctypes.c_int
        L.fipa_backward_packed.argtypes = [ctypes.POINTER(FipaDesc), ctypes.POINTER(ctypes.c_int32)] + [vp] * 28 + [vp, sz, vp]
        L.fipa_backward.restype = ctypes.c_int
        L.fipa_backward.argtypes = [ctypes.POINTER(FipaDesc)] + [vp] * 32 + [vp, sz, vp]
        L.fipa_module_workspace_bytes.restype = ctypes.c_int
        L.fipa_module_workspace_bytes.argtypes = [ctypes.POINTER(FipaDesc), ctypes.c_int32, ctypes.POINTER(sz)]
        L.fipa_module_forward.restype = ctypes.c_int
        L.fipa_module_forward.argtypes = [ctypes.POINTER(FipaDesc), ctypes.c_int32] + [vp] * 13 + [vp, sz, vp]
        L.fipa_module_backward_workspace_bytes.restype = ctypes.c_int
        L.fipa_module_backward_workspace_bytes.argtypes = [ctypes.POINTER(FipaDesc), ctypes.c_int32, ctypes.POINTER(sz)]
        L.fipa_module_backward.restype = ctypes.c_int
        L.fipa_module_backward.argtypes = [ctypes.POINTER(FipaDesc), ctypes.c_int32] + [vp] * 24 + [vp, sz, vp]
        L.fipa_knn_distogram.restype = ctypes.c_int
        L.fipa_knn_distogram.argtypes = [ctypes.c_int32] * 4 + [ctypes.c_float] * 2 + [vp] * 5 + [vp]
        L.fipa_factor_project.restype = ctypes.c_int
        L.fipa_factor_project.argtypes = [ctypes.c_int32] * 7 + [vp] * 6 + [vp]
        L.fipa_factor_project_backward.restype = ctypes.c_int
        L.fipa_factor_project_backward.argtypes = [ctypes.c_int32] * 7 + [vp] * 7 + [vp]
        L.fipa_profile_begin.restype = ctypes.c_int
        L.fipa_profile_begin.argtypes = [ctypes.c_int]
        L.fipa_profile_begin_every.restype = ctypes.c_int
        L.fipa_profile_begin_every.argtypes = [ctypes.c_int, ctypes.c_int]
        L.fipa_profile_end.restype = ctypes.c_int
        L.fipa_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
        L.fipa_probe_mfma.restype = ctypes.c_int
        L.fipa_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, ctypes.POINTER(ctypes.c_double)]
        _LIB = L
    return _LIB


def status_string(code):
    return lib().fipa_status_string(int(code)).decode()


def make_desc(B, L, H, c, Pq, Pv, cz, r, dtype, w_L=None, w_C=None, qk_scale=None):
    """Description struct; defaults are the AlphaFold2 constants w_L = sqrt(1/3),
    w_C = sqrt(2/(9 Pq)) and qk_scale = 1/sqrt(c)."""
    return FipaDesc(B, L, H, c, Pq, Pv, cz, r, dtype,
                    math.sqrt(1.0 / 3.0) if w_L is None else w_L,
                    math.sqrt(2.0 / (9.0 * Pq)) if w_C is None else w_C,
                    1.0 / math.sqrt(c) if qk_scale is None else qk_scale, 0)


def workspace_bytes(desc):
    fwd, bwd = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = lib().fipa_workspace_bytes(ctypes.byref(desc), ctypes.byref(fwd), ctypes.byref(bwd))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_workspace_bytes")
    return fwd.value, bwd.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def fipa_forward(desc, q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                 o, o_pts, o_pair, lse, workspace):
    """Enqueue fipa_forward on torch's current stream.  All tensors are device tensors laid
    out as include/fipa.h states; `workspace` is a uint8 device tensor.  Returns nothing;
    raises FipaError on a non-zero status."""
    args = [q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse]
    rc = lib().fipa_forward(ctypes.byref(desc), *[_ptr(t) for t in args], _ptr(workspace),
                            ctypes.c_size_t(workspace.numel() if workspace is not None else 0), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_forward")


STATIC_SCRATCH_BYTES = 64 << 20  # FIPA_STATIC_SCRATCH_BYTES of include/fipa.h


def fipa_forward_static(desc, q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                        o, o_pts, o_pair, lse):
    """Enqueue fipa_forward_static (the library's own scratch array instead of a workspace) on
    torch's current stream."""
    args = [q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse]
    rc = lib().fipa_forward_static(ctypes.byref(desc), *[_ptr(t) for t in args], _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_forward_static")


def fipa_forward_packed(desc, cu_seqlens, q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                        o, o_pts, o_pair, lse, workspace):
    """Enqueue fipa_forward_packed: tensors with a leading [total] axis, `cu_seqlens` a host
    sequence of B + 1 row offsets."""
    cu = (ctypes.c_int32 * len(cu_seqlens))(*[int(x) for x in cu_seqlens])
    args = [q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse]
    rc = lib().fipa_forward_packed(ctypes.byref(desc), cu, *[_ptr(t) for t in args], _ptr(workspace),
                                   ctypes.c_size_t(workspace.numel() if workspace is not None else 0), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_forward_packed")


def packed_workspace_bytes(desc, cu_seqlens):
    """(forward bytes, backward bytes) that the packed calls need for these chain lengths."""
    cu = (ctypes.c_int32 * len(cu_seqlens))(*[int(x) for x in cu_seqlens])
    fwd, bwd = ctypes.c_size_t(0), ctypes.c_size_t(0)
    rc = lib().fipa_packed_workspace_bytes(ctypes.byref(desc), cu, ctypes.byref(fwd), ctypes.byref(bwd))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_packed_workspace_bytes")
    return fwd.value, bwd.value


def fipa_backward_packed(desc, cu_seqlens, q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                         d_o, d_o_pts, d_o_pair, d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2,
                         d_gamma, d_w_b, d_rot, d_trans, workspace):
    """Enqueue fipa_backward_packed: tensors with a leading [total] axis, `cu_seqlens` a host
    sequence of B + 1 row offsets; d_w_b and (d_rot, d_trans) may be None."""
    cu = (ctypes.c_int32 * len(cu_seqlens))(*[int(x) for x in cu_seqlens])
    args = [q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, d_o, d_o_pts, d_o_pair,
            d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2, d_gamma, d_w_b, d_rot, d_trans]
    rc = lib().fipa_backward_packed(ctypes.byref(desc), cu, *[_ptr(t) for t in args], _ptr(workspace),
                                    ctypes.c_size_t(workspace.numel() if workspace is not None else 0), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_backward_packed")


def fipa_backward(desc, q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                  o, o_pts, o_pair, lse, d_o, d_o_pts, d_o_pair,
                  d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2, d_gamma, d_w_b, d_rot, d_trans,
                  workspace):
    """Enqueue fipa_backward on torch's current stream; d_w_b and (d_rot, d_trans) may be None."""
    args = [q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
            o, o_pts, o_pair, lse, d_o, d_o_pts, d_o_pair,
            d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2, d_gamma, d_w_b, d_rot, d_trans]
    rc = lib().fipa_backward(ctypes.byref(desc), *[_ptr(t) for t in args], _ptr(workspace),
                             ctypes.c_size_t(workspace.numel() if workspace is not None else 0), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_backward")


def module_workspace_bytes(desc, d_s):
    n = ctypes.c_size_t(0)
    rc = lib().fipa_module_workspace_bytes(ctypes.byref(desc), int(d_s), ctypes.byref(n))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_module_workspace_bytes")
    return n.value


def fipa_module_forward(desc, d_s, s, w_in, b_in, rot, trans, z1, z2, w_b, gamma, mask, w_out, b_out, s_out,
                        workspace):
    """Enqueue fipa_module_forward on torch's current stream (b_in, b_out, mask may be None)."""
    args = [s, w_in, b_in, rot, trans, z1, z2, w_b, gamma, mask, w_out, b_out, s_out]
    rc = lib().fipa_module_forward(ctypes.byref(desc), int(d_s), *[_ptr(t) for t in args], _ptr(workspace),
                                   ctypes.c_size_t(workspace.numel() if workspace is not None else 0), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_module_forward")


def fipa_knn_distogram(k, n_bins, d_min, d_max, trans, mask, nbr_idx, nbr_d2, nbr_bin):
    """Enqueue fipa_knn_distogram on torch's current stream; trans [B, L, 3] float32, outputs [B, L, k]."""
    B, L = int(trans.shape[0]), int(trans.shape[1])
    rc = lib().fipa_knn_distogram(B, L, int(k), int(n_bins), float(d_min), float(d_max), _ptr(trans), _ptr(mask),
                                  _ptr(nbr_idx), _ptr(nbr_d2), _ptr(nbr_bin), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_knn_distogram")


def fipa_factor_project(pos_mode, nbr_idx, nbr_bin, e_bin, e_pos, bias, z):
    """Enqueue fipa_factor_project on torch's current stream; nbr_idx, nbr_bin [B, L, k] int32, e_bin
    [k, n_bins, n_out] and e_pos [k, n_pos, n_out] (or None) bf16, bias [n_out] float32 or None, z [B, L, n_out] bf16."""
    B, L, k = (int(x) for x in nbr_idx.shape)
    n_bins, n_out = int(e_bin.shape[1]), int(e_bin.shape[2])
    n_pos = 0 if e_pos is None else int(e_pos.shape[1])
    rc = lib().fipa_factor_project(B, L, k, n_bins, n_pos, int(pos_mode), n_out, _ptr(nbr_idx), _ptr(nbr_bin),
                                   _ptr(e_bin), _ptr(e_pos), _ptr(bias), _ptr(z), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_factor_project")


def fipa_factor_project_backward(pos_mode, nbr_idx, nbr_bin, d_z, mask, d_e_bin, d_e_pos, d_bias):
    """Enqueue fipa_factor_project_backward on torch's current stream; d_z [B, L, n_out] bf16, d_e_bin
    [k, n_bins, n_out], d_e_pos [k, n_pos, n_out] (or None) and d_bias [n_out] (or None) float32."""
    B, L, k = (int(x) for x in nbr_idx.shape)
    n_bins, n_out = int(d_e_bin.shape[1]), int(d_e_bin.shape[2])
    n_pos = 0 if d_e_pos is None else int(d_e_pos.shape[1])
    rc = lib().fipa_factor_project_backward(B, L, k, n_bins, n_pos, int(pos_mode), n_out, _ptr(nbr_idx), _ptr(nbr_bin),
                                            _ptr(d_z), _ptr(mask), _ptr(d_e_bin), _ptr(d_e_pos), _ptr(d_bias), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_factor_project_backward")


def fipa_profile_begin(capacity):
    rc = lib().fipa_profile_begin(int(capacity))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_profile_begin")


def fipa_profile_begin_every(capacity, every):
    rc = lib().fipa_profile_begin_every(int(capacity), int(every))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_profile_begin_every")


def fipa_profile_end():
    """Returns ([mean ms of stage 0, 1, 2], number of timed calls)."""
    ms = (ctypes.c_float * PROFILE_STAGES)()
    n = ctypes.c_int(0)
    rc = lib().fipa_profile_end(ms, ctypes.byref(n))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_profile_end")
    return [float(x) for x in ms], n.value


# ---- conveniences for tests and the benchmark (allocation + upload; no arithmetic) ----------

def probe_mfma(iters, workgroups, out):
    """Enqueue the MFMA-only probe kernel on torch's current stream; returns the flop it performs."""
    flop = ctypes.c_double(0.0)
    rc = lib().fipa_probe_mfma(int(iters), int(workgroups), _ptr(out), _stream(), ctypes.byref(flop))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_probe_mfma")
    return flop.value


def upload(inp, device="cuda:0"):
    """numpy workload dict (workloads.make_inputs) -> device tensors + desc."""
    import torch
    d = inp["dims"]
    bf16 = inp["dtype"] == "bf16"
    desc = make_desc(d["B"], d["L"], d["H"], d["c"], d["Pq"], d["Pv"], d["cz"], d["r"],
                     FIPA_DTYPE_BF16 if bf16 else FIPA_DTYPE_F32, inp["w_L"], inp["w_C"])
    dev = {}
    for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts", "z1", "z2"):
        t = torch.from_numpy(inp[n]).to(device)
        dev[n] = t.to(torch.bfloat16).contiguous() if bf16 else t.contiguous()
    for n in ("rot", "trans", "w_b", "gamma", "d_o", "d_o_pts", "d_o_pair"):
        if n in inp:
            dev[n] = torch.from_numpy(inp[n]).to(device).contiguous()
    dev["mask"] = None if inp.get("mask") is None else torch.from_numpy(inp["mask"]).to(device).contiguous()
    return desc, dev


def alloc_outputs(desc, device="cuda:0"):
    import torch
    B, L, H = desc.B, desc.L, desc.H
    f = dict(dtype=torch.float32, device=device)
    fwd, _ = workspace_bytes(desc)
    return dict(o=torch.empty(B, L, H, desc.c, **f), o_pts=torch.empty(B, L, H, desc.Pv, 3, **f),
                o_pair=torch.empty(B, L, H, desc.cz, **f), lse=torch.empty(B, H, L, **f),
                workspace=torch.empty(max(fwd, 16), dtype=torch.uint8, device=device))


def forward(desc, dev, out):
    fipa_forward(desc, dev["q"], dev["k"], dev["v"], dev["q_pts"], dev["k_pts"], dev["v_pts"],
                 dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"], dev["gamma"], dev["mask"],
                 out["o"], out["o_pts"], out["o_pair"], out["lse"], out["workspace"])


def upload_module(m, device="cuda:0"):
    """numpy module workload (workloads.make_module_inputs) -> desc, device tensors."""
    import torch
    d = m["dims"]
    desc = make_desc(d["B"], d["L"], d["H"], d["c"], d["Pq"], d["Pv"], d["cz"], d["r"], FIPA_DTYPE_BF16,
                     m["w_L"], m["w_C"])
    dev = {}
    for n in ("s", "w_in", "w_out", "z1", "z2"):
        dev[n] = torch.from_numpy(np.ascontiguousarray(m[n], dtype=np.float32)).to(device).to(torch.bfloat16).contiguous()
    for n in ("rot", "trans", "w_b", "gamma", "b_in", "b_out"):
        dev[n] = None if m.get(n) is None else torch.from_numpy(np.ascontiguousarray(m[n], dtype=np.float32)).to(device)
    dev["mask"] = None if m.get("mask") is None else torch.from_numpy(m["mask"]).to(device).contiguous()
    dev["s_out"] = torch.empty(d["B"], d["L"], m["d_s"], dtype=torch.float32, device=device)
    dev["workspace"] = torch.empty(max(module_workspace_bytes(desc, m["d_s"]), 16), dtype=torch.uint8, device=device)
    return desc, dev


def module_forward(desc, d_s, dev):
    fipa_module_forward(desc, d_s, dev["s"], dev["w_in"], dev["b_in"], dev["rot"], dev["trans"], dev["z1"],
                        dev["z2"], dev["w_b"], dev["gamma"], dev["mask"], dev["w_out"], dev["b_out"], dev["s_out"],
                        dev["workspace"])


def alloc_module_grads(desc, d_s, device="cuda:0"):
    """Gradient tensors and the workspace of fipa_module_backward."""
    import torch
    B, L, H = desc.B, desc.L, desc.H
    n_in = H * (3 * desc.c + 3 * (2 * desc.Pq + desc.Pv))
    n_cat = H * (desc.cz + desc.c + 4 * desc.Pv)
    f = dict(dtype=torch.float32, device=device)
    n = ctypes.c_size_t(0)
    rc = lib().fipa_module_backward_workspace_bytes(ctypes.byref(desc), int(d_s), ctypes.byref(n))
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_module_backward_workspace_bytes")
    return dict(d_s=torch.empty(B, L, d_s, **f), d_w_in=torch.empty(n_in, d_s, **f), d_b_in=torch.empty(n_in, **f),
                d_w_out=torch.empty(d_s, n_cat, **f), d_b_out=torch.empty(d_s, **f),
                d_z1=torch.empty(B, L, desc.r, desc.cz, dtype=torch.bfloat16, device=device),
                d_z2=torch.empty(B, L, desc.r, desc.cz, dtype=torch.bfloat16, device=device),
                d_gamma=torch.empty(H, **f), d_w_b=torch.empty(H, desc.cz, **f),
                d_rot=torch.empty(B, L, 3, 3, **f), d_trans=torch.empty(B, L, 3, **f),
                workspace=torch.empty(max(n.value, 16), dtype=torch.uint8, device=device))


def module_backward(desc, d_s, dev, d_s_out, grads):
    """dev: tensors of upload_module; d_s_out: float32 device tensor [B, L, d_s]."""
    args = [dev["s"], dev["w_in"], dev["b_in"], dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"],
            dev["gamma"], dev["mask"], dev["w_out"], dev["b_out"], d_s_out,
            grads["d_s"], grads["d_w_in"], grads["d_b_in"], grads["d_w_out"], grads["d_b_out"],
            grads["d_z1"], grads["d_z2"], grads["d_gamma"], grads["d_w_b"], grads["d_rot"], grads["d_trans"]]
    ws = grads["workspace"]
    rc = lib().fipa_module_backward(ctypes.byref(desc), int(d_s), *[_ptr(t) for t in args], _ptr(ws),
                                    ctypes.c_size_t(ws.numel()), _stream())
    if rc != FIPA_OK:
        raise FipaError(rc, "fipa_module_backward")


def alloc_grads(desc, device="cuda:0"):
    """Gradient tensors (dtype of the inputs) and the backward workspace."""
    import torch
    B, L, H = desc.B, desc.L, desc.H
    dt = torch.bfloat16 if desc.dtype == FIPA_DTYPE_BF16 else torch.float32
    f = dict(dtype=dt, device=device)
    _, bwd = workspace_bytes(desc)
    return dict(d_q=torch.empty(B, L, H, desc.c, **f), d_k=torch.empty(B, L, H, desc.c, **f),
                d_v=torch.empty(B, L, H, desc.c, **f),
                d_q_pts=torch.empty(B, L, H, desc.Pq, 3, **f), d_k_pts=torch.empty(B, L, H, desc.Pq, 3, **f),
                d_v_pts=torch.empty(B, L, H, desc.Pv, 3, **f),
                d_z1=torch.empty(B, L, desc.r, desc.cz, **f), d_z2=torch.empty(B, L, desc.r, desc.cz, **f),
                d_gamma=torch.empty(H, dtype=torch.float32, device=device),
                d_w_b=torch.empty(H, desc.cz, dtype=torch.float32, device=device),
                d_rot=torch.empty(B, L, 3, 3, dtype=torch.float32, device=device),
                d_trans=torch.empty(B, L, 3, dtype=torch.float32, device=device),
                workspace=torch.empty(max(bwd, 16), dtype=torch.uint8, device=device))


def backward(desc, dev, out, grads):
    """dev must hold d_o, d_o_pts, d_o_pair; out the forward results of the same inputs."""
    fipa_backward(desc, dev["q"], dev["k"], dev["v"], dev["q_pts"], dev["k_pts"], dev["v_pts"],
                  dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"], dev["gamma"], dev["mask"],
                  out["o"], out["o_pts"], out["o_pair"], out["lse"],
                  dev["d_o"], dev["d_o_pts"], dev["d_o_pair"],
                  grads["d_q"], grads["d_k"], grads["d_v"], grads["d_q_pts"], grads["d_k_pts"],
                  grads["d_v_pts"], grads["d_z1"], grads["d_z2"], grads["d_gamma"], grads.get("d_w_b"),
                  grads.get("d_rot"), grads.get("d_trans"), grads["workspace"])
