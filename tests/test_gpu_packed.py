"""GPU parity of the packed (variable-length) entry points, through the C ABI: chains of different
lengths stored back to back must give, on every valid row, what the oracle gives for the padded,
masked batch (a masked key contributes nothing, so the two are the same function).  Both ways of
running are covered: one set of launches over all chains, and chain after chain
(FIPA_FLAG_PACKED_PER_CHAIN, or lengths so uneven that the library picks it itself)."""
import numpy as np
import pytest

from oracle import ipa_oracle
from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu
from tests.test_gpu_backward import GRADS

pytestmark = pytest.mark.gpu

PACKED_IN = ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans", "z1", "z2")


def _pack(t, lengths):
    """[B, L, ...] -> [total, ...] (torch or numpy)."""
    import torch
    parts = [t[b, :ln] for b, ln in enumerate(lengths)]
    return torch.cat(parts, dim=0).contiguous() if isinstance(t, torch.Tensor) else np.concatenate(parts, axis=0)


def _setup(inp, flags):
    desc, dev = binding.upload(inp)
    desc.flags = flags
    lengths = [int(x) for x in inp["lengths"]]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    pk = {n: _pack(dev[n], lengths) for n in PACKED_IN}
    return desc, dev, pk, cu, lengths


def packed_forward(inp, flags=0):
    import torch
    desc, dev, pk, cu, lengths = _setup(inp, flags)
    total, H = int(cu[-1]), desc.H
    f = dict(dtype=torch.float32, device="cuda:0")
    out = dict(o=torch.full((total, H, desc.c), float("nan"), **f), o_pts=torch.full((total, H, desc.Pv, 3), float("nan"), **f),
               o_pair=torch.full((total, H, desc.cz), float("nan"), **f), lse=torch.full((H * total,), float("nan"), **f))
    ws = torch.empty(max(binding.packed_workspace_bytes(desc, cu)[0], 16), dtype=torch.uint8, device="cuda:0")
    binding.fipa_forward_packed(desc, cu, *[pk[n] for n in PACKED_IN], dev["w_b"], dev["gamma"], None,
                                out["o"], out["o_pts"], out["o_pair"], out["lse"], ws)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy().astype(np.float64) for n, t in out.items()}, cu, lengths, ws.numel()


def check_packed_forward(inp, label, flags=0):
    got, cu, lengths, ws_bytes = packed_forward(inp, flags)
    want = gu.oracle_forward_chunked(inp)
    padded = gu.run_gpu(inp)
    tol = gu.TOL[inp["dtype"]]
    H = inp["dims"]["H"]
    errs = {}
    for n in gu.NAMES:
        assert np.all(np.isfinite(got[n])), (label, n)
        errs[n] = gu.rel_err(got[n], _pack(want[n], lengths))
    print(label, {k: "%.2e" % v for k, v in errs.items()}, "lengths", lengths, "workspace %.1f MB" % (ws_bytes / 1e6), flush=True)
    for n in gu.NAMES:
        assert errs[n] <= tol, (label, n, errs[n])
    for b, ln in enumerate(lengths):
        blk = got["lse"][H * cu[b]:H * cu[b + 1]].reshape(H, ln)
        assert np.allclose(blk, padded["lse"][b, :, :ln], rtol=0, atol=2e-2 if inp["dtype"] == "bf16" else 1e-4), (label, b)
    return ws_bytes


@pytest.mark.parametrize("cfg,kw", [(0, dict(B=3, L=96, min_len=5, trans_scale=0.2)),
                                    (1, dict(B=4, L=300, H=2, min_len=1)),
                                    (1, dict(B=7, L=520, H=3, min_len=100, cz=32)),
                                    (1, dict(B=3, L=200, H=2, min_len=20, c=8, Pq=2, Pv=3, cz=32)),
                                    (3, dict(B=2, L=260, H=2, min_len=40))])
def test_packed_forward_matches_the_padded_oracle(cfg, kw):
    # fp32 (always chain after chain), bf16 fused path with the key-range split, a generic head shape
    # (separate preparation, pack, unfused attention and epilogue kernels), rank 4
    inp = wl.make_inputs(cfg, varlen=True, **kw)
    one = check_packed_forward(inp, "packed cfg%d %s" % (cfg, kw))
    per = check_packed_forward(inp, "packed per chain cfg%d" % cfg, flags=binding.FIPA_FLAG_PACKED_PER_CHAIN)
    assert per <= one


def test_packed_forward_with_an_empty_and_a_dominant_chain():
    # an empty chain between two others (one launch), and one chain far longer than the rest, for
    # which the library itself goes chain by chain (more than half of a padded workspace would be padding)
    inp = wl.make_inputs(1, B=3, L=300, H=2, varlen=True, min_len=30)
    inp["lengths"] = np.array([int(inp["lengths"][0]), 0, int(inp["lengths"][2])])
    inp["mask"][1, :] = 0
    got, cu, lengths, _ = packed_forward(inp)
    keep = dict(inp)  # (the oracle takes no batch element without a valid key: it sees the other two)
    for n in PACKED_IN:
        keep[n] = inp[n][[0, 2]]
    keep["mask"] = inp["mask"][[0, 2]]
    keep["dims"] = dict(inp["dims"], B=2)
    want = gu.oracle_forward_chunked(keep)
    for n in gu.NAMES:
        assert gu.rel_err(got[n], _pack(want[n], [lengths[0], lengths[2]])) <= gu.TOL["bf16"], n
    inp = wl.make_inputs(1, B=4, L=900, H=2, varlen=True, min_len=30)
    inp["lengths"] = np.array([900, 40, 33, 70])
    inp["mask"][:] = 0
    for b, ln in enumerate(inp["lengths"]):
        inp["mask"][b, :ln] = 1
    desc, _ = binding.upload(inp)
    cu = np.concatenate([[0], np.cumsum(inp["lengths"])])
    one = binding.make_desc(1, 900, desc.H, desc.c, desc.Pq, desc.Pv, desc.cz, desc.r, desc.dtype)
    assert binding.packed_workspace_bytes(desc, cu)[0] == binding.workspace_bytes(one)[0]
    check_packed_forward(inp, "packed dominant chain")


def packed_backward(inp, flags=0):
    import torch
    desc, dev, pk, cu, lengths = _setup(inp, flags)
    total, H = int(cu[-1]), desc.H
    up = {n: _pack(dev[n], lengths) for n in ("d_o", "d_o_pts", "d_o_pair")}
    bf = dict(dtype=torch.bfloat16, device="cuda:0")
    f = dict(dtype=torch.float32, device="cuda:0")
    g = {n: torch.full_like(pk[n[2:]], float("nan")) for n in ("d_q", "d_k", "d_v", "d_q_pts", "d_k_pts", "d_v_pts", "d_z1", "d_z2")}
    g["d_gamma"] = torch.full((H,), float("nan"), **f)
    g["d_w_b"] = torch.full((H, desc.cz), float("nan"), **f)
    g["d_rot"] = torch.full((total, 3, 3), float("nan"), **f)
    g["d_trans"] = torch.full((total, 3), float("nan"), **f)
    ws = torch.empty(max(binding.packed_workspace_bytes(desc, cu)[1], 16), dtype=torch.uint8, device="cuda:0")
    binding.fipa_backward_packed(desc, cu, *[pk[n] for n in PACKED_IN], dev["w_b"], dev["gamma"], None,
                                 up["d_o"], up["d_o_pts"], up["d_o_pair"],
                                 *[g[n] for n, _ in GRADS], ws)
    torch.cuda.synchronize()
    return {n: g[n].float().cpu().numpy().astype(np.float64) for n, _ in GRADS}, lengths


@pytest.mark.parametrize("kw", [dict(B=3, L=192, H=3, min_len=40, trans_scale=0.5),
                                dict(B=5, L=140, H=2, cz=32, min_len=10, trans_scale=0.5),
                                dict(B=2, L=150, H=2, min_len=60, c=8, Pq=2, Pv=3, cz=32),
                                dict(B=3, L=200, H=2, min_len=50, cz=128, r=4, trans_scale=0.5)])
def test_packed_backward_matches_the_padded_oracle(kw):
    inp = wl.make_inputs(4, varlen=True, **kw)
    want = ipa_oracle.backward(inp, inp["d_o"], inp["d_o_pts"], inp["d_o_pair"])
    floor = 1e-3 * float(np.abs(want["dv"]).max())
    for flags, label in ((0, "one launch"), (binding.FIPA_FLAG_PACKED_PER_CHAIN, "per chain")):
        got, lengths = packed_backward(inp, flags)
        errs = {}
        for n, o in GRADS:
            assert np.all(np.isfinite(got[n])), (label, n)
            w = want[o] if n in ("d_gamma", "d_w_b") else _pack(want[o], lengths)
            errs[n] = float(np.abs(got[n] - w).max()) / max(float(np.abs(w).max()), floor)
        print("packed backward", label, kw, {k: "%.1e" % v for k, v in errs.items()}, "lengths", lengths, flush=True)
        for n, _ in GRADS:
            assert errs[n] <= 2e-2, (label, n, errs[n])


def test_packed_many_short_chains_one_launch():
    # 40 chains of 20 to 130 residues (the training regime of Table 2's lengths): forward and backward
    inp = wl.make_inputs(4, B=40, L=130, H=2, cz=32, varlen=True, min_len=20, trans_scale=0.5)
    check_packed_forward(inp, "packed 40 short chains")
    want = ipa_oracle.backward(inp, inp["d_o"], inp["d_o_pts"], inp["d_o_pair"])
    got, lengths = packed_backward(inp)
    floor = 1e-3 * float(np.abs(want["dv"]).max())
    for n, o in GRADS:
        w = want[o] if n in ("d_gamma", "d_w_b") else _pack(want[o], lengths)
        err = float(np.abs(got[n] - w).max()) / max(float(np.abs(w).max()), floor)
        assert err <= 2e-2, (n, err)
