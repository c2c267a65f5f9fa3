"""GPU tests of FIPA_FLAG_KEEP_FORWARD, through the C ABI: a forward call that fills a workspace of
the backward's size, followed by a backward call that skips the recomputation.  The forward's
outputs are held to the oracle at the usual tolerance; the gradients must be the very bits the
recomputing backward gives (the same kernels run on the same operands, in one call or in two)."""
import numpy as np
import pytest

from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu
from tests.test_gpu_backward import GRADS, run_gpu_backward
from tests.test_gpu_packed import PACKED_IN, _pack, _setup, packed_backward

pytestmark = pytest.mark.gpu


def keep_step(inp, scribble=True):
    """forward (flag) -> backward (flag) on one workspace; outputs and gradients as float64 arrays."""
    import torch
    desc, dev = binding.upload(inp)
    desc.flags = binding.FIPA_FLAG_KEEP_FORWARD
    out = binding.alloc_outputs(desc)
    grads = binding.alloc_grads(desc)
    for n in gu.NAMES:
        out[n].fill_(float("nan"))
    for n, _ in GRADS:
        grads[n].fill_(float("nan"))
    out["workspace"] = grads["workspace"]  # the backward's size
    if scribble:
        grads["workspace"].fill_(0xFF)
    binding.forward(desc, dev, out)
    binding.backward(desc, dev, out, grads)
    torch.cuda.synchronize()
    res = {n: out[n].cpu().numpy().astype(np.float64) for n in gu.NAMES}
    return res, {n: grads[n].float().cpu().numpy().astype(np.float64) for n, _ in GRADS}


@pytest.mark.parametrize("kw", [dict(B=2, L=200, H=3, trans_scale=0.5),
                                dict(B=2, L=300, H=2, varlen=True, min_len=40, trans_scale=0.3),
                                dict(B=1, L=150, H=2, c=8, Pq=2, Pv=3, cz=32),
                                dict(B=1, L=160, H=2, cz=128, r=4, trans_scale=0.5)])
def test_keep_forward_outputs_and_gradients(kw):
    # the AlphaFold2 head shape with and without padding, a generic head shape, rank 4
    inp = wl.make_inputs(4, **kw)
    out, got = keep_step(inp)
    want = gu.oracle_forward_chunked(inp)
    for n in gu.NAMES:
        assert np.all(np.isfinite(out[n])), n
        assert gu.rel_err(out[n], want[n]) <= gu.TOL["bf16"], (kw, n)
    plain = run_gpu_backward(inp)
    for n, _ in GRADS:
        assert np.array_equal(got[n], plain[n]), (kw, n, float(np.abs(got[n] - plain[n]).max()))


def test_keep_forward_packed():
    import torch
    inp = wl.make_inputs(4, B=4, L=180, H=2, cz=32, varlen=True, min_len=60, trans_scale=0.5)
    desc, dev, pk, cu, lengths = _setup(inp, binding.FIPA_FLAG_KEEP_FORWARD)
    total, H = int(cu[-1]), desc.H
    f = dict(dtype=torch.float32, device="cuda:0")
    out = dict(o=torch.full((total, H, desc.c), float("nan"), **f), o_pts=torch.full((total, H, desc.Pv, 3), float("nan"), **f),
               o_pair=torch.full((total, H, desc.cz), float("nan"), **f), lse=torch.full((H * total,), float("nan"), **f))
    up = {n: _pack(dev[n], lengths) for n in ("d_o", "d_o_pts", "d_o_pair")}
    g = {n: torch.full_like(pk[n[2:]], float("nan")) for n in ("d_q", "d_k", "d_v", "d_q_pts", "d_k_pts", "d_v_pts", "d_z1", "d_z2")}
    g["d_gamma"] = torch.full((H,), float("nan"), **f)
    g["d_w_b"] = torch.full((H, desc.cz), float("nan"), **f)
    g["d_rot"] = torch.full((total, 3, 3), float("nan"), **f)
    g["d_trans"] = torch.full((total, 3), float("nan"), **f)
    ws = torch.empty(binding.packed_workspace_bytes(desc, cu)[1], dtype=torch.uint8, device="cuda:0")
    binding.fipa_forward_packed(desc, cu, *[pk[n] for n in PACKED_IN], dev["w_b"], dev["gamma"], None,
                                out["o"], out["o_pts"], out["o_pair"], out["lse"], ws)
    binding.fipa_backward_packed(desc, cu, *[pk[n] for n in PACKED_IN], dev["w_b"], dev["gamma"], None,
                                 up["d_o"], up["d_o_pts"], up["d_o_pair"], *[g[n] for n, _ in GRADS], ws)
    torch.cuda.synchronize()
    want = gu.oracle_forward_chunked(inp)
    for n in gu.NAMES:
        assert gu.rel_err(out[n].cpu().numpy().astype(np.float64), _pack(want[n], lengths)) <= gu.TOL["bf16"], n
    plain, _ = packed_backward(inp)
    for n, _ in GRADS:
        assert np.array_equal(g[n].float().cpu().numpy().astype(np.float64), plain[n]), n


def test_keep_forward_refusals():
    import torch
    inp = wl.make_inputs(4, B=3, L=140, H=2, cz=32, varlen=True, min_len=30)
    desc, dev = binding.upload(inp)
    desc.flags = binding.FIPA_FLAG_KEEP_FORWARD
    out = binding.alloc_outputs(desc)
    full = out["workspace"]
    out["workspace"] = torch.empty(binding.workspace_bytes(desc)[1] - 256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.FipaError) as e:  # smaller than the backward's size
        binding.forward(desc, dev, out)
    out["workspace"] = full
    assert e.value.code == binding.FIPA_ERR_WORKSPACE
    with pytest.raises(binding.FipaError) as e:
        binding.fipa_forward_static(desc, dev["q"], dev["k"], dev["v"], dev["q_pts"], dev["k_pts"], dev["v_pts"],
                                    dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"], dev["gamma"], dev["mask"],
                                    out["o"], out["o_pts"], out["o_pair"], out["lse"])
    assert e.value.code == binding.FIPA_ERR_UNSUPPORTED
    # packed, forced chain by chain: each chain would overwrite what the previous one left
    desc, dev, pk, cu, lengths = _setup(inp, binding.FIPA_FLAG_KEEP_FORWARD | binding.FIPA_FLAG_PACKED_PER_CHAIN)
    total, H = int(cu[-1]), desc.H
    f = dict(dtype=torch.float32, device="cuda:0")
    o = torch.empty(total, H, desc.c, **f)
    o_pts = torch.empty(total, H, desc.Pv, 3, **f)
    o_pair = torch.empty(total, H, desc.cz, **f)
    ws = torch.empty(1 << 26, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.FipaError) as e:
        binding.fipa_forward_packed(desc, cu, *[pk[n] for n in PACKED_IN], dev["w_b"], dev["gamma"], None,
                                    o, o_pts, o_pair, None, ws)
    assert e.value.code == binding.FIPA_ERR_UNSUPPORTED
    # fp32 has no backward
    inp32 = wl.make_inputs(0, B=1, L=64)
    desc32, dev32 = binding.upload(inp32)
    desc32.flags = binding.FIPA_FLAG_KEEP_FORWARD
    out32 = binding.alloc_outputs(desc32)
    with pytest.raises(binding.FipaError) as e:
        binding.forward(desc32, dev32, out32)
    assert e.value.code == binding.FIPA_ERR_UNSUPPORTED


@pytest.mark.parametrize("kw", [dict(d_s=48, B=1, L=130, H=4, trans_scale=0.3),
                                dict(d_s=64, B=2, L=160, H=4, varlen=True, min_len=30, trans_scale=0.5),
                                dict(d_s=256, B=1, L=512, H=4, trans_scale=0.5)])
def test_keep_forward_module(kw):
    # the whole module: forward with the flag in the backward's workspace (d_s = 256 at 512 rows
    # splits the output projection, so its partial products live there too), then backward with it
    import torch
    from oracle import module_ref
    from tests.test_gpu_module import MODULE_GRADS
    m = wl.make_module_inputs(4, **kw)
    d = m["dims"]
    up = torch.from_numpy(np.random.default_rng(5).standard_normal((d["B"], d["L"], m["d_s"])).astype(np.float32)).to("cuda:0")
    desc, dev = binding.upload_module(m)
    plain = binding.alloc_module_grads(desc, m["d_s"])
    binding.module_backward(desc, m["d_s"], dev, up, plain)
    desc.flags = binding.FIPA_FLAG_KEEP_FORWARD
    kept = binding.alloc_module_grads(desc, m["d_s"])
    for n, _ in MODULE_GRADS:
        kept[n].fill_(float("nan"))
    small = dev["workspace"]
    with pytest.raises(binding.FipaError) as e:  # the forward's own workspace is too small for this
        binding.module_forward(desc, m["d_s"], dev)
    assert e.value.code == binding.FIPA_ERR_WORKSPACE and small.numel() < kept["workspace"].numel()
    dev["workspace"] = kept["workspace"]
    dev["workspace"].fill_(0xFF)
    dev["s_out"].fill_(float("nan"))
    binding.module_forward(desc, m["d_s"], dev)
    binding.module_backward(desc, m["d_s"], dev, up, kept)
    torch.cuda.synchronize()
    got = dev["s_out"].cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert gu.rel_err(got, module_ref.module_forward(m)) <= 2e-2
    for n, _ in MODULE_GRADS:
        assert torch.equal(kept[n], plain[n]), (kw, n, float((kept[n].float() - plain[n].float()).abs().max()))
