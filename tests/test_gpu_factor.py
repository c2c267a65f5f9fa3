"""GPU parity of fipa_factor_project (through the C ABI) against oracle/factor_ref.py, alone and as the
chain frames -> k nearest neighbours -> factors -> attention.  Tables are bf16 on both sides; the
kernel sums in float32 and rounds once to bf16, the oracle sums in float64: |gpu - oracle| <=
2^-8 |oracle| (half a bf16 step, with room for a double rounding) + 1e-5 max|oracle| per element."""
import numpy as np
import pytest

from oracle import factor_ref, knn_ref
from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _bf16(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)


def make_tables(rng, k, n_bins, n_pos, n_out, with_bias=True):
    """bf16-rounded tables (torch, host) and their float64 values."""
    e_bin = _bf16(rng.standard_normal((k, n_bins, n_out)) / np.sqrt(k))
    e_pos = None if n_pos == 0 else _bf16(rng.standard_normal((k, n_pos, n_out)) / np.sqrt(k))
    bias = rng.standard_normal(n_out).astype(np.float32) if with_bias else None
    return e_bin, e_pos, bias


def run_gpu(idx, bins, e_bin, e_pos, bias, pos_mode):
    import torch
    B, L, _ = idx.shape
    z = torch.full((B, L, e_bin.shape[2]), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    binding.fipa_factor_project(pos_mode, torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).cuda(),
                                torch.from_numpy(np.ascontiguousarray(bins, dtype=np.int32)).cuda(), e_bin.cuda(),
                                None if e_pos is None else e_pos.cuda(),
                                None if bias is None else torch.from_numpy(bias).cuda(), z)
    torch.cuda.synchronize()
    return z


def check(idx, bins, e_bin, e_pos, bias, pos_mode, label):
    z = run_gpu(idx, bins, e_bin, e_pos, bias, pos_mode).float().cpu().numpy().astype(np.float64)
    want = factor_ref.factor_project(idx, bins, e_bin.float().numpy(), None if e_pos is None else e_pos.float().numpy(),
                                     bias, pos_mode)
    assert np.all(np.isfinite(z)), label
    d = np.abs(z - want)
    bound = 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(want).max()
    print(label, "max |d| %.2e, worst d / bound %.2f" % (d.max(), (d / bound).max()), flush=True)
    assert np.all(d <= bound), (label, float((d / bound).max()))


@pytest.mark.parametrize("kw", [dict(B=2, L=77, k=20, n_bins=16, n_pos=65, n_out=256, pos_mode=1),
                                dict(B=1, L=300, k=20, n_bins=16, n_pos=33, n_out=512, pos_mode=0),
                                dict(B=3, L=50, k=7, n_bins=5, n_pos=0, n_out=8, pos_mode=1),
                                dict(B=1, L=130, k=64, n_bins=64, n_pos=129, n_out=1024, pos_mode=1),
                                dict(B=2, L=40, k=1, n_bins=1, n_pos=1, n_out=32, pos_mode=1)])
def test_random_neighbour_lists(kw):
    rng = np.random.default_rng(100 + kw["L"])
    B, L, k = kw["B"], kw["L"], kw["k"]
    idx = rng.integers(0, L, size=(B, L, k))
    idx[rng.random((B, L, k)) < 0.15] = -1
    idx[0, 3] = -1  # a residue without neighbours
    bins = rng.integers(0, kw["n_bins"], size=(B, L, k))
    bins[idx < 0] = -1
    e_bin, e_pos, bias = make_tables(rng, k, kw["n_bins"], kw["n_pos"], kw["n_out"], with_bias=kw["n_out"] != 8)
    check(idx, bins, e_bin, e_pos, bias, kw["pos_mode"], "factors %s" % kw)


def test_from_frames_to_attention():
    # frames -> k nearest neighbours -> z1, z2 -> attention, every step on the GPU, against the same
    # chain of oracles; the neighbour lists are bit-exact, so both sides project the same features
    import torch
    inp = wl.make_inputs(1, B=2, L=200, H=2, varlen=True, min_len=60)
    d = inp["dims"]
    k, n_bins, n_pos, n_out = 20, 16, 65, d["r"] * d["cz"]
    rng = np.random.default_rng(77)
    t1, t2 = make_tables(rng, k, n_bins, n_pos, n_out), make_tables(rng, k, n_bins, n_pos, n_out)
    desc, dev = binding.upload(inp)
    idx = torch.empty(d["B"], d["L"], k, dtype=torch.int32, device="cuda:0")
    d2 = torch.empty(d["B"], d["L"], k, dtype=torch.float32, device="cuda:0")
    bins = torch.empty_like(idx)
    binding.fipa_knn_distogram(k, n_bins, 2.0, 22.0, dev["trans"], dev["mask"], idx, d2, bins)
    for name, (e_bin, e_pos, bias) in (("z1", t1), ("z2", t2)):
        z = torch.empty(d["B"], d["L"], n_out, dtype=torch.bfloat16, device="cuda:0")
        binding.fipa_factor_project(1, idx, bins, e_bin.cuda(), e_pos.cuda(), torch.from_numpy(bias).cuda(), z)
        dev[name] = z.view(d["B"], d["L"], d["r"], d["cz"])
    out = binding.alloc_outputs(desc)
    binding.forward(desc, dev, out)
    torch.cuda.synchronize()
    o_idx, _, o_bins = knn_ref.knn_distogram(inp["trans"], inp["mask"], k, n_bins, 2.0, 22.0)
    assert np.array_equal(idx.cpu().numpy(), o_idx) and np.array_equal(bins.cpu().numpy(), o_bins)
    ref = dict(inp)
    for name, (e_bin, e_pos, bias) in (("z1", t1), ("z2", t2)):
        z = factor_ref.factor_project(o_idx, o_bins, e_bin.float().numpy(), e_pos.float().numpy(), bias, 1)
        # (the attention's inputs are bf16: the oracle gets the factors rounded as the kernel rounds them)
        ref[name] = _bf16(z).float().numpy().reshape(d["B"], d["L"], d["r"], d["cz"])
    want = gu.oracle_forward_chunked(ref)
    for n in gu.NAMES:
        err = gu.rel_err(out[n].cpu().numpy().astype(np.float64), want[n])
        print("frames -> attention", n, "%.2e" % err, flush=True)
        assert err <= gu.TOL["bf16"], (n, err)


def test_workload3_size_timed():
    # four chains of up to 8192 residues, k = 20, 16 bins, offsets to +-32, r c_z = 512: every row
    import torch
    inp = wl.make_inputs(3)
    d = inp["dims"]
    k, n_bins, n_pos, n_out = 20, 16, 65, d["r"] * d["cz"]
    rng = np.random.default_rng(78)
    e_bin, e_pos, bias = make_tables(rng, k, n_bins, n_pos, n_out)
    trans = torch.from_numpy(inp["trans"]).cuda()
    mask = torch.from_numpy(inp["mask"]).cuda()
    idx = torch.empty(d["B"], d["L"], k, dtype=torch.int32, device="cuda:0")
    d2 = torch.empty(d["B"], d["L"], k, dtype=torch.float32, device="cuda:0")
    bins = torch.empty_like(idx)
    binding.fipa_knn_distogram(k, n_bins, 2.0, 22.0, trans, mask, idx, d2, bins)
    z = torch.full((d["B"], d["L"], n_out), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    g = [e_bin.cuda(), e_pos.cuda(), torch.from_numpy(bias).cuda()]
    binding.fipa_factor_project(1, idx, bins, *g, z)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        binding.fipa_factor_project(1, idx, bins, *g, z)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    rows = d["B"] * d["L"]
    print("factor projection B=%d L=%d n_out=%d: %.3f ms per call; %.0f GB/s of output + index bytes, %.2f TB/s of table rows"
          % (d["B"], d["L"], n_out, ms, rows * (n_out * 2 + 8 * k) / ms / 1e6, rows * 2.0 * k * n_out * 2 / ms / 1e9), flush=True)
    want = factor_ref.factor_project(idx.cpu().numpy(), bins.cpu().numpy(), e_bin.float().numpy(), e_pos.float().numpy(), bias, 1)
    dd = np.abs(z.float().cpu().numpy().astype(np.float64) - want)
    assert np.all(dd <= 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(want).max()), float(dd.max())


@pytest.mark.parametrize("kw", [dict(B=2, L=77, k=20, n_bins=16, n_pos=65, n_out=256, pos_mode=1),
                                dict(B=1, L=300, k=20, n_bins=16, n_pos=33, n_out=512, pos_mode=0),
                                dict(B=3, L=50, k=7, n_bins=5, n_pos=0, n_out=8, pos_mode=1),
                                dict(B=1, L=130, k=64, n_bins=30, n_pos=129, n_out=136, pos_mode=1),
                                dict(B=2, L=40, k=1, n_bins=1, n_pos=1, n_out=32, pos_mode=1),
                                dict(B=1, L=90, k=3, n_bins=64, n_pos=95, n_out=64, pos_mode=1)])
def test_table_gradients(kw):
    # (the last two shapes: a single table row that every residue hits; the tallest tables the call takes,
    # five blocks of 32 rows)
    import torch
    rng = np.random.default_rng(200 + kw["L"])
    B, L, k, n_bins, n_pos, n_out = kw["B"], kw["L"], kw["k"], kw["n_bins"], kw["n_pos"], kw["n_out"]
    idx = rng.integers(0, L, size=(B, L, k))
    idx[rng.random((B, L, k)) < 0.15] = -1
    bins = rng.integers(0, n_bins, size=(B, L, k))
    bins[idx < 0] = -1
    mask = (rng.random((B, L)) > 0.2).astype(np.uint8)
    d_z = _bf16(rng.standard_normal((B, L, n_out)))
    f = dict(dtype=torch.float32, device="cuda:0")
    g_bin = torch.full((k, n_bins, n_out), float("nan"), **f)
    g_pos = None if n_pos == 0 else torch.full((k, n_pos, n_out), float("nan"), **f)
    g_bias = torch.full((n_out,), float("nan"), **f)
    args = (kw["pos_mode"], torch.from_numpy(idx.astype(np.int32)).cuda(), torch.from_numpy(bins.astype(np.int32)).cuda(),
            d_z.cuda(), torch.from_numpy(mask).cuda())
    binding.fipa_factor_project_backward(*args, g_bin, g_pos, g_bias)
    torch.cuda.synchronize()
    first = [t.clone() for t in (g_bin, g_pos, g_bias) if t is not None]
    w_bin, w_pos, w_bias = factor_ref.factor_project_backward(idx, bins, d_z.float().numpy(), n_bins, n_pos, kw["pos_mode"], mask)
    # float32 sums of up to B L bf16 values against float64 sums: a few 1e-7 of the sum of magnitudes
    scale = float(np.abs(d_z.float().numpy()).sum(axis=(0, 1)).max())
    for got, want, name in ((g_bin, w_bin, "d_e_bin"), (g_pos, w_pos, "d_e_pos"), (g_bias, w_bias, "d_bias")):
        if got is None:
            continue
        g = got.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(g)), (kw, name)
        assert np.abs(g - want).max() <= 2e-6 * scale, (kw, name, float(np.abs(g - want).max()), scale)
    # the same bits on a second run
    for t in (g_bin, g_pos, g_bias):
        if t is not None:
            t.fill_(float("nan"))
    binding.fipa_factor_project_backward(*args, g_bin, g_pos, g_bias)
    torch.cuda.synchronize()
    for a, b in zip(first, [t for t in (g_bin, g_pos, g_bias) if t is not None]):
        assert torch.equal(a, b), kw


def test_table_gradients_workload3_size_timed():
    import torch
    B, L, k, n_bins, n_pos, n_out = 4, 8192, 20, 16, 65, 512
    rng = np.random.default_rng(300)
    idx = np.clip(np.arange(L)[None, :, None] + rng.integers(-40, 41, size=(B, L, k)), 0, L - 1)  # near neighbours along the chain
    bins = np.minimum(rng.geometric(0.25, size=(B, L, k)) - 1, n_bins - 1)                        # low bins much more often
    d_z = _bf16(rng.standard_normal((B, L, n_out)))
    f = dict(dtype=torch.float32, device="cuda:0")
    g_bin, g_pos, g_bias = torch.empty(k, n_bins, n_out, **f), torch.empty(k, n_pos, n_out, **f), torch.empty(n_out, **f)
    args = (1, torch.from_numpy(idx.astype(np.int32)).cuda(), torch.from_numpy(bins.astype(np.int32)).cuda(), d_z.cuda(), None)
    binding.fipa_factor_project_backward(*args, g_bin, g_pos, g_bias)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        binding.fipa_factor_project_backward(*args, g_bin, g_pos, g_bias)
    e1.record()
    torch.cuda.synchronize()
    print("factor projection backward B=%d L=%d n_out=%d: %.3f ms per call" % (B, L, n_out, e0.elapsed_time(e1) / 10), flush=True)
    w_bin, w_pos, w_bias = factor_ref.factor_project_backward(idx, bins, d_z.float().numpy(), n_bins, n_pos, 1)
    scale = float(np.abs(d_z.float().numpy()).sum(axis=(0, 1)).max())
    for got, want in ((g_bin, w_bin), (g_pos, w_pos), (g_bias, w_bias)):
        assert np.abs(got.cpu().numpy().astype(np.float64) - want).max() <= 2e-6 * scale
