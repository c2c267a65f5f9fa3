"""GPU parity of fipa_knn_distogram (through the C ABI) against oracle/knn_ref.py: neighbour indices,
squared distances and bins are integer / same-precision decisions, so the comparison is bit-exact."""
import numpy as np
import pytest

from oracle import knn_ref
from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_gpu(trans, mask, k, n_bins, d_min, d_max, time_it=False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(trans, dtype=np.float32)).cuda()
    m = None if mask is None else torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).cuda()
    B, L = t.shape[:2]
    idx = torch.full((B, L, k), -7, dtype=torch.int32, device="cuda:0")
    d2 = torch.full((B, L, k), float("nan"), dtype=torch.float32, device="cuda:0")
    bins = torch.full((B, L, k), -7, dtype=torch.int32, device="cuda:0")
    binding.fipa_knn_distogram(k, n_bins, d_min, d_max, t, m, idx, d2, bins)
    torch.cuda.synchronize()
    ms = None
    if time_it:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            binding.fipa_knn_distogram(k, n_bins, d_min, d_max, t, m, idx, d2, bins)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
    return idx.cpu().numpy(), d2.cpu().numpy(), bins.cpu().numpy(), ms


def check(trans, mask, k, n_bins, d_min, d_max, label, time_it=False):
    got = run_gpu(trans, mask, k, n_bins, d_min, d_max, time_it)
    want = knn_ref.knn_distogram(trans, mask, k, n_bins, d_min, d_max)
    for name, g, w in zip(("idx", "d2", "bins"), got, want):
        assert np.array_equal(g, w), (label, name, int((g != w).sum()))
    if time_it:
        print(label, "%.3f ms per call" % got[3], flush=True)


def test_chain_geometry_with_and_without_mask():
    inp = wl.make_inputs(1, B=3, L=300, H=1, varlen=True, min_len=25)
    check(inp["trans"], None, 20, 16, 2.0, 22.0, "knn chain")
    check(inp["trans"], inp["mask"], 20, 16, 2.0, 22.0, "knn chain masked")  # padded slots hold 1e3 garbage
    check(inp["trans"], inp["mask"], 64, 64, 0.0, 50.0, "knn k=64")
    check(inp["trans"], inp["mask"], 1, 2, 3.0, 4.0, "knn k=1")


def test_ties_on_a_lattice_and_short_chains():
    rng = np.random.default_rng(5)
    trans = rng.integers(-3, 4, size=(2, 150, 3)).astype(np.float32)  # many equal distances, coincident points
    mask = (rng.random((2, 150)) > 0.3).astype(np.uint8)
    check(trans, mask, 20, 8, 1.0, 6.0, "knn lattice")
    check(trans[:, :7], mask[:, :7], 20, 8, 1.0, 6.0, "knn L=7 < k")
    check(trans[:, :1], None, 5, 8, 1.0, 6.0, "knn L=1")
    none = np.zeros((2, 150), dtype=np.uint8)
    none[1, 17] = 1  # one element without valid residues, one with a single valid residue
    check(trans, none, 4, 8, 1.0, 6.0, "knn nearly empty")


def test_workload3_geometry_full_size():
    # four ragged chains of up to 8192 residues (the long-chain workload's frames), every row compared
    inp = wl.make_inputs(3)
    check(inp["trans"], inp["mask"], 20, 16, 2.0, 22.0, "knn workload 3 (B=4, L=8192, k=20)", time_it=True)
