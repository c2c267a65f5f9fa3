"""fipa_forward_static (the entry point for callers that cannot allocate: scratch memory in an array
of the library's device image instead of a caller workspace) against fipa_forward, through the C
ABI: two calls in a row on the same GPU, the second with a smaller input, must each reproduce
fipa_forward's outputs bit for bit (same kernels, same deterministic merge order)."""
import ctypes

import numpy as np
import pytest

from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl

pytestmark = pytest.mark.gpu

OUT = ("o", "o_pts", "o_pair", "lse")


def _both(inp):
    import torch
    desc, dev = binding.upload(inp)
    ref = binding.alloc_outputs(desc)
    for n in OUT:
        ref[n].fill_(float("nan"))
    binding.forward(desc, dev, ref)
    got = {n: torch.full_like(ref[n], float("nan")) for n in OUT}
    binding.fipa_forward_static(desc, dev["q"], dev["k"], dev["v"], dev["q_pts"], dev["k_pts"], dev["v_pts"],
                                dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"], dev["gamma"], dev["mask"],
                                got["o"], got["o_pts"], got["o_pair"], got["lse"])
    torch.cuda.synchronize()
    return {n: ref[n].cpu().numpy() for n in OUT}, {n: got[n].cpu().numpy() for n in OUT}


def test_static_scratch_matches_workspace_entry_point_on_two_calls():
    # first call: a key-range-split launch (its arrival counters and exchange buffer live in the
    # scratch) on a ragged masked batch; second call: a smaller problem, which finds the first
    # call's contents in the array
    cases = [("bf16 B=3 H=4 L=640 ragged", wl.make_inputs(1, B=3, L=640, H=4, varlen=True, min_len=40)),
             ("bf16 B=1 H=2 L=200", wl.make_inputs(1, B=1, L=200, H=2, cz=32, r=2)),
             ("bf16 r=4 B=1 H=2 L=150", wl.make_inputs(3, B=1, L=150, H=2, varlen=False)),
             ("fp32 B=1 L=64", wl.make_inputs(0))]
    for label, inp in cases:
        ref, got = _both(inp)
        for n in OUT:
            assert np.all(np.isfinite(got[n])), (label, n)
            assert np.array_equal(got[n], ref[n]), (label, n, float(np.abs(got[n] - ref[n]).max()))
        print("static scratch:", label, "identical to fipa_forward", flush=True)


def test_static_scratch_rejects_problems_beyond_its_size():
    desc = binding.make_desc(4, 8192, 12, 16, 4, 8, 128, 4, binding.FIPA_DTYPE_BF16)
    assert binding.workspace_bytes(desc)[0] > binding.STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p(4096)  # any aligned non-null value: the size check comes before any use of it
    rc = binding.lib().fipa_forward_static(ctypes.byref(desc), *([p] * 12), None, p, p, p, None, None)
    assert rc == binding.FIPA_ERR_WORKSPACE
