"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle."""
import numpy as np

from oracle import ipa_oracle
from paper_2505_11580_amd import binding

NAMES = ("o", "o_pts", "o_pair")
TOL = {"fp32": 1e-4, "bf16": 2e-2}  # max|gpu - oracle| / max|oracle| per output tensor


def run_gpu(inp, flags=0):
    import torch
    desc, dev = binding.upload(inp)
    desc.flags = flags
    out = binding.alloc_outputs(desc)
    for n in NAMES:
        out[n].fill_(float("nan"))  # every element must be overwritten
    binding.forward(desc, dev, out)
    torch.cuda.synchronize()
    res = {n: out[n].cpu().numpy().astype(np.float64) for n in NAMES}
    res["lse"] = out["lse"].cpu().numpy().astype(np.float64)
    return res


def rel_err(got, want):
    scale = max(float(np.abs(want).max()), 1e-30)
    return float(np.abs(got - want).max()) / scale


def elem_err(got, want):
    """Second, element-wise figure (reported, not gated): max |d| / (|oracle| + 1e-3 max|oracle|), which
    also sees errors on entries that are small next to the tensor's largest."""
    scale = max(float(np.abs(want).max()), 1e-30)
    return float((np.abs(got - want) / (np.abs(want) + 1e-3 * scale)).max())


def oracle_forward_chunked(inp, rows=None, chunk=512):
    """ipa_oracle.forward over all rows (or the given rows) in chunks of query rows, so that the
    dense pair rows of one chunk (chunk x L x c_z doubles per batch element) stay small."""
    B, L = inp["q"].shape[:2]
    if rows is None:
        rows = [np.arange(L, dtype=np.int32)] * B
    n = len(rows[0])
    parts = [ipa_oracle.forward(inp, rows=[r[s0:s0 + chunk] for r in rows]) for s0 in range(0, n, chunk)]
    return {k: np.concatenate([p[k] for p in parts], axis=1) for k in NAMES}


def check(inp, rows=None, tol=None, label="", chunk=512, flags=0):
    """Compare the HIP path with the oracle (all rows, or the given row lists); `flags` goes into
    the description's flags field (FIPA_FLAG_* bits)."""
    tol = TOL[inp["dtype"]] if tol is None else tol
    got = run_gpu(inp, flags=flags)
    want = oracle_forward_chunked(inp, rows=rows, chunk=chunk)
    errs, elem = {}, {}
    for n in NAMES:
        g = got[n]
        assert np.all(np.isfinite(g)), (label, n, "non-finite output")
        if rows is not None:
            g = np.stack([g[b][rows[b]] for b in range(g.shape[0])])
        errs[n] = rel_err(g, want[n])
        elem[n] = elem_err(g, want[n])
    print(label, "max-norm", {k: "%.2e" % v for k, v in errs.items()},
          "element-wise", {k: "%.2e" % v for k, v in elem.items()}, flush=True)
    for n in NAMES:
        assert errs[n] <= tol, (label, n, errs[n], tol)
    return errs
