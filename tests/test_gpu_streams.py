"""Calls from two host threads on two streams at once, each with its own tensors and workspace: the
library keeps no state between calls (apart from per-kernel set-up done once per device), so every
result must be the very bits the same calls give one after the other on one stream."""
import threading

import pytest

from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests.test_gpu_backward import GRADS

pytestmark = pytest.mark.gpu

NAMES = ("o", "o_pts", "o_pair", "lse")


def _job(kw):
    inp = wl.make_inputs(4, **kw)
    desc, dev = binding.upload(inp)
    return desc, dev, binding.alloc_outputs(desc), binding.alloc_grads(desc)


def _run(job, reps):
    desc, dev, out, grads = job
    for _ in range(reps):
        binding.forward(desc, dev, out)
        binding.backward(desc, dev, out, grads)


def test_two_threads_two_streams():
    import torch
    jobs = [_job(dict(B=2, L=640, H=6, varlen=True, min_len=200, trans_scale=0.5)),   # takes the key-range split
            _job(dict(B=1, L=500, H=4, cz=128, r=4, trans_scale=0.5))]                 # the windowed kernels
    want = []
    for job in jobs:
        _run(job, 1)
        torch.cuda.synchronize()
        want.append(({n: job[2][n].clone() for n in NAMES}, {n: job[3][n].clone() for n, _ in GRADS}))
        for n in NAMES:
            job[2][n].fill_(float("nan"))
        for n, _ in GRADS:
            job[3][n].fill_(float("nan"))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def worker(job, stream):
        try:
            with torch.cuda.stream(stream):
                _run(job, 20)
            stream.synchronize()
        except Exception as e:  # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(j, s)) for j, s in zip(jobs, streams)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for job, (w_out, w_grad) in zip(jobs, want):
        for n in NAMES:
            assert torch.equal(job[2][n], w_out[n]), n
        for n, _ in GRADS:
            assert torch.equal(job[3][n], w_grad[n]), n
