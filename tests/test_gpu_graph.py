"""The allocation-free forward and the one-launch packed forward under HIP graph capture: the calls
enqueue kernels only (no allocation, no host-device copy, no synchronisation), so a captured graph must
replay to the eager result every time, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl

pytestmark = pytest.mark.gpu

NAMES = ("o", "o_pts", "o_pair", "lse")


def _replay_and_compare(enqueue, outs, label):
    import torch
    enqueue()  # eager: also the first call on this device (per-device set-up happens outside the capture)
    torch.cuda.synchronize()
    want = {n: outs[n].clone() for n in NAMES}
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        enqueue()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for rep in range(4):
        for n in NAMES:
            outs[n].fill_(float("nan"))
        scratch.add_(1.0)  # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in NAMES:
            assert torch.equal(outs[n], want[n]), (label, rep, n)


@pytest.mark.parametrize("kw", [dict(B=2, L=300, H=3), dict(B=3, L=640, H=8, varlen=True, min_len=100)])
def test_static_forward_replays_from_a_graph(kw):
    # the second shape takes the key-range split (its counters are cleared by a kernel, not a memset)
    inp = wl.make_inputs(1, **kw)
    desc, dev = binding.upload(inp)
    out = binding.alloc_outputs(desc)

    def enqueue():
        binding.fipa_forward_static(desc, dev["q"], dev["k"], dev["v"], dev["q_pts"], dev["k_pts"], dev["v_pts"],
                                    dev["rot"], dev["trans"], dev["z1"], dev["z2"], dev["w_b"], dev["gamma"], dev["mask"],
                                    out["o"], out["o_pts"], out["o_pair"], out["lse"])

    _replay_and_compare(enqueue, out, "static %s" % kw)


def test_packed_forward_replays_from_a_graph():
    import torch
    inp = wl.make_inputs(1, B=6, L=400, H=4, varlen=True, min_len=60)
    desc, dev = binding.upload(inp)
    lengths = [int(x) for x in inp["lengths"]]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    names = ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans", "z1", "z2")
    pk = {n: torch.cat([dev[n][b, :ln] for b, ln in enumerate(lengths)], dim=0).contiguous() for n in names}
    total, H = int(cu[-1]), desc.H
    f = dict(dtype=torch.float32, device="cuda:0")
    out = dict(o=torch.empty(total, H, desc.c, **f), o_pts=torch.empty(total, H, desc.Pv, 3, **f),
               o_pair=torch.empty(total, H, desc.cz, **f), lse=torch.empty(H * total, **f))
    ws = torch.empty(binding.packed_workspace_bytes(desc, cu)[0], dtype=torch.uint8, device="cuda:0")

    def enqueue():
        binding.fipa_forward_packed(desc, cu, *[pk[n] for n in names], dev["w_b"], dev["gamma"], None,
                                    out["o"], out["o_pts"], out["o_pair"], out["lse"], ws)

    _replay_and_compare(enqueue, out, "packed")


def test_training_step_replays_from_a_graph():
    # forward (keeping its lifted state in the backward's workspace) and backward captured as one graph:
    # every replay must give the eager step's outputs and gradients, with the workspace scribbled over
    # between the replays (nothing in it may be expected to survive from one step to the next)
    import torch
    from tests.test_gpu_backward import GRADS
    inp = wl.make_inputs(4, B=2, L=300, H=3, varlen=True, min_len=80, trans_scale=0.5)
    desc, dev = binding.upload(inp)
    desc.flags = binding.FIPA_FLAG_KEEP_FORWARD
    out = binding.alloc_outputs(desc)
    grads = binding.alloc_grads(desc)
    out["workspace"] = grads["workspace"]
    names = [(out, n) for n in NAMES] + [(grads, n) for n, _ in GRADS]

    def enqueue():
        binding.forward(desc, dev, out)
        binding.backward(desc, dev, out, grads)

    enqueue()
    torch.cuda.synchronize()
    want = [d[n].clone() for d, n in names]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        enqueue()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(3):
        for d, n in names:
            d[n].fill_(float("nan"))
        grads["workspace"].fill_(0xFF)  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (d, n), w in zip(names, want):
            assert torch.equal(d[n], w), (rep, n)
