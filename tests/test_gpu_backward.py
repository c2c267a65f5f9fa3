"""GPU parity of fipa_backward (through the C ABI) against the oracle's analytic gradients (which
are themselves pinned by finite differences), bf16 inputs / fp32 accumulation: per gradient
tensor max|gpu - oracle| / max|oracle| <= 2e-2."""
import numpy as np
import pytest

from oracle import ipa_oracle
from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

GRADS = (("d_q", "dq"), ("d_k", "dk"), ("d_v", "dv"), ("d_q_pts", "dq_pts"), ("d_k_pts", "dk_pts"),
         ("d_v_pts", "dv_pts"), ("d_z1", "dz1"), ("d_z2", "dz2"), ("d_gamma", "dgamma"), ("d_w_b", "dw_b"),
         ("d_rot", "drot"), ("d_trans", "dtrans"))


def run_gpu_backward(inp):
    import torch
    desc, dev = binding.upload(inp)
    out = binding.alloc_outputs(desc)
    binding.forward(desc, dev, out)
    grads = binding.alloc_grads(desc)
    for n, _ in GRADS:
        grads[n].fill_(float("nan"))
    binding.backward(desc, dev, out, grads)
    torch.cuda.synchronize()
    return {n: grads[n].float().cpu().numpy().astype(np.float64) for n, _ in GRADS}


def check_backward(inp, label, tol=2e-2, samples=None):
    """All gradients against the oracle: every element (dense oracle backward), or -- at sizes the
    dense pair tensor does not fit -- the gradients of the sampled residues (one index array per
    batch element) from the oracle's row-walking backward, plus the full d_gamma and d_w_b."""
    got = run_gpu_backward(inp)
    if samples is None:
        want = ipa_oracle.backward(inp, inp["d_o"], inp["d_o_pts"], inp["d_o_pair"])
    else:
        want = ipa_oracle.backward_sampled(inp, inp["d_o"], inp["d_o_pts"], inp["d_o_pair"], samples)
        for n, _ in GRADS:
            if n not in ("d_gamma", "d_w_b"):
                got[n] = np.stack([got[n][b][samples[b]] for b in range(len(samples))])
    errs, elem = {}, {}
    # a gradient that is exactly zero in the oracle (a single key: constant softmax) is measured
    # against the scale of the value gradient instead of its own
    floor = 1e-3 * float(np.abs(want["dv"]).max())
    for n, o in GRADS:
        assert np.all(np.isfinite(got[n])), (label, n)
        errs[n] = float(np.abs(got[n] - want[o]).max()) / max(float(np.abs(want[o]).max()), floor)
        elem[n] = gu.elem_err(got[n], want[o])
    print(label, "max-norm", {k: "%.1e" % v for k, v in errs.items()},
          "element-wise", {k: "%.1e" % v for k, v in elem.items()}, flush=True)
    for n, _ in GRADS:
        assert errs[n] <= tol, (label, n, errs[n])


def test_backward_workload4_slice_l128():
    # the forward+backward workload's generators on an L = 128 slice
    check_backward(wl.make_inputs(4, B=2, L=128), "cfg4 slice L=128")


def test_backward_spread_and_ragged():
    check_backward(wl.make_inputs(4, B=1, L=160, H=4, trans_scale=0.1), "bwd spread L=160")
    check_backward(wl.make_inputs(4, B=1, L=96, H=3, cz=16, r=2, trans_scale=0.3), "bwd DZ=32 L=96")


def test_backward_masked():
    inp = wl.make_inputs(4, B=2, L=192, H=3, varlen=True, min_len=40, trans_scale=0.5)
    check_backward(inp, "bwd varlen")
    got = run_gpu_backward(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in ("d_q", "d_k", "d_v", "d_q_pts", "d_k_pts", "d_v_pts", "d_z1", "d_z2"):
            assert np.all(got[n][b, int(ln):] == 0), (n, b)


def test_backward_masked_odd_pair_count():
    # 5 x 3 = 15 (batch, head) pairs, ragged: the gradient kernels renumber the pairs of a masked batch
    check_backward(wl.make_inputs(4, B=5, L=140, H=3, cz=32, varlen=True, min_len=10, trans_scale=0.5), "bwd varlen B=5 H=3")


@pytest.mark.parametrize("kw", [dict(B=1, L=128, H=2), dict(B=2, L=300, H=2, varlen=True, min_len=40, trans_scale=0.3),
                                dict(B=1, L=200, H=3, cz=256, r=2, trans_scale=0.5), dict(B=2, L=160, H=2, c=8, Pq=2, Pv=3, varlen=True, min_len=30)])
def test_backward_rank4_width512(kw):
    # r*c_z = 512 (the rank-4 workload's head shape): three windows of output columns per tile of stationary
    # rows, queries streamed through two LDS stages; all twelve gradients against the oracle
    check_backward(wl.make_inputs(3, with_grads=True, **{"varlen": False, **kw}), "bwd width 512 %s" % kw)


def test_backward_rank4_ragged_l2048_sampled():
    # the rank-4 workload's generators at B=2, L<=2048 (ragged, masked): many streamed blocks and tiles per
    # chain, gradients of 128 sampled residues per chain and the full d_gamma, d_w_b against the row-walking oracle
    inp = wl.make_inputs(3, B=2, L=2048, H=4, min_len=700, with_grads=True)
    check_backward(inp, "bwd width 512 ragged L<=2048, 128 sampled residues", samples=wl.select_rows(inp, 128))


def test_backward_workload4_full_size_sampled():
    # workload 4 at full size (B=2, L=4096): the gradients of 256 residues per batch element (first,
    # last, one in every 128-row tile, the rest random; each both as query row and as key column)
    # and the full d_gamma, d_w_b against the oracle's row-walking backward
    inp = wl.make_inputs(4)
    check_backward(inp, "cfg4 full size, 256 sampled residues", samples=wl.select_rows(inp, 256))


def test_backward_full_size_properties():
    # workload 4 at full size (B=2, L=4096): the oracle cannot sweep it; check properties that hold
    # at any size: finite, linear in the upstream gradient, and local-frame gradients unchanged
    # under a global rotation + translation of all frames.
    inp = wl.make_inputs(4)
    g1 = run_gpu_backward(inp)
    for n, _ in GRADS:
        assert np.all(np.isfinite(g1[n])), n
    twice = dict(inp)
    for n in ("d_o", "d_o_pts", "d_o_pair"):
        twice[n] = 2.0 * inp[n]
    g2 = run_gpu_backward(twice)
    for n, _ in GRADS:
        assert gu.rel_err(g2[n], 2.0 * g1[n]) <= 2e-2, n
    rng = np.random.default_rng(3)
    Rg = wl.random_rotations(rng, ()).astype(np.float32)
    tg = (20.0 * rng.standard_normal(3)).astype(np.float32)
    moved = dict(inp)
    moved["rot"] = np.einsum("xy,blyz->blxz", Rg, inp["rot"]).astype(np.float32)
    moved["trans"] = (np.einsum("xy,bly->blx", Rg, inp["trans"]) + tg).astype(np.float32)
    g3 = run_gpu_backward(moved)
    # the frame gradients are global-frame objects: they turn with the global rotation
    g3["d_rot"] = np.einsum("yx,blyz->blxz", Rg.astype(np.float64), g3["d_rot"])
    g3["d_trans"] = np.einsum("yx,bly->blx", Rg.astype(np.float64), g3["d_trans"])
    for n, _ in GRADS:
        assert gu.rel_err(g3[n], g1[n]) <= 2e-2, n
    # a common shift of all frames changes nothing: the translation gradients of a chain sum to zero
    # (up to the rounding noise of L independent terms)
    L = g1["d_trans"].shape[1]
    assert np.abs(g1["d_trans"].sum(axis=1)).max() <= 2e-2 * np.abs(g1["d_trans"]).max() * np.sqrt(L)


def test_backward_degenerate_shapes():
    check_backward(wl.make_inputs(4, B=1, L=1, H=1), "bwd L=1 H=1")
    check_backward(wl.make_inputs(4, B=2, L=40, H=2, cz=16, r=2, trans_scale=0.2), "bwd L=40 DZ=32")
