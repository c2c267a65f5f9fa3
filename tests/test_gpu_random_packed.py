"""Seeded random sweep over the widths, ranks, head counts and chain-length mixes of the packed forward
(one set of launches, or chain after chain where the library picks that), against the oracle's padded,
masked result; and of the backward at the widths that have one."""
import numpy as np
import pytest

from oracle import ipa_oracle
from paper_2505_11580_amd import binding
from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu
from tests.test_gpu_backward import GRADS
from tests.test_gpu_packed import _pack, check_packed_forward, packed_backward

pytestmark = pytest.mark.gpu

WIDTHS = [(16, 2), (32, 2), (64, 1), (128, 1), (128, 2), (64, 8), (128, 4), (128, 8), (256, 4)]  # (c_z, r)


@pytest.mark.parametrize("seed", range(6))
def test_random_packed_forward(seed):
    rng = np.random.default_rng(1000 + seed)
    cz, r = WIDTHS[int(rng.integers(len(WIDTHS)))]
    B, H = int(rng.integers(1, 7)), int(rng.integers(1, 5))
    L = int(rng.integers(40, 420))
    inp = wl.make_inputs(1, B=B, L=L, H=H, cz=cz, r=r, varlen=True, min_len=int(rng.integers(1, L // 2 + 1)),
                         trans_scale=float(rng.choice([1.0, 0.3, 0.05])), seed=2000 + seed)
    check_packed_forward(inp, "random packed seed %d: B=%d L=%d H=%d cz=%d r=%d" % (seed, B, L, H, cz, r))


@pytest.mark.parametrize("seed", range(4))
def test_random_packed_backward(seed):
    rng = np.random.default_rng(3000 + seed)
    cz, r = [(32, 2), (128, 1), (128, 2), (128, 4)][seed]
    B, H = int(rng.integers(1, 5)), int(rng.integers(1, 4))
    L = int(rng.integers(40, 260))
    inp = wl.make_inputs(4, B=B, L=L, H=H, cz=cz, r=r, varlen=True, min_len=int(rng.integers(8, L // 2 + 1)),
                         trans_scale=float(rng.choice([1.0, 0.3])), seed=4000 + seed)
    want = ipa_oracle.backward(inp, inp["d_o"], inp["d_o_pts"], inp["d_o_pair"])
    got, lengths = packed_backward(inp)
    floor = 1e-3 * float(np.abs(want["dv"]).max())
    errs = {}
    for n, o in GRADS:
        w = want[o] if n in ("d_gamma", "d_w_b") else _pack(want[o], lengths)
        errs[n] = float(np.abs(got[n] - w).max()) / max(float(np.abs(w).max()), floor)
    print("random packed backward seed %d: B=%d L=%d H=%d cz=%d r=%d lengths %s" % (seed, B, L, H, cz, r, lengths),
          {k: "%.1e" % v for k, v in errs.items()}, flush=True)
    # d_gamma is one number per head, -(w_L w_C / 2) sum_ij dS_ij D_ij with sum_j dS_ij = 0: a sum that cancels
    # by construction, so its error relative to its own (small) value can exceed that of the other gradients
    # when there is a single head and a short chain; it is held to 5e-2 here and to 2e-2 at the named workloads
    for n, _ in GRADS:
        assert errs[n] <= (5e-2 if n == "d_gamma" else 2e-2), (n, errs[n])
