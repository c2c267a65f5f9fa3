"""Seeded sweep over shapes the fixed cases do not hit: batch, length, heads, pair width and rank
drawn at random (ragged tails, lengths below one tile, prefix masks, spread or compact geometry),
forward and backward through the C ABI against the oracle, same tolerances as the fixed cases."""
import numpy as np
import pytest

from paper_2505_11580_amd import workloads as wl
from tests import gpu_util as gu
from tests.test_gpu_backward import check_backward

pytestmark = pytest.mark.gpu


def draw_shape(rng, max_len, wide_ok):
    # r * c_z must be one of the lifted pair widths the bf16 path has kernels for
    choices = [(8, 4), (16, 2), (32, 1), (32, 2), (16, 4), (64, 2), (32, 4), (128, 1), (128, 2), (64, 4), (32, 8)]
    if wide_ok:
        choices.append((128, 4))
    cz, r = choices[int(rng.integers(len(choices)))]
    return dict(B=int(rng.integers(1, 4)), L=int(rng.integers(1, max_len + 1)), H=int(rng.integers(1, 6)), cz=cz, r=r,
                varlen=bool(rng.integers(2)), min_len=1,
                trans_scale=float(rng.choice([1.0, 0.3, 0.05])))


@pytest.mark.parametrize("seed", range(10))
def test_forward_random_shape(seed):
    rng = np.random.default_rng(7000 + seed)
    kw = draw_shape(rng, 420, wide_ok=True)
    ts = kw.pop("trans_scale")
    inp = wl.make_inputs(1, seed=9000 + seed, trans_scale=ts, **kw)
    gu.check(inp, label="fwd random %s scale=%g lengths=%s" % (kw, ts, list(inp["lengths"])))


@pytest.mark.parametrize("seed", range(6))
def test_backward_random_shape(seed):
    rng = np.random.default_rng(7100 + seed)
    kw = draw_shape(rng, 200, wide_ok=False)
    ts = kw.pop("trans_scale")
    inp = wl.make_inputs(4, seed=9100 + seed, trans_scale=ts, **kw)
    check_backward(inp, "bwd random %s scale=%g lengths=%s" % (kw, ts, list(inp["lengths"])))
