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


# Head shapes other than the AlphaFold2 one (c = 16, N_query = 4, N_value = 8): these take the generic
# chain -- separate preparation launch, generic pack kernels, per-head query-side factor copy, unfused
# attention and the stand-alone epilogue kernel (including the value-point column layout for an odd
# number of value points).
HEAD_SHAPES = [dict(c=8, Pq=2, Pv=3), dict(c=32, Pq=2, Pv=4), dict(c=24, Pq=3, Pv=5), dict(c=16, Pq=1, Pv=2),
               dict(c=8, Pq=4, Pv=7), dict(c=16, Pq=4, Pv=7), dict(c=16, Pq=3, Pv=8)]


@pytest.mark.parametrize("shape", HEAD_SHAPES, ids=lambda d: "c%d_Pq%d_Pv%d" % (d["c"], d["Pq"], d["Pv"]))
def test_forward_generic_head_shapes(shape):
    lab = "fwd head shape %s" % shape
    gu.check(wl.make_inputs(1, B=2, L=203, H=3, cz=32, r=2, varlen=True, min_len=30, trans_scale=0.3, **shape),
             label=lab + " ragged, masked")
    gu.check(wl.make_inputs(1, B=1, L=160, H=2, cz=128, r=2, **shape), label=lab + " DZ=256")
    gu.check(wl.make_inputs(3, B=1, L=150, H=2, varlen=False, trans_scale=0.2, **shape), label=lab + " r=4")


@pytest.mark.parametrize("shape", [HEAD_SHAPES[0], HEAD_SHAPES[2], HEAD_SHAPES[5]],
                         ids=lambda d: "c%d_Pq%d_Pv%d" % (d["c"], d["Pq"], d["Pv"]))
def test_backward_generic_head_shapes(shape):
    check_backward(wl.make_inputs(4, B=2, L=150, H=2, cz=32, r=2, varlen=True, min_len=20, trans_scale=0.3, **shape),
                   "bwd head shape %s ragged, masked" % shape)
