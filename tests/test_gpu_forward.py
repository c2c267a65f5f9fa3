"""GPU parity of fipa_forward (through the C ABI) against the CPU oracle, element by element
on the same seeded inputs.  Tolerances: 1e-4 (fp32 mode), 2e-2 (bf16 inputs, fp32 accumulate),
as max|gpu - oracle| / max|oracle| per output tensor."""
import numpy as np
import pytest

from paper_2505_11580_amd import workloads as wl
from paper_2505_11580_amd import binding
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_f32_workload0():
    gu.check(wl.make_inputs(0), label="cfg0 fp32")


def test_f32_spread_geometry_and_ragged_length():
    # shrunken geometry spreads the attention over many keys; L = 77 leaves a ragged tail
    gu.check(wl.make_inputs(0, L=77, trans_scale=0.1, B=2), label="cfg0 fp32 spread L=77")
    gu.check(wl.make_inputs(0, L=150, chain=True, H=3, cz=24, r=3), label="fp32 chain L=150 r=3")


def test_f32_mask_and_garbage():
    inp = wl.make_inputs(0, L=96, B=3, varlen=True, min_len=5, trans_scale=0.2)
    gu.check(inp, label="fp32 varlen")
    got = gu.run_gpu(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in gu.NAMES:
            assert np.all(got[n][b, int(ln):] == 0), (n, b)
    # a non-prefix mask
    inp = wl.make_inputs(0, L=64, B=1, trans_scale=0.2)
    m = np.ones((1, 64), dtype=np.uint8)
    m[0, [0, 5, 6, 33, 63]] = 0
    inp["mask"] = m
    gu.check(inp, label="fp32 scattered mask")


def test_f32_large_pair_width():
    gu.check(wl.make_inputs(0, L=80, H=2, cz=128, r=2, chain=True), label="fp32 DZ=256")


@pytest.mark.parametrize("cz,r", [(16, 2), (32, 2), (64, 2), (128, 2)])
def test_bf16_small(cz, r):
    # several key tiles, two query tiles, ragged tail
    inp = wl.make_inputs(1, B=2, L=200, H=3, cz=cz, r=r)
    gu.check(inp, label="bf16 L=200 DZ=%d" % (cz * r))
    gu.check(wl.make_inputs(1, B=1, L=131, H=2, cz=cz, r=r, trans_scale=0.1),
             label="bf16 spread L=131 DZ=%d" % (cz * r))


def test_bf16_iid_far_apart_geometry():
    # translations N(0, 10 A) i.i.d.: nearly one-hot attention, large coordinates
    gu.check(wl.make_inputs(1, B=1, L=256, H=4, chain=False), label="bf16 iid geometry")


def test_bf16_mask_and_garbage():
    inp = wl.make_inputs(1, B=3, L=300, H=2, varlen=True, min_len=10)
    gu.check(inp, label="bf16 varlen")
    got = gu.run_gpu(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in gu.NAMES:
            assert np.all(got[n][b, int(ln):] == 0), (n, b)
    inp = wl.make_inputs(1, B=1, L=192, H=2, trans_scale=0.2)
    m = np.ones((1, 192), dtype=np.uint8)
    m[0, 0:70] = 0           # a whole leading key tile masked
    m[0, [100, 101, 191]] = 0
    inp["mask"] = m
    gu.check(inp, label="bf16 scattered mask")


@pytest.mark.parametrize("B,H,L", [(2, 4, 512), (5, 4, 512), (3, 8, 640), (1, 5, 640)])
def test_bf16_key_range_split(B, H, L):
    # few enough tiles that each is cut into 4 / 3 / 2 / 4 key-range parts whose partial rows are
    # merged by the last part to arrive (the last shape puts the parts of a tile on different
    # XCDs); ragged lengths leave some parts short or empty
    inp = wl.make_inputs(1, B=B, L=L, H=H, varlen=True, min_len=40)
    gu.check(inp, label="bf16 split B=%d H=%d L=%d lengths=%s" % (B, H, L, list(inp["lengths"])))
    inp = wl.make_inputs(1, B=B, L=L, H=H, trans_scale=0.05)  # spread attention: every part matters
    gu.check(inp, label="bf16 split spread B=%d H=%d L=%d" % (B, H, L))
    got = [gu.run_gpu(inp) for _ in range(3)]                 # the merge order is fixed: bit-identical reruns
    for n in gu.NAMES + ("lse",):
        assert np.array_equal(got[0][n], got[1][n]) and np.array_equal(got[0][n], got[2][n]), n


@pytest.mark.parametrize("cz,r", [(32, 1), (32, 2), (128, 1), (128, 2)])
def test_bf16_wave_specialised_kernel(cz, r):
    # the opt-in attention kernel with two waves per SIMD (FIPA_FLAG_WAVE_SPECIALISED): one to a few
    # key blocks (the peeled start and end of its loop), whole tiles, ragged and masked chains, the
    # reference raised late (spread geometry, far-apart i.i.d. geometry)
    ws = binding.FIPA_FLAG_WAVE_SPECIALISED
    for L in (20, 50, 97, 131, 300):
        gu.check(wl.make_inputs(1, B=1, L=L, H=2, cz=cz, r=r), label="ws L=%d DZ=%d" % (L, cz * r), flags=ws)
    gu.check(wl.make_inputs(1, B=3, L=600, H=3, cz=cz, r=r, varlen=True, min_len=30),
             label="ws varlen DZ=%d" % (cz * r), flags=ws)
    gu.check(wl.make_inputs(1, B=1, L=400, H=2, cz=cz, r=r, trans_scale=0.05), label="ws spread DZ=%d" % (cz * r), flags=ws)
    gu.check(wl.make_inputs(1, B=1, L=256, H=4, cz=cz, r=r, chain=False), label="ws iid DZ=%d" % (cz * r), flags=ws)


def test_bf16_wave_specialised_kernel_workload2_sampled_rows():
    inp = wl.make_inputs(2)
    rows = wl.select_rows(inp, 256)
    gu.check(inp, rows=rows, label="cfg2 ws 256 rows", chunk=128, flags=binding.FIPA_FLAG_WAVE_SPECIALISED)
    got = [gu.run_gpu(inp, flags=binding.FIPA_FLAG_WAVE_SPECIALISED) for _ in range(2)]
    for n in gu.NAMES + ("lse",):
        assert np.array_equal(got[0][n], got[1][n]), n


def test_bf16_workload1_full():
    gu.check(wl.make_inputs(1), label="cfg1 bf16 full")


def test_bf16_workload2_full():
    # every element of every output (the oracle sweeps the rows in chunks of 256)
    gu.check(wl.make_inputs(2), label="cfg2 bf16 full", chunk=256)


def test_bf16_rank4_small():
    # r*c_z = 512 (lifted width 576): the windowed kernel
    gu.check(wl.make_inputs(3, B=1, L=200, H=2, varlen=False), label="bf16 r=4 L=200")
    gu.check(wl.make_inputs(3, B=2, L=300, H=2, min_len=40, trans_scale=0.2), label="bf16 r=4 varlen spread")


@pytest.mark.parametrize("cz,r,kw", [(64, 8, {}), (256, 2, {}), (32, 16, {}), (128, 4, dict(c=8, Pq=2, Pv=3)),
                                     (128, 4, dict(c=16, Pq=3, Pv=7))])
def test_bf16_width512_other_factor_shapes(cz, r, kw):
    # r*c_z = 512 with other splits into rank and width: c_z = 64 and 256 take the windows that keep the
    # contraction over rho inside a window (epilogue on the registers); c_z = 32 and head shapes other
    # than c = 16, N_value = 8 take the natural-order windows with the separate epilogue kernel
    inp = wl.make_inputs(3, B=2, L=260, H=2, cz=cz, r=r, min_len=30, trans_scale=0.3, **kw)
    gu.check(inp, label="bf16 width 512: cz=%d r=%d %s" % (cz, r, kw))
    got = gu.run_gpu(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in gu.NAMES:
            assert np.all(got[n][b, int(ln):] == 0), (n, b)


@pytest.mark.parametrize("cz,r,kw", [(128, 8, {}), (64, 16, {}), (256, 4, {}), (128, 8, dict(c=8, Pq=2, Pv=3))])
def test_bf16_width1024_rank8(cz, r, kw):
    # r*c_z = 1024 (lifted width 1088: rank 8 at c_z = 128): four windows, two LDS stages, separate epilogue;
    # several key blocks, three query tiles with a ragged tail, a masked batch, spread attention
    inp = wl.make_inputs(3, B=2, L=300, H=2, cz=cz, r=r, min_len=40, trans_scale=0.3, **kw)
    gu.check(inp, label="bf16 width 1024: cz=%d r=%d %s" % (cz, r, kw))
    gu.check(wl.make_inputs(3, B=1, L=70, H=1, cz=cz, r=r, varlen=False, **kw), label="bf16 width 1024 L=70")
    got = gu.run_gpu(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in gu.NAMES:
            assert np.all(got[n][b, int(ln):] == 0), (n, b)


def test_bf16_workload3_sampled_rows():
    # variable-length padded batch, lengths U[1024, 8192], r = 4: 256 rows of every batch element
    # (first / last valid / first padded, one in every 128-row query tile, the rest random) against
    # the oracle's row-subset form
    inp = wl.make_inputs(3)
    gu.check(inp, rows=wl.select_rows(inp, 256), label="cfg3 bf16 sampled rows", chunk=64)
    got = gu.run_gpu(inp)
    for b, ln in enumerate(inp["lengths"]):
        for n in gu.NAMES:
            assert np.all(got[n][b, int(ln):] == 0), (n, b)


def test_bf16_one_chain_of_32768_residues_sampled_rows():
    # far beyond the named workloads (Section 3.1 scales the method in length): 1024 key blocks per tile,
    # 256 query tiles per head, one sampled row in each of them
    inp = wl.make_inputs(1, B=1, L=32768, H=4)
    gu.check(inp, rows=wl.select_rows(inp, 258), label="L=32768 bf16 sampled rows", chunk=16)


def test_bf16_workload4_forward_sampled_rows():
    inp = wl.make_inputs(4, with_grads=False)
    gu.check(inp, rows=wl.select_rows(inp, 256), label="cfg4 fwd bf16 sampled rows", chunk=128)


def test_se3_invariance_on_gpu():
    # Section 3.1: outputs unchanged under a global rotation + translation of all frames
    for cfg, kw, tol in ((0, dict(L=64), 1e-4), (1, dict(B=1, L=256, H=4), 2e-2)):
        inp = wl.make_inputs(cfg, **kw)
        rng = np.random.default_rng(5)
        Rg = wl.random_rotations(rng, ()).astype(np.float32)
        tg = (30.0 * rng.standard_normal(3)).astype(np.float32)
        moved = dict(inp)
        moved["rot"] = np.einsum("xy,blyz->blxz", Rg, inp["rot"]).astype(np.float32)
        moved["trans"] = (np.einsum("xy,bly->blx", Rg, inp["trans"]) + tg).astype(np.float32)
        a, b = gu.run_gpu(inp), gu.run_gpu(moved)
        for n in gu.NAMES:
            assert gu.rel_err(b[n], a[n]) <= tol, (cfg, n, gu.rel_err(b[n], a[n]))


def test_runs_are_bit_identical():
    inp = wl.make_inputs(1, B=1, L=320, H=4)
    a, b = gu.run_gpu(inp), gu.run_gpu(inp)
    for n in gu.NAMES + ("lse",):
        assert np.array_equal(a[n], b[n]), n


def test_bf16_degenerate_shapes():
    # a single residue, a single head, and a chain shorter than one key block
    gu.check(wl.make_inputs(1, B=1, L=1, H=1), label="bf16 L=1 H=1")
    gu.check(wl.make_inputs(1, B=2, L=3, H=2, cz=16, r=2), label="bf16 L=3")
    gu.check(wl.make_inputs(1, B=1, L=33, H=1, trans_scale=0.1), label="bf16 L=33 H=1")


def test_bf16_batch_element_without_valid_residues():
    # one chain of the batch is fully masked: its outputs are zero, the others are unaffected
    inp = wl.make_inputs(1, B=3, L=150, H=2, trans_scale=0.3)
    mask = np.ones((3, 150), dtype=np.uint8)
    mask[1, :] = 0
    mask[2, 100:] = 0
    inp["mask"] = mask
    got = gu.run_gpu(inp)
    for n in gu.NAMES:
        assert np.all(np.isfinite(got[n])), n
        assert np.all(got[n][1] == 0), n
    keep = dict(inp)
    for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans", "z1", "z2"):
        keep[n] = inp[n][[0, 2]]
    keep["mask"] = mask[[0, 2]]
    keep["dims"] = dict(inp["dims"], B=2)
    want = ipa_oracle_forward(keep)
    for n in gu.NAMES:
        assert gu.rel_err(got[n][[0, 2]], want[n]) <= 2e-2, n


def ipa_oracle_forward(inp):
    from oracle import ipa_oracle
    return ipa_oracle.forward(inp)


def test_stage_timer_samples_every_nth_call():
    import torch
    inp = wl.make_inputs(1, B=1, L=256, H=4)
    desc, dev = binding.upload(inp)
    out = binding.alloc_outputs(desc)
    binding.fipa_profile_begin_every(10, 4)
    for _ in range(9):
        binding.forward(desc, dev, out)
    torch.cuda.synchronize()
    stage_ms, n_timed = binding.fipa_profile_end()
    assert n_timed == 3  # calls 0, 4 and 8
    assert stage_ms[0] > 0 and stage_ms[1] > 0


@pytest.mark.parametrize("B,H,L", [(5, 3, 200), (66, 1, 128), (9, 2, 130)])
def test_masked_batches_with_odd_pair_counts(B, H, L):
    # masked batches renumber their (batch, head) pairs (ranked by chain length, dealt to the XCDs);
    # pair counts that are no multiples of 8, more batch elements than a wave has lanes, equal lengths
    inp = wl.make_inputs(1, B=B, H=H, L=L, varlen=True, min_len=3, cz=32)
    gu.check(inp, label="bf16 masked B=%d H=%d L=%d" % (B, H, L))
    inp = wl.make_inputs(1, B=B, H=H, L=L, varlen=True, min_len=L, cz=32)   # a mask, all chains full length
    gu.check(inp, label="bf16 masked, equal lengths B=%d H=%d" % (B, H))
