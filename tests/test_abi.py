"""The C-ABI library loads and exports what include/fipa.h declares; host-side argument
checks answer with error codes before anything touches a device (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2505_11580_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fipa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fipa_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert binding.lib().fipa_version() >= 100
    for code in (0, -1, -2, -3, -4, -5):
        assert binding.status_string(code) != "unknown status"
    assert binding.status_string(-99) == "unknown status"


def test_workspace_is_affine_in_length():
    # linear memory in L (Section 2.3): equal steps in L give equal steps in bytes
    for dtype, r in ((binding.FIPA_DTYPE_BF16, 2), (binding.FIPA_DTYPE_F32, 2)):
        sizes = [binding.workspace_bytes(binding.make_desc(1, L, 12, 16, 4, 8, 128, r, dtype))[0]
                 for L in (1024, 2048, 3072, 4096, 8192)]
        steps = [sizes[1] - sizes[0], sizes[2] - sizes[1], sizes[3] - sizes[2], (sizes[4] - sizes[3]) // 4]
        assert len(set(steps)) == 1 and steps[0] > 0, sizes


def test_bad_descriptions_are_rejected_on_the_host():
    lib = binding.lib()
    sz = ctypes.c_size_t(0)
    bad = binding.make_desc(1, 0, 4, 16, 4, 8, 16, 2, binding.FIPA_DTYPE_F32)
    assert lib.fipa_workspace_bytes(ctypes.byref(bad), ctypes.byref(sz), None) == binding.FIPA_ERR_INVALID_ARG
    bad = binding.make_desc(1, 64, 4, 16, 4, 8, 16, 2, 7)
    assert lib.fipa_workspace_bytes(ctypes.byref(bad), ctypes.byref(sz), None) == binding.FIPA_ERR_INVALID_ARG
    odd = binding.make_desc(1, 64, 4, 16, 4, 8, 24, 2, binding.FIPA_DTYPE_BF16)  # r*cz = 48
    assert lib.fipa_workspace_bytes(ctypes.byref(odd), ctypes.byref(sz), None) == binding.FIPA_ERR_UNSUPPORTED
    assert lib.fipa_workspace_bytes(None, ctypes.byref(sz), None) == binding.FIPA_ERR_INVALID_ARG


def test_forward_argument_checks_need_no_device():
    lib = binding.lib()
    d = binding.make_desc(1, 64, 4, 16, 4, 8, 16, 2, binding.FIPA_DTYPE_F32)
    nulls = [None] * 17
    assert lib.fipa_forward(ctypes.byref(d), *nulls, None, 0, None) == binding.FIPA_ERR_INVALID_ARG
    fake = [ctypes.c_void_p(0x1000)] * 17
    fake[12] = None  # mask may be NULL
    assert lib.fipa_forward(ctypes.byref(d), *fake, ctypes.c_void_p(0x1000), 0, None) == binding.FIPA_ERR_WORKSPACE
    mis = list(fake)
    mis[0] = ctypes.c_void_p(0x1004)
    assert lib.fipa_forward(ctypes.byref(d), *mis, ctypes.c_void_p(0x1000), 1 << 30, None) == binding.FIPA_ERR_ALIGNMENT
    with pytest.raises(binding.FipaError):
        binding.workspace_bytes(binding.make_desc(1, -5, 4, 16, 4, 8, 16, 2, 0))


def test_packed_forward_argument_checks_need_no_device():
    lib = binding.lib()
    d = binding.make_desc(3, 64, 4, 16, 4, 8, 16, 2, binding.FIPA_DTYPE_BF16)
    fake = [ctypes.c_void_p(0x1000)] * 17
    ws = ctypes.c_void_p(0x1000)

    def call(cu, size=1 << 30):
        arr = (ctypes.c_int32 * len(cu))(*cu)
        return lib.fipa_forward_packed(ctypes.byref(d), arr, *fake, ws, size, None)

    assert lib.fipa_forward_packed(ctypes.byref(d), None, *fake, ws, 1 << 30, None) == binding.FIPA_ERR_INVALID_ARG
    assert call([1, 10, 20, 30]) == binding.FIPA_ERR_INVALID_ARG      # does not start at 0
    assert call([0, 10, 5, 30]) == binding.FIPA_ERR_INVALID_ARG       # decreasing
    assert call([0, 10, 80, 90]) == binding.FIPA_ERR_INVALID_ARG      # a chain longer than desc->L
    assert call([0, 10, 20, 30], size=0) == binding.FIPA_ERR_WORKSPACE
    assert call([0, 0, 0, 0]) == binding.FIPA_OK                      # only empty chains: nothing to enqueue


def test_packed_workspace_query_and_backward_argument_checks_need_no_device():
    lib = binding.lib()
    d = binding.make_desc(4, 900, 12, 16, 4, 8, 128, 2, binding.FIPA_DTYPE_BF16)
    one = binding.make_desc(1, 900, 12, 16, 4, 8, 128, 2, binding.FIPA_DTYPE_BF16)
    even = binding.make_desc(4, 700, 12, 16, 4, 8, 128, 2, binding.FIPA_DTYPE_BF16)
    # chains of similar lengths: one set of launches, workspace of the padded batch (at the longest chain) + offsets
    fwd, bwd = binding.packed_workspace_bytes(d, [0, 700, 1300, 1900, 2500])
    pf, pb = binding.workspace_bytes(even)
    assert pf < fwd <= pf + 1024 and pb < bwd <= pb + 1024
    # one dominant chain: chain after chain, workspace of the longest chain alone (+ the per-chain gamma / w_b sums)
    fwd, bwd = binding.packed_workspace_bytes(d, [0, 900, 940, 973, 1043])
    assert fwd == binding.workspace_bytes(one)[0]
    assert binding.workspace_bytes(one)[1] < bwd <= binding.workspace_bytes(one)[1] + 4 * 4 * (12 + 12 * 128) + 1024
    # the flag forces it
    d.flags = binding.FIPA_FLAG_PACKED_PER_CHAIN
    per = binding.make_desc(1, 700, 12, 16, 4, 8, 128, 2, binding.FIPA_DTYPE_BF16)
    assert binding.packed_workspace_bytes(d, [0, 700, 1300, 1900, 2500])[0] == binding.workspace_bytes(per)[0]
    d.flags = 0
    with pytest.raises(binding.FipaError):
        binding.packed_workspace_bytes(d, [0, 950, 1000, 1100, 1200])  # a chain longer than desc->L
    fake = [ctypes.c_void_p(0x1000)] * 28
    fake[12] = None  # mask
    cu = (ctypes.c_int32 * 5)(0, 700, 1300, 1900, 2500)
    ws = ctypes.c_void_p(0x1000)
    assert lib.fipa_backward_packed(ctypes.byref(d), cu, *fake, ws, 0, None) == binding.FIPA_ERR_WORKSPACE
    assert lib.fipa_backward_packed(ctypes.byref(d), None, *fake, ws, 1 << 40, None) == binding.FIPA_ERR_INVALID_ARG
    only_rot = list(fake)
    only_rot[27] = None  # d_trans without d_rot's partner
    assert lib.fipa_backward_packed(ctypes.byref(d), cu, *only_rot, ws, 1 << 40, None) == binding.FIPA_ERR_INVALID_ARG
    f32 = binding.make_desc(4, 900, 12, 16, 4, 8, 16, 2, binding.FIPA_DTYPE_F32)
    assert lib.fipa_backward_packed(ctypes.byref(f32), cu, *fake, ws, 1 << 40, None) == binding.FIPA_ERR_UNSUPPORTED


def test_knn_distogram_argument_checks_need_no_device():
    lib = binding.lib()
    p = ctypes.c_void_p(0x1000)

    def call(B=2, L=50, k=20, n_bins=16, d_min=2.0, d_max=22.0, trans=p, idx=p):
        return lib.fipa_knn_distogram(B, L, k, n_bins, d_min, d_max, trans, None, idx, p, p, None)

    assert call(L=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(k=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_bins=1) == binding.FIPA_ERR_INVALID_ARG
    assert call(d_min=5.0, d_max=5.0) == binding.FIPA_ERR_INVALID_ARG
    assert call(d_min=-1.0) == binding.FIPA_ERR_INVALID_ARG
    assert call(trans=None) == binding.FIPA_ERR_INVALID_ARG
    assert call(k=65) == binding.FIPA_ERR_UNSUPPORTED
    assert call(idx=ctypes.c_void_p(0x1002)) == binding.FIPA_ERR_ALIGNMENT


def test_factor_project_argument_checks_need_no_device():
    lib = binding.lib()
    p = ctypes.c_void_p(0x1000)

    def call(B=2, L=50, k=20, n_bins=16, n_pos=65, pos_mode=1, n_out=256, idx=p, e_pos=p, z=p):
        return lib.fipa_factor_project(B, L, k, n_bins, n_pos, pos_mode, n_out, idx, p, p, e_pos, None, z, None)

    assert call(L=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_bins=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(pos_mode=2) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_pos=64) == binding.FIPA_ERR_INVALID_ARG          # offsets need an odd number of rows
    assert call(n_pos=0) == binding.FIPA_ERR_INVALID_ARG           # a table without rows
    assert call(e_pos=None) == binding.FIPA_ERR_INVALID_ARG        # rows without a table
    assert call(z=None) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_out=100) == binding.FIPA_ERR_UNSUPPORTED
    assert call(k=65) == binding.FIPA_ERR_UNSUPPORTED
    assert call(z=ctypes.c_void_p(0x1008)) == binding.FIPA_ERR_ALIGNMENT
    assert call(idx=ctypes.c_void_p(0x1002)) == binding.FIPA_ERR_ALIGNMENT


def test_factor_project_backward_argument_checks_need_no_device():
    lib = binding.lib()
    p = ctypes.c_void_p(0x1000)

    def call(B=2, L=50, k=20, n_bins=16, n_pos=65, pos_mode=1, n_out=256, d_z=p, d_e_pos=p, d_e_bin=p):
        return lib.fipa_factor_project_backward(B, L, k, n_bins, n_pos, pos_mode, n_out, p, p, d_z, None, d_e_bin, d_e_pos,
                                                None, None)

    assert call(B=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(d_z=None) == binding.FIPA_ERR_INVALID_ARG
    assert call(d_e_pos=None) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_pos=0) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_pos=64) == binding.FIPA_ERR_INVALID_ARG
    assert call(n_out=100) == binding.FIPA_ERR_UNSUPPORTED
    assert call(n_bins=4096) == binding.FIPA_ERR_UNSUPPORTED      # the table slice does not fit LDS
    assert call(d_e_bin=ctypes.c_void_p(0x1004)) == binding.FIPA_ERR_ALIGNMENT


def test_stage_timer_argument_checks_need_no_device():
    lib = binding.lib()
    assert lib.fipa_profile_begin_every(10, 0) == binding.FIPA_ERR_INVALID_ARG
    assert lib.fipa_profile_begin_every(0, 1) == binding.FIPA_ERR_INVALID_ARG
    assert lib.fipa_profile_begin_every(5000, 1) == binding.FIPA_ERR_INVALID_ARG
    assert lib.fipa_profile_end(None, None) == binding.FIPA_ERR_INVALID_ARG  # timing is not active


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: the benchmark says so instead of running on a subset
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2
    assert "single-GPU" in res.stderr
