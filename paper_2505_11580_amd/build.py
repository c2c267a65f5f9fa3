"""Compile libfipa.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfipa.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the attention kernels rely on full unrolling of long constant-trip-count loops
         "-mllvm", "-pragma-unroll-threshold=4000000",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]


# Per-file additions.  The MFMA kernels are compiled with the MFMA results selected in the general
# vector-register class, so that the register allocator decides per value between architectural
# and accumulation registers: accumulators that the vector ALU reads (S^T, dP, the output
# accumulator when it is rescaled) then need no copies out of accumulation registers, while the
# stationary fragments are pinned to accumulation registers in the source.  Measured against
# the default (every MFMA result in accumulation registers): fused attention -3.5 % at B=2,
# L=2048, rank-4 kernel -2.7 %, gradient kernels -4 / -6 / -10 % (dV^, dQ^, dK^; without the pins
# they got 1.6 % slower).
_VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
PER_FILE = {
    "fipa_bf16_attn_fwd.hip": _VGPR_FORM,
    "fipa_bf16_attn_fwd_ws.hip": _VGPR_FORM,
    "fipa_bf16_attn_fwd_wide.hip": _VGPR_FORM,
    "fipa_bf16_bwd_kernel.hip": _VGPR_FORM,
    # the neighbour search specifies its distance arithmetic with one rounding per operation
    "fipa_knn.hip": ["-ffp-contract=off"],
}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, jobs: int = 8, csrc: str = CSRC, out: str = LIB, extra=()) -> str:
    """Compile every csrc/*.hip to an object (in parallel) and link libfipa.so."""
    objdir = os.path.join(os.path.dirname(out), "_build_" + os.path.basename(out)) if out != LIB else os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in sorted(glob.glob(os.path.join(csrc, "*.hip"))):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [HIPCC] + [f if f != CSRC else csrc for f in FLAGS] + PER_FILE.get(os.path.basename(src), []) + list(extra) + ["-c", src, "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout)
    return out


def _drain(procs, verbose):
    while procs:
        src, pr = procs.pop(0)
        out, _ = pr.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln]
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, "\n".join(lines)))
        if verbose and lines:
            print("\n".join(lines))


if __name__ == "__main__":
    print(build(verbose=True))
