#!/usr/bin/env python3
"""Benchmark of the factorized-IPA forward hot path on one MI355X.

One "step" = one fipa_forward call (pack -> fused attention -> epilogue) over one batch of
the long-chain workload (B=2, L=2048, H=12, c=16, N_query=4, N_value=8, c_z=128, r=2; bf16
inputs, fp32 accumulation), with all inputs resident in HBM before the timed region.
Prints ONE JSON line: whole-path algorithmic TFLOP/s (`value`), residues/s, the roofline
of the dominant kernel (fused attention, bf16 MFMA) from HIP events recorded around that
kernel inside the timed region, and the CPU oracle timed on a bounded sample of the same
workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def cpu_baseline(inp, flops_per_pair, budget_s=12.0, single_budget_s=6.0):
    """Time the oracle (as it stands) on whole passes over the same workload, about budget_s seconds on
    all host threads, then on a row sample with one thread."""
    import numpy as np
    from oracle import ipa_oracle
    d = inp["dims"]
    L, H, B = d["L"], d["H"], d["B"]
    rows = [np.arange(int(n), dtype=np.int32) for n in inp["lengths"]]  # every valid query row
    n_rows = sum(len(r) for r in rows)
    threads = ipa_oracle.num_threads()
    passes, secs = 0, 0.0
    while secs < budget_s and passes < 50:
        t0 = time.perf_counter()
        ipa_oracle.forward(inp, rows=rows)
        secs += time.perf_counter() - t0
        passes += 1
    pairs = passes * n_rows * L * H
    # one thread: the first rows of every chain, sized from the all-thread rate to about single_budget_s
    per_row_s = secs / (passes * n_rows) * threads
    n1 = int(max(4, min(min(len(r) for r in rows), single_budget_s / max(per_row_s, 1e-9) / B)))
    ipa_oracle.set_num_threads(1)
    t0 = time.perf_counter()
    ipa_oracle.forward(inp, rows=[r[:n1] for r in rows])
    secs1 = time.perf_counter() - t0
    ipa_oracle.set_num_threads(threads)
    return {
        "value": pairs * flops_per_pair / secs / 1e12,
        "unit": "TFLOP/s",
        "residues_per_s": passes * n_rows / secs,
        "cores": threads,
        "kind": "oracle",
        "sample": "%d whole pass(es) of the fp64 C oracle (OpenMP) over the same workload "
                  "(all %d query rows, %d keys, %d heads), %.1f s" % (passes, n_rows, L, H, secs),
        "single_thread": {"value": n1 * B * L * H * flops_per_pair / secs1 / 1e12, "unit": "TFLOP/s",
                          "residues_per_s": n1 * B / secs1, "cores": 1,
                          "sample": "the first %d query rows of each of the %d chains, %.1f s" % (n1, B, secs1)},
    }


def measured_peaks():
    """What this machine sustains: an MFMA-only kernel (bf16 32x32x16, independent accumulators) and a plain
    256 MiB elementwise copy.  Second denominators beside the published peaks; HIP-event timing."""
    import torch
    from paper_2505_11580_amd import binding
    wgs, iters = 1024, 4000
    buf = torch.empty(wgs * 256, dtype=torch.float32, device="cuda:0")
    for _ in range(3):
        flop = binding.probe_mfma(iters, wgs, buf)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        binding.probe_mfma(iters, wgs, buf)
    e1.record()
    torch.cuda.synchronize()
    mfma = 5 * flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    n = 256 << 20
    src = torch.ones(n // 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    e0.record()
    for _ in range(10):
        torch.mul(src, 1.0, out=dst)
    e1.record()
    torch.cuda.synchronize()
    copy = 10 * 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return {"mfma_bf16_tflops": mfma, "copy_read_plus_write_gbs": copy,
            "how": "MFMA-only kernel (%d workgroups x 4 waves x %d x 16 MFMAs) and a 256 MiB elementwise copy, HIP events" % (wgs, iters)}


def backward_leg(workload, steps=30, warmup=10):
    """fipa_backward (recomputation of the lifted forward + the three gradient kernels + unpack) on
    the gradient workload; reported beside the headline forward number, not part of `value`."""
    import torch
    from paper_2505_11580_amd import binding, workloads
    inp = workloads.make_inputs(workload, with_grads=True)
    dims = inp["dims"]
    desc, dev = binding.upload(inp)
    out = binding.alloc_outputs(desc)
    grads = binding.alloc_grads(desc)
    binding.forward(desc, dev, out)
    for _ in range(warmup):
        binding.backward(desc, dev, out, grads)
    torch.cuda.synchronize()
    binding.fipa_profile_begin(steps)
    t0 = time.perf_counter()
    for _ in range(steps):
        binding.backward(desc, dev, out, grads)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    stage_ms, _ = binding.fipa_profile_end()
    pairs = workloads.valid_pairs(inp)
    fpp = workloads.bwd_flops_per_pair(dims)

    # a training step = forward call + backward call: as two independent calls (the backward
    # recomputes what it needs), and with FIPA_FLAG_KEEP_FORWARD (the forward leaves it in the
    # backward's workspace)
    def step_ms(flags, ws):
        desc.flags = flags
        out_ws = out["workspace"]
        out["workspace"] = ws
        for _ in range(warmup):
            binding.forward(desc, dev, out)
            binding.backward(desc, dev, out, grads)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            binding.forward(desc, dev, out)
            binding.backward(desc, dev, out, grads)
        torch.cuda.synchronize()
        out["workspace"] = out_ws
        desc.flags = 0
        return (time.perf_counter() - t0) / steps * 1e3

    step_plain = step_ms(0, out["workspace"])
    step_keep = step_ms(binding.FIPA_FLAG_KEEP_FORWARD, grads["workspace"])
    return {
        "workload": "workload %d: B=%d L=%d H=%d cz=%d r=%d, bf16" % (workload, dims["B"], dims["L"], dims["H"],
                                                                    dims["cz"], dims["r"]),
        "ms_per_call": ms, "value": pairs * fpp / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
        "valid_pairs": pairs, "flops_per_pair": fpp, "steps": steps,
        "stage_ms": {"recompute_forward": stage_ms[0], "gradient_kernels": stage_ms[1], "unpack": stage_ms[2]},
        "training_step_ms": {"forward_then_backward": step_plain, "with_keep_forward_flag": step_keep},
    }


def module_leg(workload, d_s=256, steps=300, warmup=100):
    """fipa_module_forward (input projection + core + output projection) on the headline
    workload; reported beside the headline number, not part of `value`."""
    import torch
    from paper_2505_11580_amd import binding, workloads
    m = workloads.make_module_inputs(workload, d_s=d_s)
    desc, dev = binding.upload_module(m)
    for _ in range(warmup):
        binding.module_forward(desc, d_s, dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        binding.module_forward(desc, d_s, dev)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    n_in, n_cat = workloads.module_widths(m["dims"])
    rows = m["dims"]["B"] * m["dims"]["L"]
    out = {"workload": "workload %d with d_s=%d" % (workload, d_s), "ms_per_call": ms, "steps": steps,
           "projection_gflop": 2.0 * rows * d_s * (n_in + n_cat) / 1e9,
           "residues_per_s": float(m["lengths"].sum()) / (ms * 1e-3)}
    # fipa_module_backward on the same inputs (recomputes the forward inside)
    grads = binding.alloc_module_grads(desc, d_s)
    up = torch.randn(m["dims"]["B"], m["dims"]["L"], d_s, device="cuda:0")
    bsteps = max(3, steps // 5)
    for _ in range(max(2, warmup // 10)):
        binding.module_backward(desc, d_s, dev, up, grads)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(bsteps):
        binding.module_backward(desc, d_s, dev, up, grads)
    torch.cuda.synchronize()
    out["backward_ms_per_call"] = (time.perf_counter() - t0) / bsteps * 1e3

    # a training step = forward call + backward call, as two independent calls and with
    # FIPA_FLAG_KEEP_FORWARD (the forward runs in the backward's workspace and leaves its results there)
    def step_ms(flags, ws):
        desc.flags = flags
        fwd_ws, dev["workspace"] = dev["workspace"], ws
        for _ in range(3):
            binding.module_forward(desc, d_s, dev)
            binding.module_backward(desc, d_s, dev, up, grads)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(bsteps):
            binding.module_forward(desc, d_s, dev)
            binding.module_backward(desc, d_s, dev, up, grads)
        torch.cuda.synchronize()
        dev["workspace"] = fwd_ws
        desc.flags = 0
        return (time.perf_counter() - t0) / bsteps * 1e3

    out["training_step_ms"] = {"forward_then_backward": step_ms(0, dev["workspace"]),
                               "with_keep_forward_flag": step_ms(binding.FIPA_FLAG_KEEP_FORWARD, grads["workspace"])}
    return out


def packed_leg(B=32, lo=64, hi=512, steps=100, warmup=30):
    """Variable-length batch of short chains (lengths drawn as in the paper's protein training sets, Table 2:
    up to 512 residues), stored back to back: fipa_forward_packed / fipa_backward_packed as one set of
    launches, chain after chain, and the same chains padded to the longest with a mask through
    fipa_forward / fipa_backward.  Opt-in (--packed-leg); not part of `value`."""
    import numpy as np
    import torch
    from paper_2505_11580_amd import binding, workloads
    inp = workloads.make_inputs(1, B=B, L=hi, varlen=True, min_len=lo, with_grads=True)
    lengths = [int(x) for x in inp["lengths"]]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    desc, dev = binding.upload(inp)
    names = ("q", "k", "v", "q_pts", "k_pts", "v_pts", "rot", "trans", "z1", "z2")
    pk = {n: torch.cat([dev[n][b, :ln] for b, ln in enumerate(lengths)], dim=0).contiguous()
          for n in names + ("d_o", "d_o_pts", "d_o_pair")}
    total, H = int(cu[-1]), desc.H
    f = dict(dtype=torch.float32, device="cuda:0")
    o = [torch.empty(total, H, desc.c, **f), torch.empty(total, H, desc.Pv, 3, **f), torch.empty(total, H, desc.cz, **f),
         torch.empty(H * total, **f)]
    g = [torch.empty_like(pk[n]) for n in ("q", "k", "v", "q_pts", "k_pts", "v_pts", "z1", "z2")]
    g += [torch.empty(H, **f), torch.empty(H, desc.cz, **f), torch.empty(total, 3, 3, **f), torch.empty(total, 3, **f)]
    out = binding.alloc_outputs(desc)
    grads = binding.alloc_grads(desc)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    res = {"workload": "B=%d chains of %d..%d residues (total %d, longest %d), H=%d cz=%d r=%d, bf16"
                       % (B, lo, hi, total, max(lengths), H, desc.cz, desc.r)}
    for label, flags in (("one_launch", 0), ("per_chain", binding.FIPA_FLAG_PACKED_PER_CHAIN)):
        desc.flags = flags
        fwd_b, bwd_b = binding.packed_workspace_bytes(desc, cu)
        ws = torch.empty(max(fwd_b, bwd_b, 16), dtype=torch.uint8, device="cuda:0")
        fwd = timed(lambda: binding.fipa_forward_packed(desc, cu, *[pk[n] for n in names], dev["w_b"], dev["gamma"], None,
                                                        o[0], o[1], o[2], o[3], ws))
        bwd = timed(lambda: binding.fipa_backward_packed(desc, cu, *[pk[n] for n in names], dev["w_b"], dev["gamma"], None,
                                                         pk["d_o"], pk["d_o_pts"], pk["d_o_pair"], *g, ws))
        res[label] = {"forward_ms": fwd, "backward_ms": bwd, "forward_workspace_mb": fwd_b / 1e6,
                      "backward_workspace_mb": bwd_b / 1e6}
        del ws
    desc.flags = 0
    res["padded_with_mask"] = {"forward_ms": timed(lambda: binding.forward(desc, dev, out)),
                               "backward_ms": timed(lambda: binding.backward(desc, dev, out, grads)),
                               "forward_workspace_mb": binding.workspace_bytes(desc)[0] / 1e6,
                               "backward_workspace_mb": binding.workspace_bytes(desc)[1] / 1e6}
    return res


def calibrate_copy(nbytes=256 << 20):
    """A plain elementwise copy of known size (reads nbytes, writes nbytes), so that a counter run of
    this script sees a kernel whose HBM traffic is known next to the attention kernel."""
    import torch
    src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()


# HBM traffic of one launch of the attention kernel: NOT measured in this run.  The figure comes from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the same counters read
# for calibrate_copy(); the summary with the commands is the file named here.
MEASURED_TRAFFIC = {2: (163.3e6, "profiles/attn_fwd_bf16_workload2_hbm_traffic.md")}  # 107.0 MB fetched + 56.3 MB written


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (the clocks settle over the first few hundred launches after an idle period: the step time
    # falls by about 10 % during that time, so the default warm-up is long and the timed region
    # covers 1000 steps = 0.15 s)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--clock-warmup", type=int, default=300,
                    help="least number of untimed steps before the timed region: when --warmup is smaller, the "
                         "difference is run first (reported as clock_warmup_steps), so that a short warm-up does "
                         "not time the GPU on its way up from idle clocks; 0 = exactly --warmup steps")
    ap.add_argument("--workload", type=int, default=2, help="workload index (2 = the L=2048 headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true", help="skip the fipa_backward leg (workload 4)")
    ap.add_argument("--backward-workload", type=int, default=4, help="workload of the fipa_backward leg (3: the ragged rank-4 batch)")
    ap.add_argument("--no-module", action="store_true", help="skip the module leg (fipa_module_forward / backward)")
    ap.add_argument("--no-measured-peaks", action="store_true", help="skip the MFMA-only and copy probes")
    ap.add_argument("--wave-specialised", action="store_true",
                    help="run the forward leg with FIPA_FLAG_WAVE_SPECIALISED (the opt-in attention kernel with two "
                         "waves per SIMD); the JSON line says so in config.attention_kernel")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (same generators)")
    ap.add_argument("--seq-len", type=int, default=0, help="override the workload's sequence length (same generators)")
    ap.add_argument("--rank", type=int, default=0, help="override the workload's factor rank r (same generators)")
    ap.add_argument("--packed-leg", action="store_true",
                    help="also time a packed batch of 32 short chains (one launch / chain after chain / padded)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB copy kernel (for scaling hardware counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; --gpus %d is not supported (run with --gpus 1)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_11580_amd import binding, workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    over = {}
    if args.batch > 0:
        over["B"] = args.batch
    if args.seq_len > 0:
        over["L"] = args.seq_len
    if args.rank > 0:
        over["r"] = args.rank
    inp = workloads.make_inputs(args.workload, with_grads=False, **over)
    dims = inp["dims"]
    desc, dev = binding.upload(inp)
    if args.wave_specialised:
        desc.flags = binding.FIPA_FLAG_WAVE_SPECIALISED
    out = binding.alloc_outputs(desc)
    pairs = workloads.valid_pairs(inp)
    fpp = workloads.fwd_flops_per_pair(dims)
    residues = int(inp["lengths"].sum())

    clock_warmup_steps = max(0, args.clock_warmup - args.warmup)
    warmup_run = clock_warmup_steps + args.warmup  # untimed steps actually run
    for _ in range(warmup_run):
        binding.forward(desc, dev, out)
    torch.cuda.synchronize()

    # The stage timers record HIP events on the stream around each kernel; with every step timed
    # they cost about 13 us per 150 us step, so only one step in eight of the timed region
    # carries them (one in four, or every step, when the run is short).
    every = 8 if args.steps >= 64 else (4 if args.steps >= 8 else 1)
    binding.fipa_profile_begin_every((args.steps + every - 1) // every, every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        binding.forward(desc, dev, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stage_ms, n_timed = binding.fipa_profile_end()

    ms_per_step = elapsed / args.steps * 1e3
    tflops = pairs * fpp / (ms_per_step * 1e-3) / 1e12
    attn_ms = stage_ms[1]
    attn_tflops = pairs * fpp / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else 0.0

    result = {
        "metric": "factorized-IPA fwd TFLOP/s + residues/s at L=2048; % of bf16 MFMA peak",
        "value": tflops,
        "unit": "TFLOP/s",
        "residues_per_s": residues / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": warmup_run,
        "warmup_requested": args.warmup,
        "clock_warmup_steps": clock_warmup_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "workload %d: B=%d L=%d H=%d c=%d Pq=%d Pv=%d cz=%d r=%d, bf16 in / fp32 "
                               "accumulate, random-walk chain frames, forward only"
                               % (args.workload, dims["B"], dims["L"], dims["H"], dims["c"], dims["Pq"],
                                  dims["Pv"], dims["cz"], dims["r"]),
                   "valid_pairs": pairs, "flops_per_pair": fpp,
                   "attention_kernel": "wave-specialised (opt-in)" if args.wave_specialised else "default",
                   "shape_override": over or None},
        "stage_ms": {"pack": stage_ms[0], "attention": stage_ms[1], "epilogue": stage_ms[2],
                     "timed_calls": n_timed, "timed_every": every},
        "roofline": {"kernel": "fipa_attn_fwd_wide_kernel" if dims["r"] * dims["cz"] > 256
                     else ("fipa_attn_fwd_ws_kernel" if args.wave_specialised else "fipa_attn_fwd_bf16_kernel"),
                     "bound": "mfma", "achieved": attn_tflops,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None if over or args.wave_specialised else MEASURED_TRAFFIC.get(args.workload, (None, None))[0],
                     "traffic_source": "not measured for this variant" if over or args.wave_specialised
                     else MEASURED_TRAFFIC.get(args.workload, (None, "not measured for this workload"))[1]},
    }
    # the pack kernel against the HBM roofline: bytes it must move per residue (bf16 inputs of Algorithm 1
    # steps 2-6 read once; head-specific lifted rows, the shared z2 copy and the two bias vectors written once)
    H, DZ = dims["H"], dims["r"] * dims["cz"]
    pack_bytes = residues * (2 * (3 * H * dims["c"] + 3 * H * (2 * dims["Pq"] + dims["Pv"])) + 48 + 2 * DZ  # read (z1 is the attention kernel's)
                             + 3 * H * 128 + 2 * DZ + 8 * H)                                                      # written
    if stage_ms[0] > 0:
        result["pack_roofline"] = {"kernel": "fipa_pack_heads_af2_bf16_kernel", "bound": "hbm", "bytes": pack_bytes,
                                   "achieved": pack_bytes / (stage_ms[0] * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                                   "frac": pack_bytes / (stage_ms[0] * 1e-3) / 8e12}
    if not args.no_measured_peaks:
        pk = measured_peaks()
        result["roofline"]["peak_measured"] = pk["mfma_bf16_tflops"]
        result["roofline"]["frac_of_measured_peak"] = attn_tflops / pk["mfma_bf16_tflops"] if pk["mfma_bf16_tflops"] > 0 else None
        result["measured_peaks"] = pk
    if args.calibrate_copy:
        calibrate_copy()
    del out, dev
    torch.cuda.empty_cache()
    if not args.no_module:
        result["module"] = module_leg(args.workload)
    if not args.no_backward:
        result["backward"] = backward_leg(args.backward_workload, steps=30 if args.backward_workload == 4 else 5,
                                          warmup=10 if args.backward_workload == 4 else 2)
    if args.packed_leg:
        result["packed"] = packed_leg()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(inp, fpp)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
