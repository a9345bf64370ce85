#!/usr/bin/env python3
"""Benchmark of the FO-SGD gradient codec (arXiv 2405.11095) on one MI355X.

A step is one whole FO-SGD iteration of the codec (Sec. 4): M uplink encodes, the server's
decode + average + re-encode, one downlink decode and the SGD update, all inside fo_step with
the M synthetic gradients already resident in HBM.  The workload is the ResNet-50-sized one:
d = 25,557,032 fp32 coordinates zero-padded to n = 2^25, M = 16 workers, heavy-tailed entries.

Prints ONE JSON line.  `value` is GB/s of fp32 gradient processed (4 d M bytes per step).
`roofline` is for the kernel with the largest share of the step, timed with HIP events on the
launch stream inside the timed region.  `cpu_baseline` is the plain fp64 oracle timed on the host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch on workload c3 measured with rocprofv3 --pmc (FETCH_SIZE scaled by 2.000, WRITE_SIZE
# by 1.000, the factors of a 1 GiB copy; profiles/c3_fo_step_hbm_traffic.md), keyed by kernel name.  For the
# kernels launched with two batch sizes per step the figure is the per-step sum divided by two.
MEASURED_TRAFFIC = {
    "k_strided<ENC_FIRST>": 3783807574,
    "k_contig<IN_F32,OUT_PACK>": (2214798093 + 138661273) // 2,
    "k_strided<SERVER>": 1208240742,
    "k_declow": (1140953485 + 71407510) // 2,
    "k_strided<DEC_LAST>": 271920344,
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4"],
                    help="c3 is the headline workload; the others are the parity configurations, timed for the report")
    ap.add_argument("--block-log2", type=int, default=None,
                    help="transform length 2^k (default: the workload's first entry; c4 has 10, 12, 14, 16)")
    ap.add_argument("--K", type=int, default=1, help="averaging count of the downlink quantiser")
    ap.add_argument("--server-scale", default="thm", choices=["thm", "l2"],
                    help="server amplitude: Thm 5.5 as stated (default) or from the measured norm of the mean")
    ap.add_argument("--eps-mode", default="independent", choices=["independent", "shared", "all"],
                    help="independent: the paper's protocol (default, the headline number); shared: one eps for all "
                         "workers and the popcount server; all: the server shares that eps too and needs no transform")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known HBM traffic, used to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the M workers are M buffers on one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2405_11095_amd import binding as B, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = inputs.WORKLOADS[args.workload]
    d, M = wl["d"], wl["M"]
    t0 = time.time()
    gs_host = inputs.workload(args.workload)
    gs = [torch.from_numpy(g).to(dev) for g in gs_host]
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    eps_mode = {"independent": B.EPS_INDEPENDENT, "shared": B.EPS_SHARED_WORKERS, "all": B.EPS_SHARED_ALL}[args.eps_mode]
    blk = wl["block_log2"][0] if args.block_log2 is None else args.block_log2
    seed = 0xF05D + int(args.workload[1])
    srv = B.SERVER_SCALE_L2 if args.server_scale == "l2" else B.SERVER_SCALE_THM
    plan = B.Plan(d=d, M=M, block_log2=blk, K=args.K, seed=seed, eps_mode=eps_mode, server_scale=srv)
    n = plan.ntot
    print(f"[bench] workload {args.workload}: d={d} n={n} M={M}; inputs ready in {time.time() - t0:.1f}s; "
          f"plan scratch {plan.scratch_bytes / 2**30:.2f} GiB", file=sys.stderr, flush=True)

    copy_gbs = None
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9   # read + write of 1 GiB, five times
        print(f"[bench] 1 GiB device-to-device copy: {copy_gbs:.0f} GB/s (read + write)", file=sys.stderr, flush=True)
        del src, dst

    delta = 1e-3
    for w in range(args.warmup):
        plan.fo_step(gs, x, delta, w)
    torch.cuda.synchronize()
    # Untimed pass with every kernel bracketed by events: the per-kernel breakdown, and which kernel dominates.
    # (Events between kernels keep one from starting while the previous one drains, about 3 % of the step, so the
    # timed region below brackets the dominant kernel only.)
    nbreak = max(3, min(args.steps, 10))
    plan.fo_profile_begin()
    for k in range(nbreak):
        plan.fo_step(gs, x, delta, 1000 + k)
    torch.cuda.synchronize()
    breakdown = plan.fo_profile_end()
    dom = max(breakdown, key=lambda k: breakdown[k][1])
    # Timed region: exactly `steps` steps, HIP events around the dominant kernel's launches only.
    plan.fo_profile_begin_kernel(dom)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        plan.fo_step(gs, x, delta, args.warmup + k)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    prof = plan.fo_profile_end()
    sec = (t_end - t_start) / args.steps
    value = 4.0 * d * M / sec / 1e9

    # roofline of the dominant kernel
    per_kernel = {k: (l, ms) for k, (l, ms) in breakdown.items()}
    launches, total_ms = prof[dom]
    avg_ms = total_ms / launches
    # kernels launched with two different batch sizes per step have a per-step algorithmic figure
    W8 = n // 8
    per_step = {
        "k_strided<ENC_FIRST>": M * (4 * d + 4 * n),
        # with blocks of 2^16 the workers' encode is one pass (k_contig_pair); only the server re-encodes in two
        "k_contig<IN_F32,OUT_PACK>": ((M + 1) if "k_contig_pair" not in per_kernel else 1) * (4 * n + W8),
        "k_contig_pair": M * (4 * d + W8),
        "k_declow": ((M + (0 if "k_decode_pair" in per_kernel else 1)) if args.eps_mode == "independent" else 1) * (W8 + 4 * n),
        "k_strided<SERVER>": (M * 4 * n + 4 * n) if args.eps_mode == "independent" else 8 * n,
        "k_contig<IN_COUNT>": M * W8 + 4 * n,
        "k_mean_tile": M * W8 + 4 * n,
        "k_shall": M * W8 + W8,
        "k_strided<DEC_LAST>": 4 * n + 8 * d,
        "k_contig<IN_GRAD,OUT_PACK>": M * (4 * d + W8) + (4 * n + W8),
        "k_decode_tile": W8 + 8 * d,
        "k_decode_pair": W8 + 8 * d,
    }
    step_bytes = per_step.get(dom)
    bytes_per_launch = step_bytes * args.steps / launches if step_bytes else None
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if bytes_per_launch else None
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": round(achieved, 1) if achieved else None, "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4) if achieved else None,
        "traffic": MEASURED_TRAFFIC.get(dom) if (args.workload == "c3" and args.eps_mode == "independent" and args.K == 1) else None,
        "avg_launch_ms": round(avg_ms, 4), "bytes_per_launch": bytes_per_launch,
        "kernel_ms_per_step": {k: round(ms / nbreak, 4) for k, (l, ms) in sorted(per_kernel.items())},
        "kernel_ms_per_step_from": f"an untimed pass of {nbreak} steps with every kernel bracketed by events",
        "step_model_bytes": sum(v for k, v in per_step.items() if k in per_kernel),
    }
    roofline["step_frac_of_hbm_peak"] = round(roofline["step_model_bytes"] / sec / 1e9 / HBM_PEAK_GBS, 4)
    if copy_gbs:
        roofline["device_copy_gbs"] = round(copy_gbs, 1)   # what a plain copy of 1 GiB reaches on this machine

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fo_oracle as O
        Ms = min(8, M)                                   # bounded sample: the first Ms workers, full d
        nthreads = max(1, min(Ms, 16, os.cpu_count() or 1))
        p = O.params(d=d, M=Ms, block_log2=blk, K=args.K, seed=seed, eps_mode=int(eps_mode), server_scale=int(srv))
        xo = np.zeros(d, dtype=np.float64)
        c0 = time.perf_counter()
        O.round_trip(p, gs_host[:Ms], xo, delta, 0, nthreads=nthreads)
        c1 = time.perf_counter()
        cpu = {"value": round(4.0 * d * Ms / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": nthreads, "kind": "oracle",
               "sample": f"one full round trip of the same workload with the first {Ms} of {M} workers "
                         f"(d={d}, n={n}), fp64; the {Ms} encodes run one per thread, the server and the "
                         f"downlink decode on one thread; {c1 - c0:.1f} s"}

    out = {
        "metric": "GB/s of fp32 gradient encoded+aggregated+decoded; % of HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: d={d} fp32 padded to n={n}, M={M} workers, "
                               f"{'full-length' if blk == 0 else f'blocks of 2^{blk}'} randomized FWHT, uniform dither, "
                               f"L2 scale rule, alpha=alpha_s=2, K={args.K}, {args.eps_mode} eps, server amplitude {args.server_scale}, "
                               f"one fo_step per step",
                   "d": d, "n": n, "M": M, "block_log2": blk},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
