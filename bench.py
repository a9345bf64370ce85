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

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def measured_traffic(workload, block_log2, eps_mode, K, kernel):
    """HBM bytes per launch of `kernel` as rocprofv3 --pmc measured them (FETCH_SIZE, WRITE_SIZE, each scaled by what
    the same counter reads for a 1 GiB copy), from the table kept next to the rocprofv3 summaries under profiles/.
    Returns (bytes, source file) or (None, None) when the table has no row for this workload and kernel."""
    try:
        lines = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None, None
    for ln in lines:
        f = ln.split()
        if len(f) < 7 or ln.startswith("#"):
            continue
        if (f[0], int(f[1]), f[2], int(f[3]), f[4]) == (workload, block_log2, eps_mode, K, kernel):
            return int(f[5]), f[6]
    return None, None


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
    ap.add_argument("--server-scale", default="thm", choices=["thm", "l2", "sup"],
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
    srv = {"thm": B.SERVER_SCALE_THM, "l2": B.SERVER_SCALE_L2, "sup": B.SERVER_SCALE_SUP}[args.server_scale]
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
    # Median step time, from a second pass of `steps` steps with one event between steps (kept out of the timed
    # region above: an event keeps the next step's first kernel from overlapping the tail of the last one).
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the launch stream
    marks[0].record()
    for k in range(args.steps):
        plan.fo_step(gs, x, delta, 2000 + k)
        marks[k + 1].record()
    torch.cuda.synchronize()
    step_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    med_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])

    # roofline of the dominant kernel
    per_kernel = {k: (l, ms) for k, (l, ms) in breakdown.items()}
    launches, total_ms = prof[dom]
    avg_ms = total_ms / launches
    # Bytes per step, per kernel.  `model`: the two-pass byte model the workload is priced with (every operand once,
    # 4-byte intermediates between passes).  `moved`: the operands as this build lays them out (the decode side's
    # intermediates are int16), i.e. what the kernels have to move through HBM; rocprofv3's counters agree with it.
    W8 = n // 8
    ind = args.eps_mode == "independent"
    pair = "k_contig_pair" in per_kernel
    n_low = (M + 1) if not pair else 1                       # vectors through the encode's low pass
    n_dlow = (M + (0 if "k_decode_pair" in per_kernel else 1)) if ind else 1
    model = {
        "k_strided<ENC_FIRST>": M * (4 * d + 4 * n),
        # with blocks of 2^16 the workers' encode is one pass (k_contig_pair); only the server re-encodes in two
        "k_contig<IN_F32,OUT_PACK>": n_low * (4 * n + W8),
        # blocks of 2^16: the server's re-encode of the mean is one more vector through the pair kernel
        "k_contig_pair": M * (4 * d + W8) + ((4 * n + W8) if "k_mean_mfma" in per_kernel else 0),
        "k_declow": n_dlow * (W8 + 4 * n),
        "k_strided<SERVER>": (M * 4 * n + 4 * n) if ind else 8 * n,
        "k_server_mfma": M * 4 * n + 4 * n,
        "k_contig<IN_COUNT>": M * W8 + 4 * n,
        "k_mean_mfma": M * W8 + 4 * n,
        "k_shall": M * W8 + W8,
        "k_strided<DEC_LAST>": 4 * n + 8 * d,
        "k_contig<IN_GRAD,OUT_PACK>": M * (4 * d + W8) + (4 * n + W8 if "k_mean_mfma" in per_kernel else 0),
        "k_decode_tile": W8 + 8 * d,
        "k_decode_pair": W8 + 8 * d,
    }
    moved = dict(model)
    moved["k_declow"] = n_dlow * (W8 + 2 * n)
    moved["k_strided<SERVER>"] = (M * 2 * n + 4 * n) if ind else 8 * n
    moved["k_server_mfma"] = M * 2 * n + 4 * n
    moved["k_strided<DEC_LAST>"] = 2 * n + 8 * d
    step_bytes = model.get(dom)
    bytes_per_launch = step_bytes * args.steps / launches if step_bytes else None
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if bytes_per_launch else None
    traffic, traffic_src = measured_traffic(args.workload, blk, args.eps_mode, args.K, dom)
    step_model = sum(v for k, v in model.items() if k in per_kernel)
    step_moved = sum(v for k, v in moved.items() if k in per_kernel)
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": round(achieved, 1) if achieved else None, "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4) if achieved else None,
        "traffic": traffic, "traffic_source": traffic_src,
        "avg_launch_ms": round(avg_ms, 4), "bytes_per_launch": bytes_per_launch,
        "kernel_ms_per_step": {k: round(ms / nbreak, 4) for k, (l, ms) in sorted(per_kernel.items())},
        "kernel_ms_per_step_from": f"an untimed pass of {nbreak} steps with every kernel bracketed by events",
        # whole step: the headline fraction is on the bytes this build moves; the model's bytes are given beside it
        "step_moved_bytes": step_moved, "step_model_bytes": step_model,
        "step_frac_of_hbm_peak": round(step_moved / sec / 1e9 / HBM_PEAK_GBS, 4),
        "step_frac_of_hbm_peak_on_model_bytes": round(step_model / sec / 1e9 / HBM_PEAK_GBS, 4),
    }
    if copy_gbs:
        roofline["device_copy_gbs"] = round(copy_gbs, 1)   # what a plain copy of 1 GiB reaches on this machine

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fo_oracle as O
        Ms = M                                           # the whole round: all M workers, full d
        nthreads = max(1, min(Ms, 16, os.cpu_count() or 1))
        p = O.params(d=d, M=Ms, block_log2=blk, K=args.K, seed=seed, eps_mode=int(eps_mode), server_scale=int(srv))
        xo = np.zeros(d, dtype=np.float64)
        c0 = time.perf_counter()
        O.round_trip(p, gs_host[:Ms], xo, delta, 0, nthreads=nthreads)
        c1 = time.perf_counter()
        cpu = {"value": round(4.0 * d * Ms / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": nthreads, "kind": "oracle",
               "sample": f"one full round trip of the same workload, all {M} workers (d={d}, n={n}), fp64; the "
                         f"encodes run one per thread on {nthreads} threads, the server and the downlink decode on "
                         f"one thread; {c1 - c0:.1f} s"}

    out = {
        "metric": "GB/s of fp32 gradient encoded+aggregated+decoded; % of HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4), "ms_per_step_median": round(med_ms, 4),
        "value_at_median_step": round(4.0 * d * M / (med_ms * 1e-3) / 1e9, 2), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
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
