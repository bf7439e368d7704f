"""Throughput of the fused + pruned ResNet forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--batch B]

A step is one forward pass of the whole optimised network (every convolution
with its fused epilogue, pools, fc) over one batch already resident in HBM,
replayed from a HIP graph on one stream.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT = 2.5e15   # dense bf16 / fp16 MFMA, FLOP/s
PEAK_FP32 = 157.3e12       # fp32 vector, FLOP/s
PEAK_HBM = 8.0e12          # B/s


def cpu_baseline(model, batch, aggressive="off", budget_s=12.0):
    """The CPU oracle (unfused, zero-masked, double precision) timed on the host
    cores over a bounded sample of the same workload: as many images of the
    batch as fit the time budget, and whole passes over them until it is spent."""
    import synth
    from oracle import reference as orc
    if aggressive != "off":
        model = orc.aggressive_fuse(model)
    masks = orc.select_masks(model) if aggressive != "fused" else {}
    seed = synth.BASE_SEED + model.get("config_index", 0)
    x1 = synth.make_input(seed, 1, model["in_shape"])
    orc.forward(model, x1, masks=masks)            # warm-up (library load, page faults)
    t0 = time.perf_counter()
    orc.forward(model, x1, masks=masks)
    t1 = time.perf_counter() - t0
    n = int(max(1, min(batch, budget_s / max(t1, 1e-6))))
    x = synth.make_input(seed, n, model["in_shape"])
    passes, spent = 0, 0.0
    while spent < budget_s and passes < 1000:
        t0 = time.perf_counter()
        orc.forward(model, x, masks=masks)
        spent += time.perf_counter() - t0
        passes += 1
    return {"value": n * passes / spent, "unit": "images/s", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"{n} of {batch} images of the workload, {passes} passes, {spent:.1f} s"}


def quick_measure(config, steps=40, warmup=5):
    """Graph-replay time of another configuration of the same path (context beside
    the headline workload): images/s, TFLOP/s at algorithmic flops."""
    import torch
    import synth
    from paper_2010_16165_amd import binding as B, network
    model, batch = synth.make_config(config)
    dt = B.DTYPES[model["dtype"]]
    fm, _ = network.build(network.optimise(model))
    x = synth.make_input(synth.BASE_SEED + config, batch, model["in_shape"])
    xd = B.DeviceTensor.from_nchw(x, dt)
    stream = torch.cuda.Stream()
    sp = B.C.c_void_p(stream.cuda_stream)
    with torch.cuda.stream(stream):
        out, ws = fm.alloc(batch)
        stream.synchronize()
        graph = fm.fupr_graph_create(xd, out, ws, sp)
        for _ in range(warmup):
            fm.fupr_graph_launch(graph, sp)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fm.fupr_graph_launch(graph, sp)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
    flops = sum(fm.launch_stats(batch, i)["flops"] for i in range(fm.num_launches))
    peak = PEAK_FP32 if dt == B.F32 else PEAK_MFMA_16BIT
    return {"workload": model["name"], "config_index": config, "batch": batch,
            "dtype": model["dtype"], "kernel_launches": fm.num_launches, "ms_per_step": ms,
            "images_per_s": batch / (ms * 1e-3), "tflops": flops / (ms * 1e-3) / 1e12,
            "mfma_frac": flops / (ms * 1e-3) / peak}


def measured_traffic(kernel, args):
    """HBM bytes per launch of the dominant kernel from the stored rocprofv3 counter
    runs (FETCH_SIZE and WRITE_SIZE, each scaled by a copy of known size); None when
    there is no record for this kernel and workload, or when the kernel sources have
    changed since the counters were taken."""
    from paper_2010_16165_amd import record_traffic as rt
    if (args.config != 1 or args.batch or args.schedule != "auto" or args.aggressive != "off"
            or not os.path.exists(rt.STORE)):
        return None
    with open(rt.STORE) as f:
        rec = json.load(f)
    if rec.get("sources_sha256") != rt.sources_hash():
        return None
    entry = rec.get("kernels", {}).get(kernel)
    return entry["bytes_per_launch"] if entry else None


def measured_peaks(B, torch, dt):
    """What two kernels of known work and nothing else reach on this GPU (beside the
    published peaks the roofline entry is priced against): MFMAs on registers only,
    and a 1 GiB device-to-device copy (bytes read + bytes written per second)."""
    out = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mfma_dt = dt if dt in (B.BF16, B.F16) else B.BF16
    best_mfma = 0.0
    B.fupr_measure_mfma(mfma_dt, 100, 2048, out)
    for _ in range(3):
        start.record()
        flops = B.fupr_measure_mfma(mfma_dt, 20000, 2048, out)
        stop.record()
        stop.synchronize()
        best_mfma = max(best_mfma, flops / (start.elapsed_time(stop) * 1e-3))
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    best_copy = 0.0
    B.fupr_measure_copy(src, dst, n)
    for _ in range(5):
        start.record()
        B.fupr_measure_copy(src, dst, n)
        stop.record()
        stop.synchronize()
        best_copy = max(best_copy, 2.0 * n / (start.elapsed_time(stop) * 1e-3))
    return {"mfma_tflops": best_mfma / 1e12, "mfma_dtype": "bf16" if mfma_dt == B.BF16 else "f16",
            "copy_gbs": best_copy / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--workload", choices=["resnet20", "resnet32", "resnet18", "resnet34"],
                    help="one of the paper's own networks (Table II) instead of --config; "
                         "batch 1 unless --batch is given (Tables V-VI are batch-1 latencies)")
    ap.add_argument("--permille", type=int, default=300, help="pruning rate of --workload")
    ap.add_argument("--out-permille", type=int, default=0,
                    help="with --workload: pruning rate of the last convolution of every block "
                         "with an identity shortcut (its kept filters add into the full-width "
                         "block output)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--schedule", choices=["auto", "per-layer"], default="auto")
    ap.add_argument("--aggressive", choices=["off", "fused", "fused-pruned"], default="off",
                    help="aggressive fusion of the basic blocks (Sec. IV-B): fused = dilated "
                         "convolutions, no additions; fused-pruned = then the n - m prune-back of Alg. 1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-op", action="store_true", help="print a per-operator table to stderr")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the two measuring kernels (MFMA rate, 1 GiB copy)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the ImageNet-size configurations")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run a plain device-to-device copy of MIB mebibytes (a kernel of "
                         "known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: images are independent, so N GPUs would each run "
                 "this same forward pass on their share of the batch; run with --gpus 1")

    import numpy as np
    import torch
    import synth
    from paper_2010_16165_amd import binding as B, network

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.workload:
        model, batch = synth.make_paper_workload(args.workload, args.permille,
                                                 out_permille=args.out_permille), 1
        args.config = -1
    else:
        model, batch = synth.make_config(args.config)
    if args.batch:
        batch = args.batch
    dt = B.DTYPES[model["dtype"]]
    plan = network.optimise(model, aggressive=args.aggressive != "off",
                            prune_fused=args.aggressive == "fused-pruned")
    fm, sites = network.build(plan)
    if args.schedule == "per-layer":
        fm.set_schedule(B.SCHEDULE_PER_LAYER)
    x = synth.make_input(synth.BASE_SEED + max(args.config, 0), batch, model["in_shape"])
    xd = B.DeviceTensor.from_nchw(x, dt)

    stream = torch.cuda.Stream()
    sp = B.C.c_void_p(stream.cuda_stream)
    with torch.cuda.stream(stream):
        out, ws = fm.alloc(batch)
        stream.synchronize()
        graph = None if args.no_graph else fm.fupr_graph_create(xd, out, ws, sp)

        def step():
            if graph is None:
                fm.fupr_forward(xd, out, ws, sp)
            else:
                fm.fupr_graph_launch(graph, sp)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

        # per-operator durations from HIP events on the same stream
        reps = 20
        fm.fupr_forward_timed(xd, out, ws, sp)
        op_ms = np.zeros(fm.num_ops)
        for _ in range(reps):
            op_ms += fm.fupr_forward_timed(xd, out, ws, sp)
        op_ms /= reps

    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = elapsed / args.steps * 1e3
    n_launch = fm.num_launches
    stats = [fm.launch_stats(batch, i) for i in range(n_launch)]
    op_ms = op_ms[:n_launch]
    # a launch may cover several operators: name it after them
    def launch_site(st):
        if st["n_ops"] == fm.num_ops and fm.num_ops > 2:
            return "network"
        names = [str(sites[i]) for i in range(st["first_op"], st["first_op"] + st["n_ops"])
                 if sites[i] is not None]
        return "+".join(names) if names else "None"
    sites = [launch_site(st) for st in stats]
    total_flops = sum(s["flops"] for s in stats)
    total_bytes = sum(s["bytes"] for s in stats)
    images_per_s = batch / (ms_per_step * 1e-3)
    tflops = total_flops / (ms_per_step * 1e-3) / 1e12

    groups = {}
    for s, ms in zip(stats, op_ms):
        g = groups.setdefault(s["kernel"], {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
        g["ms"] += ms
        g["flops"] += s["flops"]
        g["bytes"] += s["bytes"]
        g["launches"] += 1
    dom_name, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
    peak_flops = PEAK_FP32 if dt == B.F32 else PEAK_MFMA_16BIT
    ridge = peak_flops / PEAK_HBM
    if dom["flops"] / dom["bytes"] >= ridge:
        roof = {"bound": "mfma" if dt != B.F32 else "alu",
                "achieved": dom["flops"] / (dom["ms"] * 1e-3) / 1e12,
                "peak": peak_flops / 1e12, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": dom["bytes"] / (dom["ms"] * 1e-3) / 1e9,
                "peak": PEAK_HBM / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(dom_name, args)
    roof["kernel"] = dom_name
    roof["launches_per_step"] = dom["launches"]
    roof["avg_launch_us"] = dom["ms"] / dom["launches"] * 1e3
    roof["algorithmic_bytes_per_launch"] = dom["bytes"] / dom["launches"]
    roof["algorithmic_flops_per_launch"] = dom["flops"] / dom["launches"]

    if args.per_op:
        # per launch: time, algorithmic work, rates, their share of the published MFMA (or
        # fp32 vector) and HBM peaks, and which of the two the operator's arithmetic
        # intensity puts it under
        print(f"{'op':>3} {'site':<18} {'kernel':<21} {'M':>9} {'C':>5} {'K':>5} RxS/s "
              f"{'us':>8} {'GFLOP':>8} {'MB':>8} {'TF/s':>7} {'GB/s':>7} {'%flop':>6} {'%hbm':>6} bound",
              file=sys.stderr)
        for i, (s, ms) in enumerate(zip(stats, op_ms)):
            sec = ms * 1e-3
            bound = "flop" if s["bytes"] and s["flops"] / s["bytes"] >= ridge else "hbm"
            print(f"{i:>3} {str(sites[i]):<18} {s['kernel']:<21} {s['M']:>9} {s['C']:>5} {s['K']:>5} "
                  f"{s['R']}x{s['S']}/{s['stride']} {ms * 1e3:>8.1f} {s['flops'] / 1e9:>8.3f} "
                  f"{s['bytes'] / 1e6:>8.2f} {s['flops'] / ms / 1e9:>7.1f} {s['bytes'] / ms / 1e6:>7.0f} "
                  f"{100 * s['flops'] / sec / peak_flops:>6.1f} {100 * s['bytes'] / sec / PEAK_HBM:>6.1f} "
                  f"{bound}", file=sys.stderr)
        print(f"sum of per-op event times {op_ms.sum() * 1e3:.1f} us; graph step {ms_per_step * 1e3:.1f} us",
              file=sys.stderr)

    line = {
        "metric": "images_per_sec_fused_pruned_resnet_fwd",
        "value": images_per_s, "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": model["dtype"], "data": "synthetic",
        "config": {"workload": model["name"], "config_index": args.config, "batch": batch,
                   "kernel_launches": n_launch, "schedule": args.schedule,
                   "aggressive_fusion": args.aggressive,
                   "hip_graph": graph is not None},
        "tflops": tflops, "mfma_frac": tflops * 1e12 / peak_flops,
        "algorithmic_gflop_per_step": total_flops / 1e9,
        "algorithmic_mb_per_step": total_bytes / 1e6,
        "hbm_frac_network": total_bytes / (ms_per_step * 1e-3) / PEAK_HBM,
        "roofline": roof,
    }
    default_run = (args.config == 1 and not args.batch and args.schedule == "auto"
                   and args.aggressive == "off" and not args.workload)
    if default_run and not args.no_other_workloads:
        # the larger configurations of the same path, a few replays each
        del xd, out, ws
        torch.cuda.empty_cache()
        line["other_workloads"] = [quick_measure(c) for c in (2, 3, 4)]
    # last, so that the sustained MFMA loop does not heat the chip under the timed runs
    if not args.no_measured_peaks:
        mp = measured_peaks(B, torch, dt)
        line["measured_peaks"] = mp
        measured = mp["mfma_tflops"] if roof["unit"] == "TFLOP/s" and dt != B.F32 else mp["copy_gbs"]
        if roof["unit"] == "TFLOP/s" and dt == B.F32:
            measured = None      # the fp32 path is plain vector arithmetic, not priced against MFMAs
        roof["frac_of_measured_peak"] = roof["achieved"] / measured if measured else None
        for w in line.get("other_workloads", []):
            w["mfma_frac_of_measured_peak"] = w["tflops"] / mp["mfma_tflops"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(model, batch, args.aggressive)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
