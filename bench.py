"""Throughput of the fused + pruned ResNet forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--batch B]

A step is one forward pass of the whole optimised network (every convolution
with its fused epilogue, pools, fc) over one batch already resident in HBM,
replayed from a HIP graph on one stream.  The default workload is the largest
baseline configuration (ResNet-50 shape, fp16, 256 images, irregular pruned
channel counts); the smaller configurations are measured briefly beside it.
Prints one JSON line.

    python bench.py --record-traffic FETCH_DIR WRITE_DIR [--config N]

turns two rocprofv3 counter runs of this script into the HBM-traffic table that
the roofline entries quote (see record_traffic below).
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT = 2.5e15   # dense bf16 / fp16 MFMA, FLOP/s
PEAK_FP32 = 157.3e12       # fp32 vector, FLOP/s
PEAK_HBM = 8.0e12          # B/s

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_kernel.txt")
KERNEL_SOURCES = os.path.join(ROOT, "paper_2010_16165_amd", "csrc")


# ---- HBM traffic measured with rocprofv3 counters ------------------------------------

def sources_hash():
    """Hash of everything the kernels are compiled from: a stored counter value is
    quoted only while the kernels are still the ones it was taken from."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCES)):
        with open(os.path.join(KERNEL_SOURCES, name), "rb") as f:
            h.update(name.encode())
            h.update(f.read())
    return h.hexdigest()[:16]


def group_of_device_kernel(name):
    """The launch-list name (fupr_op_stats.kernel) of a device kernel as rocprofv3
    prints it, from its template arguments; None for kernels that are not the library's."""
    m = re.match(r"(?:void )?(?:fupr::)?(?:\(anonymous namespace\)::)?(\w+)(?:<([^>]*)>)?", name)
    if not m:
        return None
    fn = m.group(1)
    args = [a.strip() for a in (m.group(2) or "").split(",") if a.strip()]
    num = lambda i: int(args[i])
    if fn == "conv1x1_pipe_kernel":
        return f"conv1x1p_{num(1) * num(3) * 16}x{num(2) * num(4) * 16}"
    if fn == "conv1x1_pipe32_kernel":
        return f"conv1x1q_{num(1) * num(3) * 32}x{num(2) * num(4) * 32}"
    if fn == "conv_patch32_kernel":
        return None   # (selected only when forced)
    if fn == "conv_patch_kernel":
        wide = "w" if (num(1), num(2), num(3), num(4)) == (4, 1, 2, 4) else ""
        return f"conv3x3p_{num(1) * num(3) * 16}x{num(2) * num(4) * 16}{wide}"
    if fn == "conv1x1_stream_kernel":
        if len(args) > 3 and num(3) > 0:
            return "conv1x1s_256f+conv1x1"
        return {(16, 2): "conv1x1s_256f", (16, 4): "conv1x1s_256f_c128", (8, 8): "conv1x1s_128f",
                (4, 8): "conv1x1s_64f", (4, 16): "conv1x1s_64f_c512", (2, 8): "conv1x1s_32f"}.get(
                    (num(1), num(2)))
    if fn == "conv16_tiled_kernel":
        return f"conv16t_{num(1) * 64}x{num(2) * 16}"
    return {"stem_pool_kernel": "stem7x7_maxpool", "resident_kernel": "resident_network",
            "maxpool_kernel": "maxpool", "avgpool_kernel": "global_avgpool",
            "conv32_kernel": "conv32_direct"}.get(fn)


def counter_rows(directory, counter):
    rows = []
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] == counter:
                    rows.append((row["Kernel_Name"], float(row["Counter_Value"])))
    return rows


TRAFFIC_HEADER = """\
# HBM bytes per launch of every kernel group, per configuration N, from two counter runs
# (from the repository root, with TMPDIR=/tmp; OUT is any directory for the profiler's output):
#   rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT/pmc_fetch_cN -o r -- \\
#       python3 bench.py --config N --steps 3 --warmup 1 --split 1 --only-headline \\
#       --no-cpu-baseline --no-measured-peaks --copy-calibration 1024
#   rocprofv3 --pmc WRITE_SIZE ... -d OUT/pmc_write_cN ... (the same command)
# folded into this file by
#   python3 bench.py --record-traffic OUT/pmc_fetch_cN OUT/pmc_write_cN --config N
# fetch_bytes / write_bytes: mean counter value per dispatch (KiB) x 1024 x the factor that makes the
# same counter read 1 GiB for the 1 GiB device copy of that run.  sources: hash of the kernel sources.
"""


def record_traffic(fetch_dir, write_dir, config):
    """FETCH_DIR / WRITE_DIR hold the CSV output of

        rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d FETCH_DIR -o r -- \\
            python3 bench.py --config N --steps 3 --warmup 1 --split 1 --only-headline \\
            --no-cpu-baseline --no-measured-peaks --copy-calibration 1024
        rocprofv3 --pmc WRITE_SIZE ... (the same command)

    Both counters are KiB per dispatch.  Each is scaled by what the same counter reads
    for the plain 1 GiB device-to-device copy that --copy-calibration adds to the run (a
    kernel of known traffic).  Per launch-list kernel name: mean bytes per dispatch.
    The lines replace those of the same configuration in profiles/hbm_traffic_per_kernel.txt."""
    fetch, write = counter_rows(fetch_dir, "FETCH_SIZE"), counter_rows(write_dir, "WRITE_SIZE")
    copy_kib = 1024 * 1024.0

    def largest(rows):
        hits = [v for k, v in rows if "copyBuffer" in k or "copy_kernel" in k]
        if not hits:
            raise SystemExit("no calibration copy in the counter output")
        return max(hits)

    f_factor, w_factor = copy_kib / largest(fetch), copy_kib / largest(write)
    per = {}
    for rows, key, factor in ((fetch, "fetch", f_factor), (write, "write", w_factor)):
        for kname, v in rows:
            g = group_of_device_kernel(kname)
            if g:
                e = per.setdefault(g, {"fetch": [], "write": []})
                e[key].append(v * factor * 1024.0)
    lines = []
    if os.path.exists(TRAFFIC_TABLE):
        with open(TRAFFIC_TABLE) as f:
            lines = [ln.rstrip("\n") for ln in f if ln.strip() and not ln.startswith("#")
                     and not ln.startswith(f"config={config} ")]
    for g, e in sorted(per.items()):
        if not e["fetch"] or not e["write"]:
            continue
        fb, wb = sum(e["fetch"]) / len(e["fetch"]), sum(e["write"]) / len(e["write"])
        lines.append(f"config={config} kernel={g} dispatches={len(e['fetch'])} fetch_bytes={fb:.0f} "
                     f"write_bytes={wb:.0f} bytes_per_launch={fb + wb:.0f} fetch_factor={f_factor:.4f} "
                     f"write_factor={w_factor:.4f} sources={sources_hash()}")
    with open(TRAFFIC_TABLE, "w") as f:
        f.write(TRAFFIC_HEADER + "\n".join(lines) + "\n")
    print("\n".join(ln for ln in lines if ln.startswith(f"config={config} ")))


def measured_traffic(config, kernel, default_shape):
    """HBM bytes per launch of a kernel group from the stored counter runs; None when
    there is no record for this configuration and kernel, when the run is not the
    recorded shape (batch, schedule), or when the kernel sources have changed since."""
    if not default_shape or not os.path.exists(TRAFFIC_TABLE):
        return None
    want = sources_hash()
    with open(TRAFFIC_TABLE) as f:
        for ln in f:
            kv = dict(p.split("=", 1) for p in ln.split() if "=" in p)
            if kv.get("config") == str(config) and kv.get("kernel") == kernel and kv.get("sources") == want:
                return float(kv["bytes_per_launch"])
    return None


# ---- the measurements ----------------------------------------------------------------

def cpu_baseline(model, batch, aggressive="off", fuse_stages=None, budget_s=12.0):
    """The CPU oracle (unfused, zero-masked, double precision) timed on the host
    cores over a bounded sample of the same workload: as many images of the
    batch as fit the time budget, and whole passes over them until it is spent."""
    import synth
    from oracle import reference as orc
    if aggressive != "off":
        model = orc.aggressive_fuse(model, stages=fuse_stages)
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


def roofline_of(group_name, g, dt_is_f32, traffic):
    """The roofline entry of a kernel group: algorithmic flops or bytes (whichever
    roof its arithmetic intensity puts it under) over its event-timed duration."""
    peak_flops = PEAK_FP32 if dt_is_f32 else PEAK_MFMA_16BIT
    ridge = peak_flops / PEAK_HBM
    if g["bytes"] and g["flops"] / g["bytes"] >= ridge:
        roof = {"bound": "alu" if dt_is_f32 else "mfma",
                "achieved": g["flops"] / (g["ms"] * 1e-3) / 1e12,
                "peak": peak_flops / 1e12, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": g["bytes"] / (g["ms"] * 1e-3) / 1e9,
                "peak": PEAK_HBM / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = traffic
    roof["kernel"] = group_name
    roof["launches_per_step"] = g["launches"]
    roof["avg_launch_us"] = g["ms"] / g["launches"] * 1e3
    roof["share_of_step"] = g["share"]
    roof["algorithmic_bytes_per_launch"] = g["bytes"] / g["launches"]
    roof["algorithmic_flops_per_launch"] = g["flops"] / g["launches"]
    return roof


class Workload:
    """One configuration built, uploaded and captured; measures itself."""

    def __init__(self, model, batch, args, config_index):
        import torch
        import synth
        from paper_2010_16165_amd import binding as B, network
        self.torch, self.B = torch, B
        self.model, self.batch, self.config_index = model, batch, config_index
        self.dt = B.DTYPES[model["dtype"]]
        plan = network.optimise(model, aggressive=args.aggressive != "off",
                                prune_fused=args.aggressive == "fused-pruned",
                                fuse_stages=args.fuse_stages)
        self.fm, self.sites = network.build(plan)
        if args.schedule == "per-layer":
            self.fm.set_schedule(B.SCHEDULE_PER_LAYER)
        x = synth.make_input(synth.BASE_SEED + max(config_index, 0), batch, model["in_shape"])
        self.xd = B.DeviceTensor.from_nchw(x, self.dt)
        self.stream = torch.cuda.Stream()
        self.sp = B.C.c_void_p(self.stream.cuda_stream)
        with torch.cuda.stream(self.stream):
            self.out, self.ws = self.fm.alloc(batch)
            self.stream.synchronize()
            self.graph = None if args.no_graph else self.fm.fupr_graph_create(self.xd, self.out, self.ws, self.sp)

    def step(self):
        if self.graph is None:
            self.fm.fupr_forward(self.xd, self.out, self.ws, self.sp)
        else:
            self.fm.fupr_graph_launch(self.graph, self.sp)

    def timed_steps(self, steps, warmup):
        """Wall-clock mean over `steps` back-to-back steps (the driver's contract)."""
        torch = self.torch
        with torch.cuda.stream(self.stream):
            for _ in range(warmup):
                self.step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3

    def event_timed_replays(self, replays):
        """Each step bracketed by HIP events on the launch stream: median and minimum."""
        torch = self.torch
        times = []
        with torch.cuda.stream(self.stream):
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                     for _ in range(replays)]
            for a, b in pairs:
                a.record(self.stream)
                self.step()
                b.record(self.stream)
            self.stream.synchronize()
            times = sorted(a.elapsed_time(b) for a, b in pairs)
        return {"median": times[len(times) // 2], "min": times[0], "replays": replays}

    def cold_replays(self, replays=10, flush_mib=512):
        """Steps that start with the caches holding another buffer (a device fill of
        flush_mib between steps evicts L2 and the 256 MB memory-side cache)."""
        torch = self.torch
        times = []
        with torch.cuda.stream(self.stream):
            junk = torch.empty(flush_mib << 20, dtype=torch.uint8, device="cuda")
            for _ in range(replays):
                junk.fill_(1)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(self.stream)
                self.step()
                b.record(self.stream)
                self.stream.synchronize()
                times.append(a.elapsed_time(b))
        times.sort()
        return {"median": times[len(times) // 2], "min": times[0], "replays": replays}

    def per_launch(self, reps=20):
        """Per-launch durations from HIP events around every kernel on the launch stream
        (whole-batch launches, one stream), with each launch's algorithmic work."""
        import numpy as np
        fm = self.fm
        with self.torch.cuda.stream(self.stream):
            fm.fupr_forward_timed(self.xd, self.out, self.ws, self.sp)
            op_ms = np.zeros(fm.num_ops)
            for _ in range(reps):
                op_ms += fm.fupr_forward_timed(self.xd, self.out, self.ws, self.sp)
        op_ms /= reps
        n_launch = fm.num_launches
        stats = [fm.launch_stats(self.batch, i) for i in range(n_launch)]
        return stats, op_ms[:n_launch]

    def launch_site(self, st):
        fm = self.fm
        if st["n_ops"] == fm.num_ops and fm.num_ops > 2:
            return "network"
        names = [str(self.sites[i]) for i in range(st["first_op"], st["first_op"] + st["n_ops"])
                 if self.sites[i] is not None]
        return "+".join(names) if names else "None"

    def groups(self, stats, op_ms):
        total = float(op_ms.sum())
        groups = {}
        for s, ms in zip(stats, op_ms):
            g = groups.setdefault(s["kernel"], {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
            g["ms"] += float(ms)
            g["flops"] += s["flops"]
            g["bytes"] += s["bytes"]
            g["launches"] += 1
        for g in groups.values():
            g["share"] = g["ms"] / total if total else 0.0
        return groups

    def summary(self, ms_per_step, stats, op_ms, default_shape):
        """Network-level rates and the roofline entries of every kernel group, the
        one with the largest share of the time first."""
        B = self.B
        peak = PEAK_FP32 if self.dt == B.F32 else PEAK_MFMA_16BIT
        flops = sum(s["flops"] for s in stats)
        nbytes = sum(s["bytes"] for s in stats)
        groups = self.groups(stats, op_ms)
        rooflines = [roofline_of(name, g, self.dt == B.F32,
                                 measured_traffic(self.config_index, name, default_shape))
                     for name, g in sorted(groups.items(), key=lambda kv: -kv[1]["ms"])]
        return {"workload": self.model["name"], "config_index": self.config_index, "batch": self.batch,
                "dtype": self.model["dtype"], "kernel_launches": self.fm.num_launches,
                "ms_per_step": ms_per_step, "images_per_s": self.batch / (ms_per_step * 1e-3),
                "tflops": flops / (ms_per_step * 1e-3) / 1e12,
                "mfma_frac": flops / (ms_per_step * 1e-3) / peak,
                "algorithmic_gflop_per_step": flops / 1e9, "algorithmic_mb_per_step": nbytes / 1e6,
                "hbm_frac_network": nbytes / (ms_per_step * 1e-3) / PEAK_HBM,
                "roofline": rooflines[0], "kernel_groups": rooflines[1:]}


def measured_peaks(torch, dt_code):
    """What kernels of known work and nothing else reach on this GPU (beside the
    published peaks the roofline entries are priced against): MFMAs on registers
    only, in both instruction shapes, and a 1 GiB device-to-device copy (bytes
    read + bytes written per second)."""
    from paper_2010_16165_amd import measure as M
    out = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mfma_dt = dt_code if dt_code in (1, 2) else 1
    rates = {}
    for shape in (16, 32):
        best = 0.0
        M.fupr_measure_mfma(mfma_dt, shape, 100, 2048, out)
        for _ in range(3):
            start.record()
            flops = M.fupr_measure_mfma(mfma_dt, shape, 20000 if shape == 16 else 10000, 2048, out)
            stop.record()
            stop.synchronize()
            best = max(best, flops / (start.elapsed_time(stop) * 1e-3))
        rates[shape] = best / 1e12
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    best_copy = 0.0
    M.fupr_measure_copy(src, dst, n)
    for _ in range(5):
        start.record()
        M.fupr_measure_copy(src, dst, n)
        stop.record()
        stop.synchronize()
        best_copy = max(best_copy, 2.0 * n / (start.elapsed_time(stop) * 1e-3))
    return {"mfma_tflops": max(rates.values()), "mfma_16x16x32_tflops": rates[16],
            "mfma_32x32x16_tflops": rates[32], "mfma_dtype": "bf16" if mfma_dt == 1 else "f16",
            "copy_gbs": best_copy / 1e9}


def print_per_op(w, stats, op_ms, ms_per_step):
    """Per launch: time, algorithmic work, rates, their share of the published MFMA (or
    fp32 vector) and HBM peaks, and which of the two the operator's arithmetic
    intensity puts it under."""
    peak_flops = PEAK_FP32 if w.dt == w.B.F32 else PEAK_MFMA_16BIT
    ridge = peak_flops / PEAK_HBM
    print(f"{'op':>3} {'site':<18} {'kernel':<21} {'M':>9} {'C':>5} {'K':>5} RxS/s "
          f"{'us':>8} {'GFLOP':>8} {'MB':>8} {'TF/s':>7} {'GB/s':>7} {'%flop':>6} {'%hbm':>6} bound",
          file=sys.stderr)
    for i, (s, ms) in enumerate(zip(stats, op_ms)):
        sec = ms * 1e-3
        bound = "flop" if s["bytes"] and s["flops"] / s["bytes"] >= ridge else "hbm"
        print(f"{i:>3} {w.launch_site(s):<18} {s['kernel']:<21} {s['M']:>9} {s['C']:>5} {s['K']:>5} "
              f"{s['R']}x{s['S']}/{s['stride']} {ms * 1e3:>8.1f} {s['flops'] / 1e9:>8.3f} "
              f"{s['bytes'] / 1e6:>8.2f} {s['flops'] / ms / 1e9:>7.1f} {s['bytes'] / ms / 1e6:>7.0f} "
              f"{100 * s['flops'] / sec / peak_flops:>6.1f} {100 * s['bytes'] / sec / PEAK_HBM:>6.1f} "
              f"{bound}", file=sys.stderr)
    print(f"sum of per-op event times {op_ms.sum() * 1e3:.1f} us; graph step {ms_per_step * 1e3:.1f} us",
          file=sys.stderr)


def filter_tail_point(reps=50):
    """The paper's remark that a layer with 64 filters is often faster than one with
    63 (Sec. VI-B), as one data point of the tail handling here: a 3 x 3 and a 1 x 1
    layer of ResNet-18 / ResNet-50 shape at 64 images with 60 .. 66 filters, microseconds
    per launch by HIP events."""
    import numpy as np
    import torch
    from paper_2010_16165_amd import binding as B
    out = {}
    for name, c, h, r in (("3x3 64->K 56x56 x64", 64, 56, 3), ("1x1 256->K 56x56 x64", 256, 56, 1)):
        row = {}
        xd = B.DeviceTensor.empty(64, h, h, c, B.BF16)
        xd.data.normal_()
        for k in (60, 62, 63, 64, 65, 66):
            w = (np.random.default_rng(k).standard_normal((k, c, r, r)) * 0.05).astype(np.float32)
            sh = B.shape_of(w, 1, r // 2)
            packed = B.upload_blob(B.fupr_pack(sh, w, None, B.BF16))
            yd = B.DeviceTensor.empty(64, h, h, k, B.BF16)
            for _ in range(5):
                B.fupr_conv_fused(sh, xd, packed, None, B.FUSE_RELU, yd)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                B.fupr_conv_fused(sh, xd, packed, None, B.FUSE_RELU, yd)
            b.record()
            b.synchronize()
            row[str(k)] = a.elapsed_time(b) / reps * 1e3
        out[name] = row
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--workload", choices=["resnet20", "resnet32", "resnet18", "resnet34"],
                    help="one of the paper's own networks (Table II) instead of --config; "
                         "batch 1 unless --batch is given (Tables V-VI are batch-1 latencies)")
    ap.add_argument("--permille", type=int, default=300, help="pruning rate of --workload")
    ap.add_argument("--out-permille", type=int, default=0,
                    help="with --workload: pruning rate of the last convolution of every block "
                         "with an identity shortcut (its kept filters add into the full-width "
                         "block output)")
    ap.add_argument("--fuse-stages", type=int, default=None, metavar="X",
                    help="with --aggressive: the paper's fusion option x/n, the first X stages "
                         "are fused (Sec. V, optimization setting); default all")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--schedule", choices=["auto", "per-layer"], default="auto")
    ap.add_argument("--split", type=int, default=0,
                    help="sub-batches of the per-operator schedule (0 = the library's rule)")
    ap.add_argument("--aggressive", choices=["off", "fused", "fused-pruned"], default="off",
                    help="aggressive fusion of the basic blocks (Sec. IV-B): fused = dilated "
                         "convolutions, no additions; fused-pruned = then the n - m prune-back of Alg. 1")
    ap.add_argument("--replays", type=int, default=100,
                    help="event-timed replays for the median / minimum step time")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-op", action="store_true", help="print a per-operator table to stderr")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the measuring kernels (MFMA rate, 1 GiB copy)")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the short runs of the other configurations and the cold replays")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run a plain device-to-device copy of MIB mebibytes (a kernel of "
                         "known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE by)")
    ap.add_argument("--filter-tail-point", action="store_true",
                    help="instead of a workload: time one 3 x 3 and one 1 x 1 layer with 60 .. 66 "
                         "filters (the paper's 63-against-64-filters remark, Sec. VI-B)")
    ap.add_argument("--record-traffic", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU run: turn two rocprofv3 counter outputs into the traffic table")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: images are independent, so N GPUs would each run "
                 "this same forward pass on their share of the batch; run with --gpus 1")
    if args.record_traffic:
        record_traffic(args.record_traffic[0], args.record_traffic[1], args.config)
        return

    import torch
    import synth
    from paper_2010_16165_amd import binding as B

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.filter_tail_point:
        print(json.dumps({"filter_tail_us": filter_tail_point()}))
        return
    if args.split:
        B.fupr_tuning_set("split", args.split)
    if args.workload:
        model, batch = synth.make_paper_workload(args.workload, args.permille,
                                                 out_permille=args.out_permille), 1
        config_index = -1
    else:
        model, batch = synth.make_config(args.config)
        config_index = args.config
    default_batch = batch
    if args.batch:
        batch = args.batch
    # the shape the stored traffic counters were taken at
    default_shape = (batch == default_batch and args.schedule == "auto" and args.aggressive == "off"
                     and not args.workload)

    w = Workload(model, batch, args, config_index)
    ms_per_step = w.timed_steps(args.steps, args.warmup)
    replay = w.event_timed_replays(args.replays)
    stats, op_ms = w.per_launch()
    if args.copy_calibration:
        src = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if args.per_op:
        print_per_op(w, stats, op_ms, ms_per_step)
    head = w.summary(ms_per_step, stats, op_ms, default_shape)

    line = {
        "metric": "images_per_sec_fused_pruned_resnet_fwd",
        "value": head["images_per_s"], "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": model["dtype"], "data": "synthetic",
        "config": {"workload": model["name"], "config_index": config_index, "batch": batch,
                   "kernel_launches": head["kernel_launches"], "schedule": args.schedule,
                   "sub_batches": args.split or "auto",
                   "aggressive_fusion": args.aggressive, "hip_graph": w.graph is not None},
        "tflops": head["tflops"], "mfma_frac": head["mfma_frac"],
        "algorithmic_gflop_per_step": head["algorithmic_gflop_per_step"],
        "algorithmic_mb_per_step": head["algorithmic_mb_per_step"],
        "hbm_frac_network": head["hbm_frac_network"],
        "step_ms_by_events": replay,
        "roofline": head["roofline"],
        "kernel_groups": head["kernel_groups"],
    }
    headline_run = default_shape and config_index == 4
    if not args.only_headline:
        line["step_ms_by_events_cold_caches"] = w.cold_replays()
    if headline_run and not args.only_headline:
        # the smaller configurations of the same path, a few replays each, each with the
        # roofline entries of its own kernels
        del w
        torch.cuda.empty_cache()
        others = []
        for c in (3, 2, 1):
            m2, b2 = synth.make_config(c)
            w2 = Workload(m2, b2, args, c)
            ms2 = w2.timed_steps(40, 5)
            st2, op2 = w2.per_launch(reps=10)
            s2 = w2.summary(ms2, st2, op2, True)
            s2["step_ms_by_events"] = w2.event_timed_replays(args.replays)
            others.append(s2)
            del w2
            torch.cuda.empty_cache()
        line["other_workloads"] = others
    # last, so that the sustained MFMA loop does not heat the chip under the timed runs
    if not args.no_measured_peaks:
        mp = measured_peaks(torch, B.DTYPES[model["dtype"]])
        line["measured_peaks"] = mp
        roof = line["roofline"]
        if roof["unit"] == "GB/s":
            roof["frac_of_measured_peak"] = roof["achieved"] / mp["copy_gbs"]
        elif roof["bound"] == "mfma":
            roof["frac_of_measured_peak"] = roof["achieved"] / mp["mfma_tflops"]
        for o in line.get("other_workloads", []):
            o["mfma_frac_of_measured_peak"] = o["tflops"] / mp["mfma_tflops"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(model, batch, args.aggressive, args.fuse_stages)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
