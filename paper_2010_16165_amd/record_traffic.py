"""Turns two rocprofv3 counter runs of bench.py into the HBM traffic figure that
bench.py reports for its dominant kernel.

    python -m paper_2010_16165_amd.record_traffic FETCH_DIR WRITE_DIR

FETCH_DIR / WRITE_DIR hold the CSV output of

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d FETCH_DIR -o r -- \
        python3 bench.py --steps 5 --warmup 2 --no-cpu-baseline --no-measured-peaks --copy-calibration 1024
    rocprofv3 --pmc WRITE_SIZE ... (the same command)

Both counters are in KiB per dispatch.  Each is scaled by what the same counter
reads for the plain 1 GiB device-to-device copy that --copy-calibration adds to
the run (a kernel of known traffic: 1 GiB read, 1 GiB written).  The result is
stored beside this file together with a hash of the kernel sources; bench.py
reports it only while the sources still hash to the same value.
"""
import csv
import glob
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
STORE = os.path.join(HERE, "traffic.json")
# what the recorded kernel is compiled from
SOURCES = ["csrc/resident.hip", "csrc/layout.h", "csrc/device_utils.h"]
KERNELS = {"resident_network": "resident_kernel"}
COPY_MIB = 1024


def sources_hash():
    h = hashlib.sha256()
    for rel in SOURCES:
        with open(os.path.join(HERE, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def counter_values(directory, counter):
    """(kernel name, counter value) of every dispatch."""
    rows = []
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] == counter:
                    rows.append((row["Kernel_Name"], float(row["Counter_Value"])))
    return rows


def mean_of(rows, fragment):
    hits = [v for k, v in rows if fragment in k]
    if not hits:
        raise SystemExit(f"no kernel matching {fragment!r} in the counter output")
    return sum(hits) / len(hits)


def largest_of(rows, fragment):
    """The calibration copy is the largest dispatch of the runtime's copy kernel
    (smaller ones are the bench's own uploads)."""
    hits = [v for k, v in rows if fragment in k]
    if not hits:
        raise SystemExit(f"no kernel matching {fragment!r} in the counter output")
    return max(hits)


def main():
    fetch_dir, write_dir = sys.argv[1], sys.argv[2]
    fetch = counter_values(fetch_dir, "FETCH_SIZE")
    write = counter_values(write_dir, "WRITE_SIZE")
    copy_kib = COPY_MIB * 1024.0
    fetch_factor = copy_kib / largest_of(fetch, "copyBuffer")   # true KiB per counted KiB
    write_factor = copy_kib / largest_of(write, "copyBuffer")
    out = {"sources_sha256": sources_hash(), "kernels": {}}
    for name, fragment in KERNELS.items():
        f_kib, w_kib = mean_of(fetch, fragment), mean_of(write, fragment)
        out["kernels"][name] = {
            "fetch_kib_counted": f_kib, "write_kib_counted": w_kib,
            "fetch_factor": fetch_factor, "write_factor": write_factor,
            "bytes_per_launch": 1024.0 * (f_kib * fetch_factor + w_kib * write_factor),
            "workload": "bench.py default (config 1, batch 128)",
        }
    with open(STORE, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
