"""Turns the raw rocprofv3 output of `bench.py --traffic-probe` into the short summary that `bench.py` reads.

Usage (the three rocprofv3 runs first, from /tmp with TMPDIR=/tmp, R = the repository root, OUT = a scratch folder for the raw output):

    rocprofv3 --pmc FETCH_SIZE -d $OUT/fetch --output-format csv -- python3 $R/bench.py --traffic-probe
    rocprofv3 --pmc WRITE_SIZE -d $OUT/write --output-format csv -- python3 $R/bench.py --traffic-probe
    rocprofv3 --kernel-trace --stats -d $OUT/kt --output-format csv -- python3 $R/bench.py --steps 200 --no-extras --no-cpu-baseline
    python3 -m paper_2603_02883_amd.profile_summary $OUT $R/profiles/headline_kernel_traffic.txt

The summary is `key: value` lines: the headline kernel's name, FETCH_SIZE / WRITE_SIZE per dispatch (KiB), the
same counters for the plain device copy of known size that calibrates them, the HBM bytes per launch that
follow, and the kernel's average duration in the kernel trace.  Nothing here touches the GPU.
"""

import csv
import glob
import os
import sys

HEADLINE = "quantize_lut_kernel<32, 8, true, false, false, 0, 512>"
COPY_BYTES = 16384 * 3072 * 2          # the probe's device-to-device copy reads and writes this much


def _counter(directory, name):
    """{kernel name: [values]} of one counter from a rocprofv3 --pmc run."""
    out = {}
    for path in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        with open(path) as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] == name:
                    out.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
    return out


def _mean(values):
    return sum(values) / len(values)


def summarize(prof_dir):
    lines = []
    fetch = _counter(os.path.join(prof_dir, "fetch"), "FETCH_SIZE")
    write = _counter(os.path.join(prof_dir, "write"), "WRITE_SIZE")
    head_f = [v for k, v in fetch.items() if HEADLINE in k]
    head_w = [v for k, v in write.items() if HEADLINE in k]
    # the calibration copy: the dispatches of the copy kernel that moved the whole tensor
    copy_f = [x for k, v in fetch.items() if "copyBuffer" in k for x in v if x > 0.4 * COPY_BYTES / 1024]
    copy_w = [x for k, v in write.items() if "copyBuffer" in k for x in v if x > 0.4 * COPY_BYTES / 1024]
    if not (head_f and head_w and copy_f and copy_w):
        raise SystemExit("profile_summary: counters of the headline kernel or of the calibration copy not found in " + prof_dir)
    f_kib, w_kib = _mean(head_f[0]), _mean(head_w[0])
    read_factor = COPY_BYTES / 1024 / _mean(copy_f)
    write_factor = COPY_BYTES / 1024 / _mean(copy_w)
    traffic = int(round((f_kib * read_factor + w_kib * write_factor) * 1024))
    lines.append("kernel: fb4::" + HEADLINE)
    lines.append("workload: cfg2 16384x3072 bf16, fb4_quantize, online selector with 8 groups")
    lines.append("dispatches_counted: %d" % len(head_f[0]))
    lines.append("fetch_size_kib_per_dispatch: %.1f" % f_kib)
    lines.append("write_size_kib_per_dispatch: %.1f" % w_kib)
    lines.append("copy_fetch_size_kib: %.1f" % _mean(copy_f))
    lines.append("copy_write_size_kib: %.1f" % _mean(copy_w))
    lines.append("copy_bytes_each_way: %d" % COPY_BYTES)
    lines.append("read_factor: %.5f" % read_factor)
    lines.append("write_factor: %.5f" % write_factor)
    lines.append("traffic_bytes_per_launch: %d" % traffic)
    lines.append("algorithmic_bytes_per_launch: %d" % (16384 * 3072 * 2 + 16384 * 3072 // 2 + 16384 * 96 * 2))
    for path in glob.glob(os.path.join(prof_dir, "kt", "**", "*kernel_stats.csv"), recursive=True):
        with open(path) as f:
            for row in csv.DictReader(f):
                if HEADLINE in row["Name"]:
                    lines.append("kernel_trace_calls: %s" % row["Calls"])
                    lines.append("kernel_trace_average_ns: %s" % row["AverageNs"])
                    lines.append("kernel_trace_min_ns: %s" % row["MinNs"])
    return lines


def read_summary(path):
    """The summary file as a dict (what bench.py uses); {} if it is not there."""
    out = {}
    try:
        with open(path) as f:
            for line in f:
                if ":" in line and not line.startswith("#"):
                    k, v = line.split(":", 1)
                    out[k.strip()] = v.strip()
    except OSError:
        pass
    return out


if __name__ == "__main__":
    if len(sys.argv) != 3:
        raise SystemExit(__doc__)
    body = summarize(sys.argv[1])
    with open(sys.argv[2], "w") as f:
        f.write("# rocprofv3 summary of the headline kernel; written by paper_2603_02883_amd/profile_summary.py (commands in its header)\n")
        f.write("\n".join(body) + "\n")
    print("\n".join(body))
