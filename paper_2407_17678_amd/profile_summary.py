"""Turns rocprofv3 counter output into the short summaries kept under profiles/.

    python -m paper_2407_17678_amd.profile_summary traffic WORKLOAD FETCH_CSV WRITE_CSV

reads the two `*counter_collection.csv` files of

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d DIR -o p -- python3 bench.py --workload WORKLOAD \
        --no-cpu-baseline --no-dense --no-extra --no-ceilings --steps 3 --warmup 1 --copy-calibration
    rocprofv3 --pmc WRITE_SIZE ... (same command)

(also: `kernels STATS_CSV` prints the per-kernel table of a --kernel-trace --stats run, `trace
TRACE_CSV` the same per kernel and grid size from the per-dispatch trace, `counters
COUNTER_CSV` the mean of every counter per kernel, `fingerprint` the hash of the kernel sources)

and prints profiles/traffic_WORKLOAD.txt: HBM bytes per launch of each kernel of this library
(FETCH_SIZE and WRITE_SIZE are in KiB per dispatch; each is scaled by what the same counter reads
for the 1 GiB device-to-device copy that --copy-calibration runs first), headed by a fingerprint of
the kernel sources, which bench.py checks before it reports the figures.
"""

import collections
import csv
import hashlib
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")


def source_fingerprint():
    """Hash of everything the kernels are compiled from."""
    h = hashlib.sha1()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def _per_kernel(path, counter):
    """kernel short name -> mean counter value per dispatch; also the copy kernels' mean."""
    sums = collections.defaultdict(list)
    copies = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            name, val = r["Kernel_Name"], float(r["Counter_Value"])
            m = re.search(r"s2::.*?(\w+_kernel)<([^>]*)>", name)
            if m:
                # the dK/dV instantiation that also leaves dS in the workspace (last template argument) is a
                # kernel of its own as far as traffic goes
                keeps = m.group(1) == "dkdv_kernel" and m.group(2).replace(" ", "").endswith(",true")
                sums[m.group(1) + ("_keeping_ds" if keeps else "")].append(val)
            elif "copyBuffer" in name:   # the runtime's device-to-device copy kernel
                copies.append(val)
    # the calibration copy (1 GiB) is the largest device-to-device copy of the run
    return {k: sum(v) / len(v) for k, v in sums.items()}, (max(copies) if copies else None)


def traffic(workload, fetch_csv, write_csv):
    fetch, fcopy = _per_kernel(fetch_csv, "FETCH_SIZE")
    write, wcopy = _per_kernel(write_csv, "WRITE_SIZE")
    if not fcopy or not wcopy:
        raise SystemExit("no calibration copy found: run bench.py with --copy-calibration under the profiler")
    gib_kib = float(1 << 20)
    fs, ws = gib_kib / fcopy, gib_kib / wcopy   # scale factors: the copy reads and writes 1 GiB
    lines = ["# sources %s" % source_fingerprint(),
             "# kernel  HBM bytes per launch (read + written); rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on bench.py "
             "--workload %s, scaled by %.2f / %.2f (1 GiB copy calibration)" % (workload, fs, ws)]
    for k in sorted(set(fetch) | set(write)):
        rd, wr = fetch.get(k, 0.0) * fs * 1024.0, write.get(k, 0.0) * ws * 1024.0
        lines.append("%s %d   # read %d written %d" % (k, round(rd + wr), round(rd), round(wr)))
    return "\n".join(lines) + "\n"


def kernel_stats(stats_csv):
    """Markdown table rows from a `*kernel_stats.csv` of rocprofv3 --kernel-trace --stats."""
    out = ["| kernel | calls | avg ms | min ms | max ms | % of GPU time |", "|---|---|---|---|---|---|"]
    with open(stats_csv) as f:
        for r in csv.DictReader(f):
            m = re.search(r"(\w+_kernel<[^>]*>)", r["Name"])
            if m:
                out.append("| %s | %s | %.3f | %.3f | %.3f | %s |" % (
                    m.group(1), r["Calls"], float(r["AverageNs"]) / 1e6, float(r["MinNs"]) / 1e6,
                    float(r["MaxNs"]) / 1e6, r["Percentage"]))
    return "\n".join(out) + "\n"


def kernel_trace(trace_csv):
    """Markdown table from a `*kernel_trace.csv` of rocprofv3 --kernel-trace: this library's kernels by
    name AND grid size, which tells the workloads of one bench.py run apart (each has its own grid)."""
    agg = collections.defaultdict(list)
    with open(trace_csv) as f:
        for r in csv.DictReader(f):
            m = re.search(r"s2::.*?(\w+_kernel<[^>]*>)", r["Kernel_Name"])
            if m:
                wg = int(r["Workgroup_Size_X"])
                agg[(m.group(1), int(r["Grid_Size_X"]) // wg)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
    out = ["| kernel | workgroups | launches | avg ms | min ms | max ms |", "|---|---|---|---|---|---|"]
    for (k, g), v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        out.append("| %s | %d | %d | %.3f | %.3f | %.3f |" % (k, g, len(v), sum(v) / len(v), min(v), max(v)))
    return "\n".join(out) + "\n"


def counters(counter_csv):
    """Mean value per dispatch of every counter in a `*counter_collection.csv`, per kernel of this library."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(counter_csv) as f:
        for r in csv.DictReader(f):
            m = re.search(r"s2::.*?(\w+_kernel<[^>]*>)", r["Kernel_Name"])
            if m:
                agg[m.group(1)][r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = []
    for k, c in sorted(agg.items()):
        out.append("%s (%d dispatches): %s" % (k, len(next(iter(c.values()))),
                                               ", ".join("%s %.4g" % (n, sum(v) / len(v)) for n, v in sorted(c.items()))))
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) == 3 and sys.argv[1] == "kernels":
        sys.stdout.write(kernel_stats(sys.argv[2]))
    elif len(sys.argv) == 3 and sys.argv[1] == "trace":
        sys.stdout.write(kernel_trace(sys.argv[2]))
    elif len(sys.argv) == 3 and sys.argv[1] == "counters":
        sys.stdout.write(counters(sys.argv[2]))
    elif len(sys.argv) == 5 and sys.argv[1] == "traffic":
        sys.stdout.write(traffic(sys.argv[2], sys.argv[3], sys.argv[4]))
    elif len(sys.argv) == 2 and sys.argv[1] == "fingerprint":
        print(source_fingerprint())
    else:
        raise SystemExit(__doc__)
