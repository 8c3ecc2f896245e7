"""Short text summaries of rocprofv3 output for this library's kernels.

  python -m paper_2403_10444_amd.profile_summary stats   <kernel_stats.csv>  "<command>"
  python -m paper_2403_10444_amd.profile_summary traffic <fetch_counters.csv> <write_counters.csv> "<commands>"

`stats` lists calls and average / min / max duration of every kernel of the library found in a
`rocprofv3 --kernel-trace --stats` kernel_stats file.  `traffic` turns the FETCH_SIZE and
WRITE_SIZE counters (KiB per dispatch) of two `rocprofv3 --pmc` runs of `bench.py --copy-probe N`
into bytes per call: each counter is scaled by what it reads for the library's plain copy kernel,
which moves a known number of bytes.
"""
from __future__ import annotations

import collections
import csv
import re
import sys

COPY_BYTES = 256 << 20


def _ours(name: str) -> bool:
    return "sv::" in name or "copy_probe_kernel" in name


def _short(name: str) -> str:
    m = re.search(r"(\w+_kernel)(<[^(]*>)?", name)
    if not m:
        return name[:40]
    return m.group(1) + (m.group(2) or "").replace("sv::", "").replace("(anonymous namespace)::", "")


def stats(path: str, command: str) -> str:
    rows = [r for r in csv.DictReader(open(path)) if _ours(r["Name"])]
    out = ["rocprofv3 --kernel-trace --stats: kernels of libspecverify.so (input-generation kernels of torch omitted)",
           "command: " + command, "",
           "%-72s %6s %12s %10s %10s" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns")]
    for r in rows:
        out.append("%-72s %6s %12.1f %10s %10s" % (_short(r["Name"]), r["Calls"], float(r["AverageNs"]), r["MinNs"], r["MaxNs"]))
    return "\n".join(out) + "\n"


def _counter_means(path: str, counter: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter and _ours(r["Kernel_Name"]) and "workspace_init" not in r["Kernel_Name"]:
            acc[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def traffic(fetch_csv: str, write_csv: str, commands: str) -> str:
    out = ["HBM traffic per call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, mean over dispatches),",
           "each scaled by the same counter's reading for copy_probe_kernel, which reads and writes %d bytes" % COPY_BYTES,
           "commands: " + commands, ""]
    total = 0.0
    for label, path, counter in (("read", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        means = _counter_means(path, counter)
        probe = [v for k, v in means.items() if k.startswith("copy_probe_kernel")]
        if not probe:
            raise SystemExit("no copy_probe_kernel dispatch in " + path)
        scale = COPY_BYTES / (probe[0][0] * 1024.0)
        out.append("%s: copy_probe_kernel reads %.1f KiB per dispatch -> scale factor %.4f" % (counter, probe[0][0], scale))
        for k, (mean, n) in sorted(means.items()):
            if k.startswith("copy_probe_kernel"):
                continue
            b = mean * 1024.0 * scale
            total += b
            out.append("  %-70s %s %14.0f bytes per dispatch (n=%d)" % (k, label, b, n))
    out += ["", "traffic_bytes_per_call: %.0f" % total]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "stats":
        sys.stdout.write(stats(sys.argv[2], sys.argv[3]))
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        sys.stdout.write(traffic(sys.argv[2], sys.argv[3], sys.argv[4]))
    else:
        raise SystemExit(__doc__)
