#!/usr/bin/env python3
"""Turn rocprofv3 output into the short tables kept under profiles/.

    python -m paper_2411_07942_amd.profile_summary stats  <..._kernel_stats.csv>
    python -m paper_2411_07942_amd.profile_summary trace  <..._kernel_trace.csv>
    python -m paper_2411_07942_amd.profile_summary pmc    <fetch/..._counter_collection.csv> <write/..._counter_collection.csv> [--traffic-json profiles/traffic.json]

`stats`: calls, average, minimum and maximum duration of every tpq:: kernel.
`trace`: the same from the per-dispatch trace, split by grid size (a kernel launched for one
device and for eight shows up as two lines).
`pmc`: FETCH_SIZE / WRITE_SIZE per dispatch of every tpq:: kernel (KiB, averaged), the factor by
which each counter misreads the known-size copy dispatch of `bench.py --copy-probe`
(torch.bitwise_not over 256 MiB in, 256 MiB out), and the scaled bytes; with --traffic-json
the encode and decode_reduce totals are written where bench.py reads `roofline.traffic` from.
Everything goes to stdout as Markdown.
"""
from __future__ import annotations

import csv
import json
import re
import sys
from collections import defaultdict

PROBE_KIB = 262144.0  # what the copy probe reads, and what it writes


def short(name: str) -> str:
    m = re.search(r"(tpq::\w+(?:<[^>]*>)?)", name)
    return m.group(1) if m else name[:60]


def cmd_stats(path):
    print("| kernel | calls | avg us | min us | max us |\n|---|---|---|---|---|")
    for row in csv.DictReader(open(path)):
        if "tpq::" not in row["Name"]:
            continue
        print("| %s | %s | %.2f | %.2f | %.2f |" % (short(row["Name"]), row["Calls"], float(row["AverageNs"]) / 1e3,
                                                    float(row["MinNs"]) / 1e3, float(row["MaxNs"]) / 1e3))


def cmd_trace(path):
    groups = defaultdict(list)
    for row in csv.DictReader(open(path)):
        if "tpq::" not in row["Kernel_Name"]:
            continue
        grid = (row.get("Grid_Size_X") or row.get("Grid_Size"), row.get("Grid_Size_Y", ""))
        groups[(short(row["Kernel_Name"]), grid)].append((int(row["End_Timestamp"]) - int(row["Start_Timestamp"])) / 1e3)
    print("| kernel | grid (x, y work-items) | launches | avg us | median us | min us |\n|---|---|---|---|---|---|")
    for (name, grid), v in sorted(groups.items()):
        v.sort()
        print("| %s | %s | %d | %.2f | %.2f | %.2f |" % (name, " x ".join(g for g in grid if g), len(v), sum(v) / len(v),
                                                         v[len(v) // 2], v[0]))


def read_counter(path, counter):
    per = defaultdict(list)
    probe = []
    for row in csv.DictReader(open(path)):
        if row["Counter_Name"] != counter:
            continue
        name = row["Kernel_Name"]
        if "bitwise_not" in name:
            probe.append(float(row["Counter_Value"]))
        elif "tpq::" in name:
            per[(short(name), row["Grid_Size"])].append(float(row["Counter_Value"]))
    return per, probe


def cmd_pmc(fetch_path, write_path, traffic_json=None):
    fetch, fprobe = read_counter(fetch_path, "FETCH_SIZE")
    write, wprobe = read_counter(write_path, "WRITE_SIZE")
    if not fprobe or not wprobe:
        raise SystemExit("no copy-probe dispatch in the counter files: run bench.py with --copy-probe")
    f_fac = PROBE_KIB / (sum(fprobe) / len(fprobe))
    w_fac = PROBE_KIB / (sum(wprobe) / len(wprobe))
    print("Scale: the 256 MiB copy probe reads FETCH_SIZE = %.1f, WRITE_SIZE = %.1f => factor %.3f for FETCH_SIZE, %.3f for WRITE_SIZE.\n"
          % (sum(fprobe) / len(fprobe), sum(wprobe) / len(wprobe), f_fac, w_fac))
    print("| kernel | grid | dispatches | FETCH_SIZE | WRITE_SIZE | read MB | written MB | total MB |\n|---|---|---|---|---|---|---|---|")
    totals = {}
    counts = {}
    for key in sorted(set(fetch) | set(write)):
        f = fetch.get(key, [])
        w = write.get(key, [])
        fa = sum(f) / len(f) if f else 0.0
        wa = sum(w) / len(w) if w else 0.0
        rd, wr = fa * f_fac * 1024 / 1e6, wa * w_fac * 1024 / 1e6
        totals[key] = (rd + wr) * 1e6
        counts[key] = max(len(f), len(w))
        print("| %s | %s | %d | %.0f | %.0f | %.1f | %.1f | %.1f |" % (key[0], key[1], max(len(f), len(w)), fa, wa, rd, wr, rd + wr))
    if traffic_json:
        def biggest(prefix):
            # the launch with the largest grid; among kernels with that grid (the accumulate modes
            # of decode_reduce) the one dispatched most often, which is the mode bench.py times
            c = [(int(k[1]), counts[k], v) for k, v in totals.items() if k[0].startswith(prefix)]
            return int(round(max(c)[2], -4)) if c else None
        out = {"tpq_encode": biggest("tpq::k_encode_direct"), "tpq_decode_reduce": biggest("tpq::k_decode_pass"),
               "source": "rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, bytes per launch at the Llama-2-13B-shaped "
                         "prefill workload, scaled by the copy probe (paper_2411_07942_amd/profile_summary.py pmc)"}
        json.dump(out, open(traffic_json, "w"), indent=2)
        open(traffic_json, "a").write("\n")


def main():
    a = sys.argv[1:]
    if len(a) >= 2 and a[0] == "stats":
        cmd_stats(a[1])
    elif len(a) >= 2 and a[0] == "trace":
        cmd_trace(a[1])
    elif len(a) >= 3 and a[0] == "pmc":
        tj = a[a.index("--traffic-json") + 1] if "--traffic-json" in a else None
        cmd_pmc(a[1], a[2], tj)
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main()
