"""Turn rocprofv3 CSV output into the short summaries kept with the benchmark.

  python -m paper_2409_20156_amd.profsum stats  <kernel_stats.csv> <out.md> "<title>" "<command>"
  python -m paper_2409_20156_amd.profsum pmc    <workload> <fetch counter csv> <write counter csv>
                                                <copy MiB> <out.md> <traffic.json> "<commands>"
  python -m paper_2409_20156_amd.profsum sq     <counter csv> <out.md> "<title>" "<command>"

`stats` lists the library's kernels from a `--kernel-trace --stats` run.  `pmc` averages
FETCH_SIZE and WRITE_SIZE (KiB per dispatch) per library kernel, scales each by what the same
counter read for the plain copy kernel of known size in the same run, and writes bytes per
launch into the JSON file the benchmark reads; for the search it also writes the bytes of one
whole search (all tile-kernel launches between two `mine_init` launches) and says whether the
searches of the run started from scratch or from earlier thresholds.  `sq` turns one run with the shader counters
SQ_VALU_MFMA_BUSY_CYCLES, SQ_INSTS_VALU_MFMA_MOPS_BF16, SQ_BUSY_CU_CYCLES, SQ_WAVE_CYCLES, SQ_WAIT_ANY
and GRBM_GUI_ACTIVE into matrix-pipe utilisation, the share of their time waves spend waiting, and
the shader clock.
"""
from __future__ import annotations

import csv
import json
import os
import sys
from collections import defaultdict

# kernel function name -> name used by the benchmark
KERNELS = {"mine_tile_kernel": "mine_tile", "mine_rows_kernel": "mine_tile", "mine_select_kernel": "mine_select",
           "mine_init_kernel": "mine_init", "mine_warm_init_kernel": "mine_warm_init",
           "sample_kernel": "sample", "gather_kernel": "gather", "radix_count_kernel": "radix_count",
           "radix_prefix_kernel": "radix_scan", "radix_scatter_kernel": "radix_scatter",
           "bucket_sort_kernel": "bucket_sort",
           "heads_count_kernel": "heads_count", "heads_write_kernel": "heads_write",
           "update_kernel": "update", "copy_probe_kernel": "copy_probe", "mfma_probe_kernel": "mfma_probe"}

kXcds, kSimds = 8, 1024          # MI355X: one GRBM per XCD; 256 CUs x 4 SIMDs


def short_name(full: str):
    if "xc::" not in full:
        return None
    fn = full.split("xc::")[1].split("(")[0].split("<")[0]
    return KERNELS.get(fn, fn)


def stats(src, out, title, cmd, trace=None):
    rows = list(csv.DictReader(open(src)))
    agg = defaultdict(lambda: [0, 0, 1 << 62, 0, 0.0])
    for r in rows:
        n = short_name(r["Name"])
        if n is None:
            continue
        a = agg[n]
        a[0] += int(r["Calls"])
        a[1] += int(r["TotalDurationNs"])
        a[2] = min(a[2], int(r["MinNs"]))
        a[3] = max(a[3], int(r["MaxNs"]))
        a[4] += float(r["Percentage"])
    with open(out, "w") as f:
        f.write("# %s\n\nCommand (on the MI355X box, from the repository root):\n\n```\n%s\n```\n\n" % (title, cmd))
        f.write("rocprofv3 kernel statistics of the library's kernels (template instances of one kernel "
                "summed; torch's input-generator kernels omitted):\n\n")
        f.write("| kernel | calls | total ms | avg us | min us | max us | % of all GPU time |\n|---|---|---|---|---|---|---|\n")
        for n, a in sorted(agg.items(), key=lambda kv: -kv[1][1]):
            f.write("| %s | %d | %.3f | %.2f | %.2f | %.2f | %.2f |\n"
                    % (n, a[0], a[1] / 1e6, a[1] / a[0] / 1e3, a[2] / 1e3, a[3] / 1e3, a[4]))
        if trace:
            f.write(_searches(trace))


def _searches(trace):
    """The mine_tile launches of the trace grouped into searches (a run of mining kernels between other
    kernels of the library)."""
    rows = [r for r in csv.DictReader(open(trace)) if short_name(r["Kernel_Name"]) is not None]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    groups, cur = [], []
    for r in rows:
        n = short_name(r["Kernel_Name"])
        if n.startswith("mine_"):
            if n == "mine_tile":
                cur.append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        elif n not in ("copy_probe", "mfma_probe"):
            if cur:
                groups.append(cur)
            cur = []
    if cur:
        groups.append(cur)
    by = defaultdict(list)
    for g in groups:
        by[len(g)].append(g)
    out = ["\nmine_tile launches grouped by search (one search = the mining kernels between two steps: one launch per phase "
           "of a search from scratch; a search started from earlier thresholds has one sweep and then the same launches, "
           "which return at once). `bench.py` reports the mean total per search from its own HIP events:\n\n",
           "| launches per search | searches | mean total us | mean per launch us | longest launch us |\n|---|---|---|---|---|\n"]
    for k in sorted(by):
        gs = by[k]
        tot = sum(sum(g) for g in gs) / len(gs)
        out.append("| %d | %d | %.1f | %.1f | %.1f |\n" % (k, len(gs), tot / 1e3, tot / k / 1e3, max(max(g) for g in gs) / 1e3))
    return "".join(out)


def _counter_means(path, counter):
    tot, cnt = defaultdict(float), defaultdict(int)
    for r in csv.DictReader(open(path)):
        if r.get("Counter_Name") != counter:
            continue
        n = short_name(r["Kernel_Name"])
        if n is None:
            continue
        tot[n] += float(r["Counter_Value"])
        cnt[n] += 1
    return {n: tot[n] / cnt[n] for n in tot}, dict(cnt)


def pmc(workload, fetch_csv, write_csv, copy_mib, out, traffic_json, cmd):
    fetch, nf = _counter_means(fetch_csv, "FETCH_SIZE")
    write, _ = _counter_means(write_csv, "WRITE_SIZE")
    copy_kib = float(copy_mib) * 1024.0
    kf = copy_kib / fetch["copy_probe"]          # true KiB per counted KiB, reads
    kw = copy_kib / write["copy_probe"]
    result = {}
    with open(out, "w") as f:
        f.write("# HBM traffic per launch, workload %s\n\nCommands (on the MI355X box, from the repository root):\n\n```\n%s\n```\n\n"
                % (workload, cmd))
        f.write("The copy kernel moved %s MiB each way; the counters read %.1f KiB (FETCH_SIZE) and %.1f KiB "
                "(WRITE_SIZE) for it, so the scale factors are %.4f and %.4f.\n\n"
                % (copy_mib, fetch["copy_probe"], write["copy_probe"], kf, kw))
        f.write("| kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled read MB | scaled written MB |\n|---|---|---|---|---|---|\n")
        for n in sorted(fetch, key=lambda n: -fetch[n]):
            rd = fetch[n] * kf * 1024.0
            wr = write.get(n, 0.0) * kw * 1024.0
            f.write("| %s | %d | %.1f | %.1f | %.3f | %.3f |\n" % (n, nf[n], fetch[n], write.get(n, 0.0), rd / 1e6, wr / 1e6))
            if n != "copy_probe":
                result[n] = {"read_bytes": rd, "write_bytes": wr, "bytes": rd + wr}
        if "mine_tile" in fetch and nf.get("mine_init"):
            # every search launches mine_init once; a search started from earlier thresholds also mine_warm_init
            searches, warm = nf["mine_init"], nf.get("mine_warm_init", 0)
            mode = "from scratch" if warm == 0 else ("from earlier thresholds" if warm == searches else
                                                      "%d from scratch, %d from earlier thresholds" % (searches - warm, warm))
            per = nf["mine_tile"] / searches
            r = result["mine_tile"]
            r.update({"searches": searches, "search_mode": mode, "launches_per_search": per,
                      "read_bytes_per_search": r["read_bytes"] * per, "write_bytes_per_search": r["write_bytes"] * per,
                      "bytes_per_search": r["bytes"] * per})
            f.write("\nThe run held %d search(es), %s: %.1f tile-kernel launches per search, %.3f GB read and %.3f GB "
                    "written per search.\n" % (searches, mode, per, r["read_bytes_per_search"] / 1e9,
                                               r["write_bytes_per_search"] / 1e9))
    data = {}
    if os.path.exists(traffic_json):
        data = json.load(open(traffic_json))
    data[workload] = result
    json.dump(data, open(traffic_json, "w"), indent=1, sort_keys=True)


def sq(src, out, title, cmd):
    """Per kernel, over all its dispatches: sums of the counters and of the durations.

    GRBM_GUI_ACTIVE is reported summed over the 8 XCDs, in shader clocks, and covers the dispatch plus
    about 12 us of counter set-up, so the clock is taken from dispatches longer than 0.4 ms only.
    SQ_VALU_MFMA_BUSY_CYCLES is in clocks summed over SIMDs (32 per 32x32x16 bf16 MFMA: its 8 passes);
    SQ_BUSY_CU_CYCLES, SQ_WAVE_CYCLES and SQ_WAIT_ANY are in units of 4 clocks.
    """
    tot = defaultdict(lambda: defaultdict(float))
    dur = defaultdict(dict)
    for r in csv.DictReader(open(src)):
        n = short_name(r["Kernel_Name"])
        if n is None:
            continue
        tot[n][r["Counter_Name"]] += float(r["Counter_Value"])
        dur[n][r["Dispatch_Id"]] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"]), r["Dispatch_Id"])
    long_gui = defaultdict(float)
    long_ns = defaultdict(float)
    for r in csv.DictReader(open(src)):
        n = short_name(r["Kernel_Name"])
        if n is None or r["Counter_Name"] != "GRBM_GUI_ACTIVE":
            continue
        ns = dur[n][r["Dispatch_Id"]][0]
        if ns > 400000:
            long_gui[n] += float(r["Counter_Value"]) / kXcds
            long_ns[n] += ns
    with open(out, "w") as f:
        f.write("# %s\n\nCommand (on the MI355X box, from the repository root):\n\n```\n%s\n```\n\n" % (title, cmd))
        f.write("Sums over all dispatches of a kernel. *matrix pipe busy* = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x "
                "GRBM_GUI_ACTIVE / 8 XCDs), the profiler's own MfmaUtil formula; *of CU-busy time* divides by "
                "4 x SQ_BUSY_CU_CYCLES instead (leaves out launch ramps and idle CUs); *waves waiting* = SQ_WAIT_ANY / "
                "SQ_WAVE_CYCLES; *MFMA TFLOP* = 512 x SQ_INSTS_VALU_MFMA_MOPS_BF16; *clock* = GRBM_GUI_ACTIVE / 8 / "
                "duration over the dispatches longer than 0.4 ms.\n\n")
        f.write("| kernel | dispatches | total ms | MFMA TFLOP | matrix pipe busy | of CU-busy time | waves waiting | clock GHz |\n"
                "|---|---|---|---|---|---|---|---|\n")
        for n in sorted(tot, key=lambda n: -sum(d[0] for d in dur[n].values())):
            c = tot[n]
            ns = sum(d[0] for d in dur[n].values())
            gui = c["GRBM_GUI_ACTIVE"] / kXcds
            busy = 4.0 * c["SQ_BUSY_CU_CYCLES"]          # clocks summed over SIMDs
            clock = "%.2f" % (long_gui[n] / long_ns[n]) if long_ns[n] else "-"
            f.write("| %s | %d | %.3f | %.3f | %.3f | %.3f | %.3f | %s |\n"
                    % (n, len(dur[n]), ns / 1e6, 512.0 * c["SQ_INSTS_VALU_MFMA_MOPS_BF16"] / 1e12,
                       c["SQ_VALU_MFMA_BUSY_CYCLES"] / (kSimds * gui) if gui else 0.0,
                       c["SQ_VALU_MFMA_BUSY_CYCLES"] / busy if busy else 0.0,
                       c["SQ_WAIT_ANY"] / c["SQ_WAVE_CYCLES"] if c["SQ_WAVE_CYCLES"] else 0.0, clock))


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "stats":
        stats(*sys.argv[2:7])
    elif len(sys.argv) >= 2 and sys.argv[1] == "pmc":
        pmc(*sys.argv[2:9])
    elif len(sys.argv) >= 2 and sys.argv[1] == "sq":
        sq(*sys.argv[2:6])
    else:
        sys.exit(__doc__)
