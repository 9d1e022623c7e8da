"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2410_22249_amd.profile_summary --workload cfg3 \
        --kernel-stats out/kt/cfg3_kernel_stats.csv \
        --fetch out/fetch/cfg3_counter_collection.csv \
        --write out/write/cfg3_counter_collection.csv \
        [--counters some_other_counter_collection.csv ...] --command "<how it was collected>"

HBM traffic: rocprofv3 reports FETCH_SIZE / WRITE_SIZE in KiB per dispatch.  Each is scaled by
what the same counter reads for the plain copy kernel of known size that bench.py launches once
(`copy_kernel`, 1 GiB read + 1 GiB written), so a counter that under- or over-reports by a fixed
factor on this chip is corrected.
"""
from __future__ import annotations

import argparse
import csv
import statistics
import sys
from collections import defaultdict

EMB = ("emb_bag_wave_kernel", "emb_bag_stream_kernel", "emb_bag_fused_kernel",
       "emb_bag_fused_uniform_kernel")   # the forward kernels
COPY = "(anonymous namespace)::copy_kernel("   # the generator's calibration copy, not torch's
CAL_BYTES = 1 << 30


def per_kernel_counter(path):
    """{counter: {kernel_name: [values per dispatch]}}"""
    out = defaultdict(lambda: defaultdict(list))
    for r in csv.DictReader(open(path)):
        out[r["Counter_Name"]][r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return out


def emb_kernels(per):
    """{kernel name: values} of the forward kernels in one counter's per-kernel table.  A call that
    splits into several launches (short-bag tables apart from the others, one launch per row
    class) shows up as several names, each dispatched once per call."""
    return {k: vs for k, vs in per.items() if any(e in k for e in EMB)}


def short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel-stats")
    ap.add_argument("--kernel-trace", help="the per-dispatch trace of the same run")
    ap.add_argument("--last", type=int, default=40,
                    help="dispatches of the forward kernel, counted from the end of the trace, that "
                         "were bench.py's timed steps (warm-up and arena-pick probes come before)")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--counters", action="append", default=[])
    ap.add_argument("--command", action="append", default=[])
    ap.add_argument("--note", action="append", default=[])
    a = ap.parse_args()

    print(f"# rocprofv3 summary: embedding-bag forward, workload {a.workload}")
    for c in a.command:
        print(f"# command: {c}")
    for n in a.note:
        print(f"# note: {n}")

    if a.kernel_stats:
        print("\n## kernel-trace --stats (per kernel)")
        print(f"{'kernel':70s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
        for r in csv.DictReader(open(a.kernel_stats)):
            print(f"{short(r['Name'])[:70]:70s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.1f} "
                  f"{float(r['MinNs']) / 1e3:10.1f} {float(r['MaxNs']) / 1e3:10.1f} "
                  f"{float(r['Percentage']):6.2f}")

    if a.kernel_trace:
        per = defaultdict(list)
        for r in csv.DictReader(open(a.kernel_trace)):
            if any(e in r["Kernel_Name"] for e in EMB):
                per[r["Kernel_Name"]].append((int(r["Start_Timestamp"]), int(r["End_Timestamp"])))
        print(f"\n## the last {a.last} dispatches of each forward kernel (bench.py's timed steps)")
        for k, spans in per.items():
            d = [(e - s) / 1e3 for s, e in sorted(spans)[-a.last:]]
            print(f"{short(k)[:70]:70s} {len(d):6d} {statistics.mean(d):10.1f} {min(d):10.1f} "
                  f"{max(d):10.1f}   (avg_us min_us max_us)")

    traffic = {}
    for label, path, counter in (("fetch", a.fetch, "FETCH_SIZE"), ("write", a.write, "WRITE_SIZE")):
        if not path:
            continue
        data = per_kernel_counter(path)[counter]
        cal = [v for k, vs in data.items() if COPY in k for v in vs]
        emb = emb_kernels(data)
        if not cal or not emb:
            print(f"\n## {counter}: calibration copy or embedding kernel not found in {path}")
            continue
        scale = (CAL_BYTES / 1024.0) / statistics.mean(cal)
        med = sum(statistics.median(vs) for vs in emb.values())
        traffic[label] = med * 1024.0 * scale
        print(f"\n## {counter} (KiB per dispatch as reported)")
        print(f"copy_kernel of {CAL_BYTES} bytes reads {statistics.mean(cal):.1f} -> scale factor {scale:.4f}")
        for k, vs in emb.items():
            print(f"{short(k)[:60]}: n={len(vs)} median {statistics.median(vs):.1f} "
                  f"min {min(vs):.1f} max {max(vs):.1f}")
        if len(emb) > 1:
            print(f"one call = {len(emb)} launches; sum of their medians {med:.1f}")
        print(f"{label}_bytes_per_{'call' if len(emb) > 1 else 'launch'} = {traffic[label]:.0f}")
    if len(traffic) == 2:
        print(f"\nhbm_bytes_per_launch = {traffic['fetch'] + traffic['write']:.0f}"
              "   (all launches of one call)")

    for path in a.counters:
        data = per_kernel_counter(path)
        print(f"\n## counters from {path.split('/')[-2] if '/' in path else path} (embedding kernel, median per dispatch)")
        for counter, per in sorted(data.items()):
            emb = emb_kernels(per)
            for k, vs in emb.items():
                tag = f"   {short(k)[:60]}" if len(emb) > 1 else ""
                print(f"{counter:32s} {statistics.median(vs):18.3f}{tag}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
