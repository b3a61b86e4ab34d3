"""Turns rocprofv3 CSV output of a `bench.py` run into the short text summaries kept under profiles/.

    python -m paper_2603_21090_amd.profile_summary trace  <dir> <bench.json>
    python -m paper_2603_21090_amd.profile_summary traffic <fetch dir> <write dir> <bench.json>
    python -m paper_2603_21090_amd.profile_summary counters <pmc dir> <kernel name part> <last n dispatches>

`trace` reads `*_kernel_stats.csv` and `*_kernel_trace.csv` of a `--kernel-trace --stats` run and
prints the per-kernel table plus, for the layer kernel, the average duration over the launches of
the batch range in which bench.py took its own event timings (`roofline.batches`).

`counters` prints, for the last n dispatches of the kernels whose name contains the given text, the
average of every counter in a `--pmc` run's `*_counter_collection.csv` and the average duration.

`traffic` reads the `*_counter_collection.csv` of one `--pmc FETCH_SIZE` and one `--pmc WRITE_SIZE`
run (both of `bench.py --calibrate-copy`), scales each counter by what it reads for the 1 GiB
elementwise copy at the end of the run, and prints HBM bytes per layer-kernel launch over the same
batch range in the `key = value` form bench.py reads back.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

GIB_KIB = float(1 << 20)


def _one(dirname, pattern):
    hits = sorted(glob.glob(os.path.join(dirname, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit(f"no {pattern} under {dirname}")
    return hits[0]


def _short(name):
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0].replace("stgn::layer_impl::", "").replace("stgn::", "")


def trace(dirname, bench_json):
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    b0, b1 = bench["roofline"]["batches"]
    layers = bench["config"]["layers"]
    print(f"{'kernel':<44}{'calls':>8}{'total ms':>12}{'avg us':>10}{'%':>8}{'min us':>10}{'max us':>10}")
    for r in csv.DictReader(open(_one(dirname, "*kernel_stats.csv"))):
        print(f"{_short(r['Name'])[:43]:<44}{int(r['Calls']):>8}{int(r['TotalDurationNs']) / 1e6:>12.3f}"
              f"{float(r['AverageNs']) / 1e3:>10.2f}{float(r['Percentage']):>8.2f}{int(r['MinNs']) / 1e3:>10.2f}"
              f"{int(r['MaxNs']) / 1e3:>10.2f}")
    rows = list(csv.DictReader(open(_one(dirname, "*kernel_trace.csv"))))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    lay = [r for r in rows if "layer_kernel" in r["Kernel_Name"]]
    dur = [int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in lay]
    # the first `layers` launches are the rebuild at creation; batch b's launches follow those of batch b - 1
    sel = dur[(b0 + 1) * layers:(b1 + 1) * layers]
    print()
    print(f"layer kernel, launches of batches [{b0}, {b1}) ({len(sel)} launches): average "
          f"{sum(sel) / max(len(sel), 1) / 1e3:.2f} us")
    print(f"bench.py's own HIP-event figure for the same launches: {bench['roofline']['avg_launch_us']:.2f} us "
          f"(+ {bench['roofline']['event_overhead_us']:.2f} us event-pair overhead already subtracted)")
    if lay:
        r = lay[len(lay) - 1]
        # fields exactly as the trace reports them: LDS_Block_Size is the static part only (the tiles are
        # dynamic LDS), and the code object's own register count is about twice the VGPR_Count shown
        print(f"layer kernel, trace fields: VGPR_Count {r['VGPR_Count']}, Accum_VGPR_Count {r['Accum_VGPR_Count']}, "
              f"SGPR_Count {r['SGPR_Count']}, LDS_Block_Size {r['LDS_Block_Size']} B (static part), "
              f"Scratch_Size {r['Scratch_Size']} B/lane (no spills), workgroup {r['Workgroup_Size_X']}"
              if r['Scratch_Size'] in ('0', 0) else
              f"layer kernel, trace fields: VGPR_Count {r['VGPR_Count']}, Accum_VGPR_Count {r['Accum_VGPR_Count']}, "
              f"SGPR_Count {r['SGPR_Count']}, LDS_Block_Size {r['LDS_Block_Size']} B (static part), "
              f"Scratch_Size {r['Scratch_Size']} B/lane, workgroup {r['Workgroup_Size_X']}")


def _counter(dirname, counter):
    per = collections.OrderedDict()
    for r in csv.DictReader(open(_one(dirname, "*counter_collection.csv"))):
        if r["Counter_Name"] != counter:
            continue
        key = int(r["Dispatch_Id"])
        ent = per.setdefault(key, [r["Kernel_Name"], 0.0])
        ent[1] += float(r["Counter_Value"])
    return [per[k] for k in sorted(per)]


def traffic(fetch_dir, write_dir, bench_json):
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    b0, b1 = bench["roofline"]["batches"]
    layers = bench["config"]["layers"]
    total = 0.0
    for counter, dirname in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        disp = _counter(dirname, counter)
        lay = [v for n, v in disp if "layer_kernel" in n][(b0 + 1) * layers:(b1 + 1) * layers]   # (creation launches first)
        cal = [v for n, v in disp if "elementwise" in n][-4:]      # the first copy also pages memory in
        cal_mean = sum(cal) / len(cal)
        factor = GIB_KIB / cal_mean
        mean = sum(lay) / len(lay)
        print(f"{counter}: 1 GiB copy kernel reads {cal_mean:.1f} (counter units) -> scale factor {factor:.4f} KiB/unit")
        print(f"{counter}: layer kernel, batches [{b0}, {b1}), {len(lay)} launches: mean {mean:.1f} units "
              f"= {mean * factor * 1024 / 1e6:.3f} MB per launch")
        total += mean * factor * 1024
    algo = bench["roofline"]["achieved"] * 1e9 * bench["roofline"]["avg_launch_us"] * 1e-6
    print(f"algorithmic bytes per launch (bench.py, same batches): {algo / 1e6:.3f} MB")
    print(f"workload = {bench['config']['workload'].split(':')[0]}")
    print(f"batches = [{b0}, {b1}]")
    print(f"traffic_bytes_per_launch = {total:.0f}")


def counters(dirname, name_part, last_n):
    rows = [r for r in csv.DictReader(open(_one(dirname, "*counter_collection.csv"))) if name_part in r["Kernel_Name"]]
    ids = sorted({int(r["Dispatch_Id"]) for r in rows})[-int(last_n):]
    keep = set(ids)
    agg, dur = collections.defaultdict(float), {}
    for r in rows:
        d = int(r["Dispatch_Id"])
        if d in keep:
            agg[r["Counter_Name"]] += float(r["Counter_Value"])
            dur[d] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    print(f"kernel: {_short(rows[0]['Kernel_Name']) if rows else name_part}; last {len(ids)} dispatches; "
          f"average duration {sum(dur.values()) / max(len(dur), 1) / 1e3:.1f} us (kernels run one at a time under --pmc)")
    for k in sorted(agg):
        print(f"  {k:<34}{agg[k] / len(ids):>18.1f}  per dispatch")
    return {k: v / len(ids) for k, v in agg.items()}, sum(dur.values()) / max(len(dur), 1) / 1e3


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "trace":
        trace(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 5 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3], sys.argv[4])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)
