"""Turn rocprofv3 output for one bench.py run into the short text summaries kept under profiles/.

    python -m paper_1705_10591_amd.profile_summary trace   <dir> <bench.json> > profiles/<kernel>_<workload>_kernel_trace.txt
    python -m paper_1705_10591_amd.profile_summary traffic <fetch dir> <write dir> <bench.json> > profiles/<kernel>_<workload>_hbm_traffic.txt

`<dir>` is what `rocprofv3 --kernel-trace --stats -d <dir> --output-format csv -- python3 bench.py
--only <workload> --no-cpu-baseline` wrote, `<bench.json>` the JSON line that run printed.  The
trace summary gives the median, minimum and maximum duration of the TIMED launches only: bench.py
warms up first (by count and by time), and the launches it times are the last `steps` dispatches
of the convolution kernel.  The traffic summary scales FETCH_SIZE and WRITE_SIZE (KiB per
dispatch, one rocprofv3 --pmc run each, bench.py run with --copy-calibration) by what the same
counter reads for a plain 1 GiB device-to-device copy.
"""
from __future__ import annotations

import csv
import glob
import json
import statistics
import sys


def _bench_line(path):
    lines = [l for l in open(path) if l.startswith("{")]
    return json.loads(lines[-1])


def _name(b):
    """The workload's name as bench.py --only takes it."""
    return b["config"]["workload"].split(":")[0]


def _dispatches(d):
    rows = []
    for f in glob.glob(d + "/**/*kernel_trace.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
    rows.sort()
    return rows


def trace(d, bench_json):
    b = _bench_line(bench_json)
    steps = int(b["steps"])
    rows = _dispatches(d)
    conv = [(s, e, n) for s, e, n in rows if "dconv::" in n and "clear_counters" not in n]
    if not conv:
        raise SystemExit("no convolution kernel in the trace")
    # the dominant kernel: the one with the largest total time
    total = {}
    for s, e, n in conv:
        total[n] = total.get(n, 0) + e - s
    name = max(total, key=total.get)
    mine = [e - s for s, e, n in conv if n == name]
    timed = mine[-steps:]
    warm = mine[:-steps]
    r = b["roofline"]
    out = [
        f"# rocprofv3 kernel trace: {r['kernel']} on workload {b['config']['workload']}",
        "# command (from /tmp, TMPDIR=/tmp): rocprofv3 --kernel-trace --stats -d <dir> --output-format csv -- "
        f"python3 bench.py --only {_name(b)} --steps {steps} --warmup {b['warmup']} --no-cpu-baseline",
        "# summary: python -m paper_1705_10591_amd.profile_summary trace <dir> <bench.json>",
        f"# bench.py line of the same run (HIP events over the {steps} timed launches): kernel_ms={r['kernel_ms']} "
        f"value={b['value']} {b['unit']} roofline={r['bound']} achieved={r['achieved']} {r['unit']} "
        f"frac={r['frac']}",
        f"kernel: {name}",
        f"timed launches (the last {len(timed)} dispatches): median {statistics.median(timed) / 1e3:.2f} us | "
        f"min {min(timed) / 1e3:.2f} us | max {max(timed) / 1e3:.2f} us | mean {statistics.fmean(timed) / 1e3:.2f} us",
    ]
    if warm:
        out.append(f"warm-up launches before them (not part of any figure): {len(warm)} dispatches | "
                   f"median {statistics.median(warm) / 1e3:.2f} us | max {max(warm) / 1e3:.2f} us")
    med_ms = statistics.median(timed) / 1e6
    ach = r["achieved"] * r["kernel_ms"] / med_ms      # (the line's rate is work / kernel_ms)
    out.append(f"from the median: achieved {ach:.1f} {r['unit']} = {ach / r['peak']:.4f} of the published peak "
               f"({r['peak']} {r['unit']})")
    others = {}
    for s, e, n in rows:
        if n != name:
            others.setdefault(n, []).append(e - s)
    for n, v in sorted(others.items(), key=lambda kv: -sum(kv[1]))[:4]:
        out.append(f"other kernel: {n[:110]} | {len(v)} dispatches | total {sum(v) / 1e3:.1f} us")
    print("\n".join(out))


def _counter(d):
    agg = {}
    for f in glob.glob(d + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            agg.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return agg


def traffic(fetch_dir, write_dir, bench_json):
    b = _bench_line(bench_json)
    r = b["roofline"]
    out = [
        f"# HBM traffic of {r['kernel']} on workload {b['config']['workload']} from rocprofv3 counters (KiB per dispatch)",
        "# commands (from /tmp, TMPDIR=/tmp): rocprofv3 --pmc FETCH_SIZE -d <fetch dir> --output-format csv -- python3 bench.py "
        f"--only {_name(b)} --steps 5 --warmup 2 --no-cpu-baseline --copy-calibration",
        "#                                    rocprofv3 --pmc WRITE_SIZE -d <write dir> --output-format csv -- python3 bench.py "
        f"--only {_name(b)} --steps 5 --warmup 2 --no-cpu-baseline --copy-calibration",
        "# summary: python -m paper_1705_10591_amd.profile_summary traffic <fetch dir> <write dir> <bench.json>",
        "# calibration: a plain device-to-device copy of 2^28 floats (1 GiB = 1048576 KiB read, the same written), "
        "the copy kernel torch launches for Tensor.copy_",
    ]
    res = {}
    for d, cname in ((fetch_dir, "FETCH_SIZE"), (write_dir, "WRITE_SIZE")):
        agg = _counter(d)
        conv = [k for k in agg if "dconv::" in k and "clear_counters" not in k]
        conv.sort(key=lambda k: -sum(agg[k]))
        for k in agg:
            v = agg[k]
            out.append(f"{cname} | {k[:100]} | dispatches {len(v)} | mean {sum(v) / len(v):.1f} KiB | "
                       f"min {min(v):.1f} | max {max(v):.1f}")
        cal = None
        for k in agg:
            if "copy" in k.lower() or "elementwise" in k.lower():
                big = [v for v in agg[k] if v > 500000]
                if big:
                    cal = sum(big) / len(big)
        cv = statistics.median(agg[conv[0]]) if conv else None
        res[cname] = (cv, cal)
    (fc, fcal), (wc, wcal) = res["FETCH_SIZE"], res["WRITE_SIZE"]
    fs = 1048576.0 / fcal if fcal else 1.0
    ws = 1048576.0 / wcal if wcal else 1.0
    out.append(f"scale factors (known / read): FETCH_SIZE {fs:.4f}, WRITE_SIZE {ws:.4f}")
    out.append(f"fetched_bytes_per_launch: {fc * fs * 1024.0:.0f}")
    out.append(f"written_bytes_per_launch: {wc * ws * 1024.0:.0f}")
    out.append(f"traffic_bytes_per_launch: {(fc * fs + wc * ws) * 1024.0:.0f}")
    print("\n".join(out))


if __name__ == "__main__":
    if len(sys.argv) == 4 and sys.argv[1] == "trace":
        trace(sys.argv[2], sys.argv[3])
    elif len(sys.argv) == 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)
