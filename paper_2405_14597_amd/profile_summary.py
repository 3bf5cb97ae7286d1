"""Reduces rocprofv3 CSV output of a bench.py run to the short text summaries kept under profiles/.

    python -m paper_2405_14597_amd.profile_summary trace   <kernel_stats.csv> --command "<the profiled command>"
    python -m paper_2405_14597_amd.profile_summary traffic <fetch counter_collection.csv> <write counter_collection.csv>
                                                           --command "<the profiled command>"
    python -m paper_2405_14597_amd.profile_summary counters <counter_collection.csv> [more passes ...] --command "..."

`trace`: per kernel of this library, dispatches, average duration and share of GPU time (rocprofv3 --kernel-trace
--stats --output-format csv writes <prefix>_kernel_stats.csv).

`traffic`: HBM bytes per dispatch from two counter passes (rocprofv3 --pmc FETCH_SIZE, then --pmc WRITE_SIZE; the
counters are in KiB per dispatch up to a factor that depends on the chip's cache-line accounting).  The factor is
taken from two kernels of known size in the same run: bench.py's streaming-read probe (stream_read_kernel reads
1 GiB) calibrates FETCH_SIZE, and its 1 GiB fill before the probe (torch's fill kernel) calibrates WRITE_SIZE.  The
lines `TRAFFIC <kernel> <bytes>` are what bench.py looks up for `roofline.traffic`.

`counters`: per kernel, the average of every counter found in the passes (SQ_* and the like), one column each.
"""
from __future__ import annotations

import argparse
import collections
import csv
import sys

GIB = 1 << 30


def short(name: str) -> str:
    """Kernel name without namespaces and argument list (templates kept)."""
    name = name.replace("void intscale::(anonymous namespace)::", "").replace("intscale::(anonymous namespace)::", "")
    name = name.replace("void intscale::", "").replace("intscale::", "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return name[:i]
    return name


def read_counters(path):
    """{kernel: {counter: (average per dispatch, dispatches, largest dispatch)}} of one counter-collection CSV."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (sum(v) / len(v), len(v), max(v)) for c, v in cs.items()} for k, cs in acc.items()}


def ours(name: str) -> bool:
    return "intscale::" in name


def cmd_trace(args):
    rows = []
    with open(args.files[0], newline="") as f:
        for r in csv.DictReader(f):
            if ours(r["Name"]):
                rows.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), float(r["Percentage"])))
    print(f"rocprofv3 kernel-trace summary, one MI355X; kernels of libintscale.so only")
    print(f"command (from /tmp, TMPDIR=/tmp): rocprofv3 --kernel-trace --stats -d <out> -o kt --output-format csv -- {args.command}")
    print("columns: kernel, dispatches, average duration (us), share of GPU time (%)\n")
    for n, c, a, p in rows:
        print(f"{n}\t{c}\t{a / 1e3:.3f}\t{p:.2f}")


def calibration(table, counter, pick, known_bytes):
    cands = [(k, v[counter]) for k, v in table.items() if counter in v and pick(k)]
    if not cands:
        sys.exit(f"profile_summary: no calibration kernel for {counter} in this pass")
    # the kernel runs at other sizes too in the same command: its largest dispatch is the one of known size
    k, (avg, n, top) = max(cands, key=lambda kv: kv[1][2])
    return k, top, known_bytes / (top * 1024.0)


def cmd_traffic(args):
    fe, wr = read_counters(args.files[0]), read_counters(args.files[1])
    kf, vf, sf = calibration(fe, "FETCH_SIZE", lambda k: "stream_read_kernel" in k, GIB)
    kw, vw, sw = calibration(wr, "WRITE_SIZE", lambda k: "FillFunctor" in k, GIB)
    print("HBM traffic per dispatch, one MI355X, from two rocprofv3 counter passes")
    print(f"commands (from /tmp, TMPDIR=/tmp): rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <out> -o p --output-format csv -- {args.command}")
    print(f"                                   rocprofv3 --pmc WRITE_SIZE --kernel-trace -d <out> -o p --output-format csv -- {args.command}")
    print(f"scaling: the 1 GiB streaming-read probe of the same run reads FETCH_SIZE = {vf:.0f}, the 1 GiB fill before")
    print(f"         it WRITE_SIZE = {vw:.0f} (KiB expected: {GIB // 1024}), so bytes = counter * 1024 * {sf:.3f} (fetch) and * {sw:.3f} (write)")
    print("columns: TRAFFIC, kernel, HBM bytes per dispatch (fetch + write) | then fetch bytes, write bytes, dispatches\n")
    order = sorted((k for k in fe if ours(k) and "FETCH_SIZE" in fe[k]),
                   key=lambda k: -fe[k]["FETCH_SIZE"][0] * fe[k]["FETCH_SIZE"][1])
    for k in order:
        fb = fe[k]["FETCH_SIZE"][0] * 1024 * sf
        wb = wr.get(k, {}).get("WRITE_SIZE", (0.0, 0, 0.0))[0] * 1024 * sw
        print(f"TRAFFIC\t{short(k)}\t{fb + wb:.0f}")
        print(f"#\t{short(k)}\tfetch {fb:.0f}\twrite {wb:.0f}\tdispatches {fe[k]['FETCH_SIZE'][1]}")


def cmd_counters(args):
    merged = collections.defaultdict(dict)
    names = []
    for path in args.files:
        for k, cs in read_counters(path).items():
            if not ours(k):
                continue
            for c, (avg, n, _) in cs.items():
                merged[short(k)][c] = avg
                merged[short(k)]["dispatches"] = n
                if c not in names:
                    names.append(c)
    print("rocprofv3 counter summary, one MI355X; averages per dispatch, kernels of libintscale.so only")
    print(f"command (from /tmp, TMPDIR=/tmp), one run per group of counters: rocprofv3 --pmc <counters> --kernel-trace -d <out> -o p --output-format csv -- {args.command}")
    print("columns: kernel, dispatches, " + ", ".join(names) + "\n")
    for k, cs in merged.items():
        print("\t".join([k, str(cs.get("dispatches", 0))] + [f"{cs.get(c, float('nan')):.4g}" for c in names]))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("mode", choices=("trace", "traffic", "counters"))
    ap.add_argument("files", nargs="+")
    ap.add_argument("--command", default="python3 bench.py", help="the command that was profiled (goes into the header)")
    args = ap.parse_args()
    if args.mode == "traffic" and len(args.files) != 2:
        sys.exit("traffic: the FETCH_SIZE pass and the WRITE_SIZE pass")
    {"trace": cmd_trace, "traffic": cmd_traffic, "counters": cmd_counters}[args.mode](args)


if __name__ == "__main__":
    main()
