"""Turns rocprofv3 CSV output into the short text tables kept under profiles/ and into
profiles/hbm_traffic.json (the HBM bytes per launch that bench.py prints as `traffic`).

    python -m paper_2503_08640_amd.profsum stats    <..._kernel_stats.csv>
    python -m paper_2503_08640_amd.profsum trace    <..._kernel_trace.csv> [--match SUBSTR ...]
    python -m paper_2503_08640_amd.profsum counters <..._counter_collection.csv> [--match SUBSTR ...]
    python -m paper_2503_08640_amd.profsum traffic  --fetch <csv> --write <csv> --out profiles/hbm_traffic.json
                                                    [--commit HASH]

Runs on the CPU on files a profiling run left behind; nothing here touches the GPU.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
import re
import sys
from collections import defaultdict

ROOT = os.path.dirname(os.path.abspath(__file__))
CALIB_COPY_KIB = 256 * 1024     # bench.py --calib-copy: one 256 MiB device-to-device copy


def kernel_sources_digest() -> str:
    """sha256 over the kernel and host sources of the library (names and contents, in name order)."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".hpp", ".cpp", ".h")):
            h.update(name.encode())
            with open(os.path.join(src, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def short_name(name: str, width: int = 64) -> str:
    name = name.replace("void ", "").replace("(anonymous namespace)::", "")
    name = re.sub(r"\(.*\)$", "", name)            # argument list
    name = re.sub(r"\s+", "", name)
    return name if len(name) <= width else name[: width - 3] + "..."


def cmd_stats(args) -> int:
    rows = list(csv.DictReader(open(args.file, newline="")))
    print(f"{'kernel':<66}{'calls':>7}{'total ms':>11}{'average us':>12}{'%':>7}{'min us':>10}{'max us':>10}")
    for r in rows:
        if float(r["Percentage"]) < args.min_percent:
            continue
        print(f"{short_name(r['Name']):<66}{int(r['Calls']):>7}{float(r['TotalDurationNs']) / 1e6:>11.3f}"
              f"{float(r['AverageNs']) / 1e3:>12.2f}{float(r['Percentage']):>7.2f}{float(r['MinNs']) / 1e3:>10.2f}"
              f"{float(r['MaxNs']) / 1e3:>10.2f}")
    return 0


def clusters(durations, ratio: float = 1.5):
    """Splits {dispatch: duration} into groups of similar duration (sorted; a new group starts where the next
    duration is more than `ratio` times the one before): one kernel name often serves launches of several sizes."""
    order = sorted(durations, key=durations.get)
    groups, cur = [], []
    for d in order:
        if cur and durations[d] > ratio * durations[cur[-1]]:
            groups.append(cur)
            cur = []
        cur.append(d)
    if cur:
        groups.append(cur)
    return groups


def cmd_trace(args) -> int:
    dur, grid = defaultdict(dict), defaultdict(dict)
    for r in csv.DictReader(open(args.file, newline="")):
        k = short_name(r["Kernel_Name"], 200)
        if args.match and not any(m in k for m in args.match):
            continue
        d = int(r["Dispatch_Id"])
        dur[k][d] = float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
        grid[k][d] = (int(r["Grid_Size_X"]) // max(1, int(r["Workgroup_Size_X"])), int(r["Grid_Size_Y"]), int(r["Grid_Size_Z"]),
                      int(r["Workgroup_Size_X"]))
    print(f"{'kernel (launches of similar duration grouped)':<58}{'calls':>6}{'average us':>12}{'min us':>10}{'max us':>10}  workgroups x threads")
    for k in sorted(dur, key=lambda k: -sum(dur[k].values())):
        for g in clusters(dur[k]):
            v = [dur[k][d] / 1e3 for d in g]
            grids = sorted({grid[k][d] for d in g})
            gs = ", ".join(f"{a}x{b}x{c} x {t}" if (b, c) != (1, 1) else f"{a} x {t}" for a, b, c, t in grids[:3]) + (" ..." if len(grids) > 3 else "")
            print(f"{short_name(k, 56):<58}{len(v):>6}{sum(v) / len(v):>12.2f}{min(v):>10.2f}{max(v):>10.2f}  {gs}")
    return 0


def read_counters(path):
    """-> {kernel: {counter: [value per dispatch]}}, {kernel: [duration ns per dispatch]}, {kernel: grid sizes}"""
    vals = defaultdict(lambda: defaultdict(dict))
    dur = defaultdict(dict)
    grid = defaultdict(dict)
    for r in csv.DictReader(open(path, newline="")):
        k, disp = short_name(r["Kernel_Name"], 200), int(r["Dispatch_Id"])
        c = r["Counter_Name"]
        vals[k][c][disp] = vals[k][c].get(disp, 0.0) + float(r["Counter_Value"])
        dur[k][disp] = float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
        grid[k][disp] = int(r["Grid_Size"])
    return vals, dur, grid


def cmd_counters(args) -> int:
    vals, dur, grid = read_counters(args.file)
    for k in sorted(vals):
        if args.match and not any(m in k for m in args.match):
            continue
        for g in clusters(dur[k]):
            n = len(g)
            mean_us = sum(dur[k][d] for d in g) / n / 1e3
            print(f"{short_name(k, 100)}   dispatches {n}   mean duration under the counters {mean_us:.1f} us   "
                  f"grid {sorted({grid[k][d] for d in g})}")
            for c in sorted(vals[k]):
                v = [vals[k][c][d] for d in g if d in vals[k][c]]
                print(f"    {c:<34} mean per dispatch {sum(v) / max(1, len(v)):>18.1f}")
    return 0


def mean_per_dispatch(path, counter):
    vals, _, grid = read_counters(path)
    out = {}
    for k in vals:
        if counter in vals[k]:
            v = vals[k][counter]
            out[k] = (sum(v.values()) / len(v), len(v), v, grid[k])
    return out


def calibration(per_kernel, what):
    """The 256 MiB copy of bench.py --calib-copy: the copy dispatch with the largest grid."""
    best = None
    for k, (_, _, v, grid) in per_kernel.items():
        if "copyBuffer" not in k and "copy" not in k.lower():
            continue
        for disp, g in grid.items():
            if best is None or g > best[0]:
                best = (g, v[disp], k)
    if best is None or best[1] <= 0:
        raise SystemExit(f"no calibration copy found in the {what} run (bench.py --calib-copy)")
    return CALIB_COPY_KIB / best[1], best


def cmd_traffic(args) -> int:
    fetch = mean_per_dispatch(args.fetch, "FETCH_SIZE")
    write = mean_per_dispatch(args.write, "WRITE_SIZE")
    f_fac, f_cal = calibration(fetch, "FETCH_SIZE")
    w_fac, w_cal = calibration(write, "WRITE_SIZE")
    print(f"calibration copy: FETCH_SIZE raw {f_cal[1]:.1f} -> factor {f_fac:.3f}; WRITE_SIZE raw {w_cal[1]:.1f} -> factor {w_fac:.3f}")

    # attn_prefill64_kernel<waves, slack, SELF, PERSIST, GATHER>: SELF = false is the pre-encode launch
    groups = {
        "preencode": [("attn_prefill64_kernel<", "SELF=false")],
        "query_prefill": [("attn_prefill64_kernel<", "SELF=true"), ("prefill_merge_kernel",)],
        "decode_step": [("decode_group_kernel",), ("decode_group_merge_kernel",)],
    }
    rec = {"_doc": "HBM bytes per launch from two rocprofv3 --pmc runs of bench.py --calib-copy (FETCH_SIZE, then "
                   "WRITE_SIZE, KiB per dispatch), each scaled by what the same counter reads for the 256 MiB copy; "
                   "written by python -m paper_2503_08640_amd.profsum traffic",
           "git_commit": args.commit, "sources_sha256": kernel_sources_digest(),
           "fetch_factor": f_fac, "write_factor": w_fac}
    print(f"{'launch':<16}{'FETCH raw KiB':>16}{'WRITE raw KiB':>16}{'total MB':>12}")
    for name, parts in groups.items():
        # a kernel whose name contains another's (decode_group_merge_kernel / decode_group_kernel) is matched exactly
        def mean_of(table, needles):
            def has(k, n):
                if n.startswith("SELF="):
                    m = re.search(r"attn_prefill64_kernel<\d+,\d+,(true|false)", k)
                    return bool(m) and m.group(1) == n[5:]
                return n in k
            hits = [k for k in table if all(has(k, n) for n in needles)]
            if needles == ("decode_group_kernel",):
                hits = [k for k in hits if "merge" not in k]
            tot = sum(table[k][0] * table[k][1] for k in hits)
            cnt = sum(table[k][1] for k in hits)
            return tot / cnt if cnt else 0.0
        f_raw = sum(mean_of(fetch, nd) for nd in parts)
        w_raw = sum(mean_of(write, nd) for nd in parts)
        total = (f_raw * f_fac + w_raw * w_fac) * 1024.0
        rec[name] = {"fetch_kib_raw": round(f_raw, 1), "write_kib_raw": round(w_raw, 1), "bytes_per_launch": int(total)}
        print(f"{name:<16}{f_raw:>16.1f}{w_raw:>16.1f}{total / 1e6:>12.1f}")
    with open(args.out, "w") as f:
        json.dump(rec, f, indent=1)
        f.write("\n")
    print(f"wrote {args.out} (sources {rec['sources_sha256'][:12]}, commit {args.commit})")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("stats")
    a.add_argument("file")
    a.add_argument("--min-percent", type=float, default=0.05)
    a.set_defaults(fn=cmd_stats)
    a = sub.add_parser("trace")
    a.add_argument("file")
    a.add_argument("--match", nargs="*", default=[])
    a.set_defaults(fn=cmd_trace)
    a = sub.add_parser("counters")
    a.add_argument("file")
    a.add_argument("--match", nargs="*", default=[])
    a.set_defaults(fn=cmd_counters)
    a = sub.add_parser("traffic")
    a.add_argument("--fetch", required=True)
    a.add_argument("--write", required=True)
    a.add_argument("--out", required=True)
    a.add_argument("--commit", default=None)
    a.set_defaults(fn=cmd_traffic)
    args = ap.parse_args()
    return args.fn(args)


if __name__ == "__main__":
    sys.exit(main())
