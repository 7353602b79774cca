"""Turns rocprofv3 CSV output into the short summaries kept under profiles/.

  python -m paper_2312_10351_amd.profile_summary stats   <dir> [--top 12]
      per-kernel calls / average / min / max / share of GPU time from *_kernel_trace.csv
  python -m paper_2312_10351_amd.profile_summary overlap <dir> --kernels N [--replay -1] [--timeline 40]
      concurrent-kernel histogram (share of the replay's span with 0, 1, 2, ... kernels in
      flight) and a short timeline of one graph replay = N consecutive opara kernels of the
      trace (--replay picks which block of N, counted from the end when negative)
  python -m paper_2312_10351_amd.profile_summary counter <dir> [--name COUNTER]
      per-kernel average of a --pmc counter from *_counter_collection.csv
  python -m paper_2312_10351_amd.profile_summary traffic <fetch_dir> <write_dir> --workload NAME
          [--calibration-kernel opara_k_elt_f16_vec --calibration-kib 65536] [--append FILE]
      HBM bytes per launch of every opara kernel: FETCH_SIZE and WRITE_SIZE averages (KiB per
      dispatch), each scaled by what the same counter reads for the calibration kernel (a
      streaming kernel that reads and writes --calibration-kib KiB per launch); --append adds
      `workload kernel fetch_bytes write_bytes` lines to FILE (bench.py reads
      profiles/hbm_traffic_per_launch.txt for its roofline.traffic field)
Markdown on stdout.  rocprofv3 must have been run with --output-format csv.
"""
import argparse
import collections
import csv
import glob
import os
import sys


def _rows(directory, suffix):
    files = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not files:
        sys.exit(f"no *{suffix} under {directory}")
    for f in files:
        with open(f, newline="") as fh:
            for r in csv.DictReader(fh):
                yield r


def kernel_trace(directory):
    out = []
    for r in _rows(directory, "_kernel_trace.csv"):
        out.append(dict(name=r["Kernel_Name"], start=int(r["Start_Timestamp"]), end=int(r["End_Timestamp"]),
                        queue=r["Queue_Id"], grid=int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"]),
                        wg=int(r["Workgroup_Size_X"])))
    out.sort(key=lambda k: k["start"])
    return out


def short(name):
    return name if len(name) <= 48 else name[:45] + "..."


def cmd_stats(a):
    by = collections.defaultdict(list)
    for k in kernel_trace(a.dir):
        by[k["name"]].append(k["end"] - k["start"])
    total = sum(sum(v) for v in by.values())
    print("| kernel | calls | avg ns | min ns | max ns | % of GPU time |")
    print("|---|---|---|---|---|---|")
    for name, v in sorted(by.items(), key=lambda kv: -sum(kv[1]))[:a.top]:
        print(f"| {short(name)} | {len(v)} | {sum(v) / len(v):.0f} | {min(v)} | {max(v)} | {100 * sum(v) / total:.2f} |")


def cmd_overlap(a):
    ks = [k for k in kernel_trace(a.dir) if k["name"].startswith("opara_k_") and (not a.only or a.only in k["name"])]
    n = a.kernels
    if len(ks) < n:
        sys.exit(f"only {len(ks)} opara kernels in the trace")
    blocks = len(ks) // n
    b = a.replay if a.replay >= 0 else blocks + a.replay
    first = len(ks) - (blocks - b) * n
    rep = ks[first:first + n]
    t0, t1 = min(k["start"] for k in rep), max(k["end"] for k in rep)
    ev = sorted([(k["start"], 1) for k in rep] + [(k["end"], -1) for k in rep])
    hist, cur, prev, peak = collections.Counter(), 0, t0, 0
    for t, d in ev:
        hist[cur] += t - prev
        prev, cur = t, cur + d
        peak = max(peak, cur)
    span = t1 - t0
    busy = sum(k["end"] - k["start"] for k in rep)
    print(f"replay {b} of {blocks}: {n} kernels, span {span / 1e3:.1f} us, sum of kernel durations {busy / 1e3:.1f} us, "
          f"hardware queues used {len(set(k['queue'] for k in rep))}, peak concurrency {peak}")
    print()
    print("| kernels in flight | share of the span | us |")
    print("|---|---|---|")
    for c in sorted(hist):
        print(f"| {c} | {100 * hist[c] / span:.1f} % | {hist[c] / 1e3:.1f} |")
    print(f"\nmean kernels in flight over the span: {busy / span:.2f}")
    if a.timeline:
        print("\n| start us | duration us | queue | kernel | workgroups |")
        print("|---|---|---|---|---|")
        for k in rep[:a.timeline]:
            print(f"| {(k['start'] - t0) / 1e3:.2f} | {(k['end'] - k['start']) / 1e3:.2f} | {k['queue']} | "
                  f"{k['name'].replace('opara_k_', '')} | {k['grid'] // max(k['wg'], 1)} |")


def counters(directory, name=None):
    by = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in _rows(directory, "_counter_collection.csv"):
        if name is None or r["Counter_Name"] == name:
            by[r["Counter_Name"]][r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return by


def cmd_counter(a):
    for cname, kernels in counters(a.dir, a.name).items():
        print(f"counter {cname}\n")
        print("| kernel | dispatches | average | min | max |")
        print("|---|---|---|---|---|")
        for k, v in sorted(kernels.items(), key=lambda kv: -sum(kv[1])):
            if k.startswith("opara_k_") or a.all:
                print(f"| {short(k)} | {len(v)} | {sum(v) / len(v):.1f} | {min(v):.1f} | {max(v):.1f} |")
        print()


def cmd_traffic(a):
    fetch = counters(a.fetch_dir, "FETCH_SIZE")["FETCH_SIZE"]
    write = counters(a.write_dir, "WRITE_SIZE")["WRITE_SIZE"]
    cal = a.calibration_kernel
    if cal not in fetch or cal not in write:
        sys.exit(f"calibration kernel {cal} not in both runs (pass --calibration-copy to bench.py)")
    # the calibration launches are the largest dispatches of that kernel
    cf, cw = max(fetch[cal]), max(write[cal])
    sf, sw = a.calibration_kib / cf, a.calibration_kib / cw
    print(f"calibration ({cal}, {a.calibration_kib} KiB read + {a.calibration_kib} KiB written per launch): FETCH_SIZE reads "
          f"{cf:.0f}, WRITE_SIZE {cw:.0f} per dispatch; scale factors: fetch x {sf:.3f}, write x {sw:.3f}\n")
    print("| kernel | dispatches | FETCH_SIZE avg | WRITE_SIZE avg | scaled HBM traffic per launch |")
    print("|---|---|---|---|---|")
    lines = []
    for k in sorted(set(fetch) & set(write), key=lambda k: -sum(fetch[k])):
        if not k.startswith("opara_k_"):
            continue
        vf, vw = fetch[k], write[k]
        if k == cal:                          # leave the calibration launches out of that kernel's own average
            vf, vw = [x for x in vf if x < 0.9 * cf] or vf, [x for x in vw if x < 0.9 * cw] or vw
        f, w = sum(vf) / len(vf) * sf, sum(vw) / len(vw) * sw
        print(f"| {k} | {len(vf)} | {sum(vf) / len(vf):.1f} | {sum(vw) / len(vw):.1f} | {f:.0f} + {w:.0f} = {f + w:.0f} KiB "
              f"({(f + w) * 1024 / 1e6:.2f} MB) |")
        lines.append(f"{a.workload} {k.replace('opara_k_', '')}{a.suffix} {f * 1024:.0f} {w * 1024:.0f}\n")
    if a.append:
        with open(a.append, "a") as fh:
            fh.writelines(lines)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("stats"); p.add_argument("dir"); p.add_argument("--top", type=int, default=12); p.set_defaults(fn=cmd_stats)
    p = sub.add_parser("overlap"); p.add_argument("dir"); p.add_argument("--kernels", type=int, required=True)
    p.add_argument("--replay", type=int, default=-1); p.add_argument("--timeline", type=int, default=0)
    p.add_argument("--only", default=""); p.set_defaults(fn=cmd_overlap)
    p = sub.add_parser("counter"); p.add_argument("dir"); p.add_argument("--name", default=None)
    p.add_argument("--all", action="store_true"); p.set_defaults(fn=cmd_counter)
    p = sub.add_parser("traffic"); p.add_argument("fetch_dir"); p.add_argument("write_dir")
    p.add_argument("--workload", required=True); p.add_argument("--suffix", default="")
    p.add_argument("--calibration-kernel", default="opara_k_elt_f16_vec"); p.add_argument("--calibration-kib", type=float, default=65536.0)
    p.add_argument("--append", default=None); p.set_defaults(fn=cmd_traffic)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
