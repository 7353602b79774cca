"""Per-operator timeline of one replay of the persistent executor.

A profiler sees a single kernel, so the executor stamps every work item itself (100 MHz
device clock).  This tool replays one config with the timeline on and prints, per operator in
launch-queue order: tiles, when its first tile had its predecessors complete, when its last
tile was published, and the median tile time; then the overlap summary (operators in flight,
busy fraction of the workgroups).  It is the counterpart of a kernel-trace timeline for the
multi-stream graph (paper Sec. 5.3 looks at the same thing through SM utilisation).

  python -m paper_2312_10351_amd.timeline [--config 1] [--policy alg2] [--rows 200] [--zero-copy-concat]
"""
import argparse
import json

import numpy as np


def operator_timeline(session, exe, order):
    from . import binding as B
    tr = session.persistent_trace(exe)
    tiles, kernels = B.opara_persistent_plan(session.dag)
    rows = []
    prefix = B.opara_persistent_prefix(exe)
    for pos, v in enumerate(order):
        m = tr[:, 3] == pos
        op = session.wl.ops[session.lib_ops[v]]
        if pos < prefix:                   # an ordinary kernel node ahead of the persistent kernel: no stamps
            rows.append(dict(pos=pos, op=v, name=op.name or op.type, kernel="(kernel node)", tiles=0, items=0,
                             first_ready_us=float("nan"), last_published_us=float("nan"),
                             median_tile_us=float("nan"), median_wait_us=float("nan")))
            continue
        rows.append(dict(pos=pos, op=v, name=op.name or op.type, kernel=B.opara_kernel_info(kernels[v])[0],
                         tiles=int(tiles[v]), items=int(m.sum()), first_ready_us=float(tr[m, 1].min()) / 1e3,
                         last_published_us=float(tr[m, 2].max()) / 1e3,
                         median_tile_us=float(np.median(tr[m, 2] - tr[m, 1])) / 1e3,
                         median_wait_us=float(np.median(tr[m, 1] - tr[m, 0])) / 1e3))
    return rows


def timeline_summary(session, exe):
    """Overlap evidence from the persistent executor's own timeline (a profiler sees one
    kernel): busy fraction of the workgroups and how many operators are in flight."""
    from . import binding as B
    tr = session.persistent_trace(exe)
    _, wgs = B.opara_persistent_info(exe)
    span = float(tr[:, 2].max() - tr[:, 0].min())
    run = (tr[:, 2] - tr[:, 1]).astype(np.float64)
    n_pos = int(tr[:, 3].max()) + 1
    prefix = B.opara_persistent_prefix(exe)    # operators ahead of the kernel (ordinary kernel nodes) carry no stamps
    ev = []
    for p in range(prefix, n_pos):
        m = tr[:, 3] == p
        ev.append((float(tr[m, 1].min()), 1))
        ev.append((float(tr[m, 2].max()), -1))
    ev.sort()
    cur, peak, area, last = 0, 0, 0.0, ev[0][0]
    hist = {}
    for t, d in ev:
        area += cur * (t - last)
        hist[cur] = hist.get(cur, 0.0) + (t - last)
        last = t
        cur += d
        peak = max(peak, cur)
    total = sum(hist.values()) or 1.0
    return dict(span_us=span / 1e3, serial_prefix_operators=prefix, workgroups=wgs, work_items=int(len(tr)),
                workgroup_busy_fraction=float(run.sum() / (span * wgs)),
                operators_in_flight_peak=peak, operators_in_flight_mean=area / total,
                time_share_by_operators_in_flight={str(k): round(v / total, 4) for k, v in sorted(hist.items())},
                median_tile_us=float(np.median(run)) / 1e3,
                median_wait_for_predecessors_us=float(np.median(tr[:, 1] - tr[:, 0])) / 1e3)


def main():
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--policy", default="alg2", choices=list(B.ORDER_POLICY_NAMES))
    ap.add_argument("--rows", type=int, default=200)
    ap.add_argument("--zero-copy-concat", action="store_true")
    a = ap.parse_args()
    pol = list(B.ORDER_POLICY_NAMES).index(a.policy)
    s = Session(build_config(a.config), zero_copy_concat=a.zero_copy_concat)
    try:
        exe = s.capture_persistent(policy=pol)
        for _ in range(5):
            s.replay(exe)
        order = B.opara_order_launch_policy(s.dag, pol)
        rows = operator_timeline(s, exe, order)
        print("| pos | op | name | kernel | tiles | first ready us | last published us | median tile us | median wait us |")
        print("|---|---|---|---|---|---|---|---|---|")
        for r in rows[:a.rows]:
            if r["items"] == 0:
                print(f"| {r['pos']} | {r['op']} | {r['name']} | {r['kernel']} | - | - | - | - | - |")
                continue
            print(f"| {r['pos']} | {r['op']} | {r['name']} | {r['kernel']} | {r['tiles']} | {r['first_ready_us']:.1f} | "
                  f"{r['last_published_us']:.1f} | {r['median_tile_us']:.2f} | {r['median_wait_us']:.2f} |")
        print()
        print(json.dumps(timeline_summary(s, exe)))
        if s.persistent_status(exe) != 0:
            raise SystemExit("a wait inside the kernel ran out")
    finally:
        s.close()


if __name__ == "__main__":
    main()
