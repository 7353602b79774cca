"""Per-operator timeline of one replay of the persistent executor.

A profiler sees a single kernel, so the executor stamps every work item itself (100 MHz
device clock).  This tool replays one config with the timeline on and prints, per operator in
launch-queue order: tiles, when its first tile had its predecessors complete, when its last
tile was published, and the median tile time; then the overlap summary (operators in flight,
busy fraction of the workgroups).  It is the counterpart of a kernel-trace timeline for the
multi-stream graph (paper Sec. 5.3 looks at the same thing through SM utilisation).

  python -m paper_2312_10351_amd.timeline [--config 1] [--policy alg2] [--rows 200] [--zero-copy-concat]
  python -m paper_2312_10351_amd.timeline --executor par|seq|fused [--config 1] ...

With --executor par / seq / fused it prints the operator timeline of a graph executor instead:
every operator kernel stamps its own start and end (opara_set_operator_trace), so the
overlap of the multi-stream graph is measured without a profiler attached.
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


def operator_overlap(t):
    """Concurrency of operator kernels from an operator timeline ([ops, 2] start / end in ns,
    Session.operator_trace): span, share of the span with 0, 1, 2, ... operators in flight,
    mean and peak."""
    iv = t[(t[:, 0] >= 0) & (t[:, 1] > t[:, 0])]
    if len(iv) == 0:
        return dict(operators_stamped=0)
    ev = sorted([(int(a), 1) for a in iv[:, 0]] + [(int(b), -1) for b in iv[:, 1]])
    t0, t1 = ev[0][0], max(int(b) for b in iv[:, 1])
    cur, peak, prev, hist = 0, 0, t0, {}
    for when, d in ev:
        hist[cur] = hist.get(cur, 0) + (when - prev)
        prev, cur = when, cur + d
        peak = max(peak, cur)
    span = max(t1 - t0, 1)
    busy = int((iv[:, 1] - iv[:, 0]).sum())
    return dict(operators_stamped=int(len(iv)), span_us=span / 1e3, sum_of_operator_durations_us=busy / 1e3,
                operators_in_flight_peak=peak, operators_in_flight_mean=busy / span,
                time_share_by_operators_in_flight={str(k): round(v / span, 4) for k, v in sorted(hist.items())},
                share_with_two_or_more=round(sum(v for k, v in hist.items() if k >= 2) / span, 4))


def graph_timeline(config, mode, zero_copy, rows, policy):
    """Operator timeline of one replay of the sequential / multi-stream / fused executor."""
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    s = Session(build_config(config), zero_copy_concat=zero_copy)
    try:
        m = {"seq": B.SEQUENTIAL, "par": B.PARALLEL, "fused": B.FUSED}[mode]
        t = s.operator_trace(m, policy=policy, replays=5)
        exe = s.execs[-1]
        order = sorted(range(len(t)), key=lambda v: t[v, 0])
        so = B.opara_assign_streams(s.dag)[0]
        node_of = B.opara_fused_plan(exe, len(s.lib_ops))[0] if mode == "fused" else None
        print(f"| operator | name | {'node' if mode == 'fused' else 'stream'} | start us | end us | duration us |")
        print("|---|---|---|---|---|---|")
        for v in order[:rows]:
            op = s.wl.ops[s.lib_ops[v]]
            where = node_of[v] if node_of else so[v]
            print(f"| {v} | {op.name or op.type} | {where} | {t[v, 0] / 1e3:.2f} | {t[v, 1] / 1e3:.2f} | {(t[v, 1] - t[v, 0]) / 1e3:.2f} |")
        print()
        print(json.dumps(dict(workload=s.wl.name, executor=mode, zero_copy_concat=zero_copy, **operator_overlap(t))))
    finally:
        s.close()


def main():
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--policy", default="alg2", choices=list(B.ORDER_POLICY_NAMES))
    ap.add_argument("--rows", type=int, default=200)
    ap.add_argument("--zero-copy-concat", action="store_true")
    ap.add_argument("--executor", default="persist", choices=["persist", "seq", "par", "fused"],
                    help="persist: per-tile timeline of the persistent executor; seq / par / fused: operator timeline "
                         "(start and end of every operator's kernel, stamped inside the kernels) and its overlap summary")
    a = ap.parse_args()
    pol = list(B.ORDER_POLICY_NAMES).index(a.policy)
    if a.executor != "persist":
        graph_timeline(a.config, a.executor, a.zero_copy_concat, a.rows, pol)
        return
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
