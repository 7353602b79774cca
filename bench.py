#!/usr/bin/env python3
"""Benchmark: batch-1 DAG latency of the operator-parallel graph replay on one MI355X.

A step is one replay of the whole captured DAG (launch order + single hipGraph) with inputs
and weights resident in HBM.  Three executors replay the same kernels on the same buffers:
the sequential single-stream graph (the baseline), the multi-stream graph (Alg. 1 streams,
Alg. 2 order, dependencies as graph edges) and the persistent executor (one kernel, Alg. 2
order, dependencies as completion flags).  The headline value is the faster of the two
operator-parallel executors, named in config.mode.  The headline workload is the
GoogLeNet-like fp16 DAG; the other configs are reported beside it.  One JSON line on
stdout.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled by
# a streaming kernel of known size (profiles/googlenet_like_graph_kernels_hbm_traffic.md,
# profiles/persist_f16_googlenet_like_hbm_traffic.md).
MEASURED_TRAFFIC_BYTES = {("googlenet_like", "igemm_f16_direct4"): (1054 + 345) * 1024,
                          ("googlenet_like", "igemm_f16_quad4"): (1220 + 136) * 1024,
                          ("googlenet_like", "persist_f16"): (51762 + 17008) * 1024,
                          ("googlenet_like", "persist_f16+zero_copy_concat"): (49159 + 12139) * 1024}


def percentile(a, q):
    return float(np.percentile(np.asarray(a), q))


def time_replays(session, exe, steps, warmup):
    """Per-replay latency (events on the launch stream, host sync after each) and
    back-to-back time per replay (no host sync between replays)."""
    import torch
    from paper_2312_10351_amd import binding as B
    st = session.make_streams(1)
    h, ts = st.handles[0], st.torch_streams[0]
    for _ in range(warmup):
        B.opara_replay(exe, h)
    ts.synchronize()
    lat = []
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    for _ in range(steps):
        e0.record(ts)
        B.opara_replay(exe, h)
        e1.record(ts)
        ts.synchronize()
        lat.append(e0.elapsed_time(e1) * 1e3)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(ts)
    for _ in range(steps):
        B.opara_replay(exe, h)
    e1.record(ts)
    ts.synchronize()
    wall = time.perf_counter() - t0
    return dict(median_us=percentile(lat, 50), mean_us=float(np.mean(lat)), p99_us=percentile(lat, 99),
                min_us=float(np.min(lat)), back_to_back_us=e0.elapsed_time(e1) * 1e3 / steps,
                wall_us_per_replay=wall * 1e6 / steps)


def isolated_op_times(session, reps=20):
    """Average duration of each operator's kernel launched alone `reps` times in a row
    on one stream, bracketed by events on that stream (microseconds)."""
    import torch
    from paper_2312_10351_amd import binding as B
    st = session.make_streams(1)
    h, ts = st.handles[0], st.torch_streams[0]
    out = []
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    for lib_id in range(len(session.lib_ops)):
        for _ in range(3):
            B.opara_launch_op(session.dag, lib_id, h)
        e0.record(ts)
        for _ in range(reps):
            B.opara_launch_op(session.dag, lib_id, h)
        e1.record(ts)
        ts.synchronize()
        out.append(e0.elapsed_time(e1) * 1e3 / reps)
    return out


def timeline_summary(session, exe):
    """Overlap evidence from the persistent executor's own timeline (a profiler sees one
    kernel): busy fraction of the workgroups and how many operators are in flight."""
    from paper_2312_10351_amd import binding as B
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


def bench_config(index, steps, warmup, with_kernels, zero_copy_concat=False):
    from paper_2312_10351_amd import binding as B
    from paper_2312_10351_amd.runtime import Session
    from paper_2312_10351_amd.roofline import dag_roofline, MFMA_FLOPS, HBM_BYTES_PER_S
    from workloads import build_config
    wl = build_config(index)
    s = Session(wl, zero_copy_concat=bool(zero_copy_concat))
    if zero_copy_concat == "auto":            # wherever the library finds a concatenation to remove
        zero_copy_concat = len(s.elided) > 0
    try:
        t0 = time.perf_counter()
        so, ns = B.opara_assign_streams(s.dag)
        t1 = time.perf_counter()
        order = B.opara_order_launch(s.dag)
        t2 = time.perf_counter()
        syncs = B.opara_sync_edges(s.dag)
        t3 = time.perf_counter()
        par = s.capture(B.PARALLEL)
        t4 = time.perf_counter()
        seq = s.capture(B.SEQUENTIAL)
        t5 = time.perf_counter()
        # work-item order of the persistent executor: Alg. 2 queue or wave by wave, whichever a short
        # probe finds faster (static dealing of tiles favours level order on very wide DAGs)
        probe = {}
        for pol in (B.ORDER_ALG2, B.ORDER_LEVEL):
            exe = s.capture_persistent(policy=pol)
            probe[pol] = time_replays(s, exe, 40, 10)["median_us"]
        per_policy = min(probe, key=probe.get)
        t5 = time.perf_counter()
        per = s.capture_persistent(policy=per_policy)
        t6 = time.perf_counter()
        r_par = time_replays(s, par, steps, warmup)
        r_seq = time_replays(s, seq, steps, warmup)
        r_per = time_replays(s, per, steps, warmup)
        if s.persistent_status(per) != 0:
            raise RuntimeError("persistent executor: a wait ran out")
        best = "persistent" if r_per["median_us"] <= r_par["median_us"] else "multi_stream_graph"
        r_best = r_per if best == "persistent" else r_par
        roof = dag_roofline(wl)
        res = dict(workload=wl.name, dtype=wl.dtype, n_ops=len(wl.ops), zero_copy_concat=zero_copy_concat,
                   n_ops_launched=len(s.lib_ops), n_streams=ns, n_sync_edges=len(syncs),
                   graph_nodes_edges=B.opara_exec_info(par),
                   assign_streams_ms=(t1 - t0) * 1e3, order_launch_ms=(t2 - t1) * 1e3, capture_ms=(t4 - t3) * 1e3,
                   persistent_capture_ms=(t6 - t5) * 1e3, persistent_queue=B.ORDER_POLICY_NAMES[per_policy],
                   persistent_queue_probe_us={B.ORDER_POLICY_NAMES[k]: v for k, v in probe.items()},
                   parallel=r_par, sequential=r_seq, persistent=r_per,
                   persistent_timeline=timeline_summary(s, per), best_mode=best, best=r_best,
                   # what runtime.Session.capture_best() would hand out: the sequential graph is a candidate too
                   fastest_executor=min((("sequential_graph", r_seq), ("multi_stream_graph", r_par), ("persistent", r_per)),
                                        key=lambda kv: kv[1]["median_us"])[0],
                   speedup_vs_sequential=r_seq["median_us"] / r_best["median_us"],
                   speedup_multi_stream_graph=r_seq["median_us"] / r_par["median_us"],
                   speedup_persistent=r_seq["median_us"] / r_per["median_us"],
                   dag_flops=roof["flops"], dag_bytes=roof["bytes"],
                   roofline_us=dict(flops=roof["t_flops_us"], bytes=roof["t_bytes_us"], critical_path=roof["t_cp_us"],
                                    bound=roof["t_roof_us"]),
                   roofline_fraction=roof["t_roof_us"] / r_best["median_us"])
        kern = None
        if with_kernels:
            t_iso = isolated_op_times(s)
            dem = B.opara_get_demands(s.dag)
            by = {}
            for op, d, t in zip([wl.ops[v] for v in s.lib_ops], dem, t_iso):
                name = B.opara_kernel_info(d.kernel_id)[0]
                f, b = roof["per_op"][op.id]
                e = by.setdefault(name, dict(launches=0, time_us=0.0, flops=0, bytes=0))
                e["launches"] += 1; e["time_us"] += t; e["flops"] += f; e["bytes"] += b
            dom = max(by, key=lambda k: by[k]["time_us"])
            e = by[dom]
            if dom.startswith("igemm") or dom.startswith("gemv"):
                peak = MFMA_FLOPS[wl.dtype] / 1e12
                ach = e["flops"] / (e["time_us"] * 1e-6) / 1e12
                kern = dict(kernel=dom, bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                            traffic=MEASURED_TRAFFIC_BYTES.get((wl.name, dom)))
            else:
                peak = HBM_BYTES_PER_S / 1e9
                ach = e["bytes"] / (e["time_us"] * 1e-6) / 1e9
                kern = dict(kernel=dom, bound="hbm", achieved=ach, peak=peak, unit="GB/s", frac=ach / peak,
                            traffic=None)
            kern.update(launches_per_step=e["launches"], avg_launch_us=e["time_us"] / e["launches"],
                        flops_per_launch=e["flops"] / e["launches"], bytes_per_launch=e["bytes"] / e["launches"])
            res["dominant_graph_kernel"] = kern
            if best == "persistent":
                # One kernel runs the DAG behind its serial prefix: its launch duration is measured on
                # ordinary launches of that kernel between HIP events on the launch stream, its work is
                # the operators inside it.
                name = "persist_" + wl.dtype
                st = s.make_streams(1)
                t_us = B.opara_persistent_time_kernel(per, st.handles[0], steps)
                if s.persistent_status(per) != 0:
                    raise RuntimeError("persistent executor: a wait ran out")
                queue = B.opara_order_launch_policy(s.dag, per_policy)
                ahead = {s.lib_ops[v] for v in queue[:B.opara_persistent_prefix(per)]}
                k_flops = sum(f for op, (f, _) in zip(wl.ops, roof["per_op"]) if op.id not in ahead)
                k_bytes = sum(b for op, (_, b) in zip(wl.ops, roof["per_op"]) if op.id not in ahead)
                bound_mfma = k_flops / MFMA_FLOPS[wl.dtype] >= k_bytes / HBM_BYTES_PER_S
                if bound_mfma:
                    peak = MFMA_FLOPS[wl.dtype] / 1e12
                    ach = k_flops / (t_us * 1e-6) / 1e12
                    kern = dict(kernel=name, bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak)
                else:
                    peak = HBM_BYTES_PER_S / 1e9
                    ach = k_bytes / (t_us * 1e-6) / 1e9
                    kern = dict(kernel=name, bound="hbm", achieved=ach, peak=peak, unit="GB/s", frac=ach / peak)
                kern.update(traffic=MEASURED_TRAFFIC_BYTES.get((wl.name, name + ("+zero_copy_concat" if zero_copy_concat else ""))),
                            launches_per_step=1, avg_launch_us=t_us, operators_in_kernel=len(wl.ops) - len(ahead),
                            operators_ahead_as_kernel_nodes=len(ahead),
                            flops_per_launch=k_flops, bytes_per_launch=k_bytes)
            res["sum_isolated_us"] = float(sum(t_iso))
            finish = [0.0] * len(wl.ops)
            for op in wl.ops:                 # an elided concatenation takes no time of its own
                t_op = t_iso[s.lib_id[op.id]] if op.id in s.lib_id else 0.0
                finish[op.id] = max([finish[u] for u in op.inputs if u >= 0], default=0.0) + t_op
            res["critical_path_isolated_us"] = float(max(finish))
            res["kernels"] = {k: dict(launches=v["launches"], avg_us=v["time_us"] / v["launches"]) for k, v in by.items()}
        return res, kern
    finally:
        s.close()


def calibration_copy(reps=10, mib=64):
    """Plain streaming kernel of known size (ReLU over `mib` MiB of fp16: that many bytes
    read and as many written per launch), used to scale the HBM traffic counters."""
    from paper_2312_10351_amd import binding as B
    from paper_2312_10351_amd.runtime import Session
    from workloads import Builder
    rows = mib * 1024 * 1024 // 2 // 4096
    b = Builder("calibration_copy", "f16")
    b.rowwise("relu", [b.ext((rows, 4096))], rows, 4096)
    s = Session(b.build(1))
    try:
        st = s.make_streams(1)
        for _ in range(reps):
            B.opara_launch_op(s.dag, 0, st.handles[0])
        st.torch_streams[0].synchronize()
    finally:
        s.close()


def cpu_baseline(budget_s=12.0):
    """The oracle executor, as it stands, on the host cores: full passes over the
    headline DAG until about `budget_s` seconds are spent."""
    from oracle import executor
    from workloads import build_config
    wl = build_config(1)
    sink = wl.sinks()
    executor.run_dag(wl, keep=sink)
    times = []
    t_end = time.perf_counter() + budget_s
    while time.perf_counter() < t_end or len(times) < 3:
        t0 = time.perf_counter()
        executor.run_dag(wl, keep=sink)
        times.append(time.perf_counter() - t0)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=percentile(times, 50) * 1e6, unit="us", cores=int(threads), kind="oracle",
                sample=f"{len(times)} full passes of the googlenet_like DAG (numpy fp64, all 81 operators), median")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--configs", type=str, default="0,2,3,4,5",
                    help="extra configs reported beside the headline one (5 = NASNet-cell-like DAG, not in BASELINE.json)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch a 64 MiB streaming kernel 10 times (scale for rocprofv3 --pmc traffic counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this path runs on ONE GPU (a batch-1 DAG is not sharded); use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if a.calibration_copy:
        calibration_copy()
    head_x, kern_x = bench_config(1, a.steps, a.warmup, with_kernels=True)
    head_z, kern_z = bench_config(1, a.steps, a.warmup, with_kernels=True, zero_copy_concat=True)
    head, kern, alt = (head_z, kern_z, head_x) if head_z["best"]["median_us"] <= head_x["best"]["median_us"] else (head_x, kern_x, head_z)
    others = []
    for idx in [int(x) for x in a.configs.split(",") if x != ""]:
        r, _ = bench_config(idx, max(100, a.steps // 4), a.warmup, with_kernels=False, zero_copy_concat="auto")
        others.append(r)
    line = {
        "metric": "batch1_dag_latency_us", "value": head["best"]["median_us"], "unit": "us",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["best"]["mean_us"] / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "googlenet_like fp16 batch 1, 1x3x224x224, 81 operators (configs[1])",
                   "concatenation": ("zero-copy: the branches write their channel slices of the concatenated tensor, "
                                     "%d of 81 operators are launched; the sequential baseline uses the same layout"
                                     % head["n_ops_launched"]) if head["zero_copy_concat"] else "explicit concatenation kernels",
                   "mode": {"persistent": "persistent executor: one hipGraph replay = the serial stem as %d kernel nodes, then one "
                                          "kernel for the rest (work items in %s order, dependencies as completion flags)"
                                          % (head["persistent_timeline"]["serial_prefix_operators"], head["persistent_queue"]),
                            "multi_stream_graph": "multi-stream hipGraph replay (Alg. 1 streams, Alg. 2 launch order)"
                            }[head["best_mode"]]},
        "throughput_inferences_per_s": 1e6 / head["best"]["back_to_back_us"],
        "speedup_vs_sequential_hipgraph": head["speedup_vs_sequential"],
        "dag_roofline_fraction": head["roofline_fraction"],
        "roofline": kern,
        "headline": head,
        "headline_other_concatenation": alt,
        "other_configs": others,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
