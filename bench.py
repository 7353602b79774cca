#!/usr/bin/env python3
"""Benchmark: batch-1 DAG latency of operator-parallel graph replay on one MI355X.

A step is one replay of the whole captured DAG (launch order + single hipGraph) with inputs
and weights resident in HBM.  Five executors replay the same kernel bodies on the same
buffers, each as ONE hipGraph:
  sequential graph     one stream, default topological order (the baseline, paper Sec. 5.1)
  multi-stream graph   Alg. 1 streams, Alg. 2 order, dependencies as graph edges (the paper's design)
  persistent executor  one kernel, Alg. 2 order, dependencies as completion flags
  chained executor     the same without a work-item loop: one tile per workgroup, blocks in queue order
  fused executor       the launch queue cut into waves, a wave of several operators is one kernel
The headline value is the fastest operator-parallel executor (named in config.mode) on the
GoogLeNet-like fp16 DAG; the other configs are reported beside it, each with its own
roofline and CPU-oracle block.  One JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def load_traffic():
    """HBM bytes per launch from the recorded rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE,
    scaled by a streaming kernel of known size): lines `workload kernel fetch_bytes write_bytes`
    in profiles/hbm_traffic_per_launch.txt, written by paper_2312_10351_amd.profile_summary."""
    out = {}
    if os.path.exists(TRAFFIC_FILE):
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 4 and not line.startswith("#"):
                out[(f[0], f[1])] = int(float(f[2]) + float(f[3]))
    return out


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


def kernel_block(name, flops, nbytes, launches, time_us, dtype, traffic, **extra):
    """The `roofline` object of one kernel: achieved = algorithmic work of all its launches /
    their total measured duration, against the published peak of the bound that applies."""
    from paper_2312_10351_amd.roofline import MFMA_FLOPS, HBM_BYTES_PER_S
    if flops / MFMA_FLOPS[dtype] >= nbytes / HBM_BYTES_PER_S:
        peak, ach, bound, unit = MFMA_FLOPS[dtype] / 1e12, flops / (time_us * 1e-6) / 1e12, "mfma", "TFLOP/s"
    else:
        peak, ach, bound, unit = HBM_BYTES_PER_S / 1e9, nbytes / (time_us * 1e-6) / 1e9, "hbm", "GB/s"
    k = dict(kernel=name, bound=bound, achieved=ach, peak=peak, unit=unit, frac=ach / peak, traffic=traffic,
             launches_per_step=launches, avg_launch_us=time_us / launches, flops_per_launch=flops / launches,
             bytes_per_launch=nbytes / launches)
    k.update(extra)
    return k


def oracle_pass(wl, budget_s, one_thread=False):
    """The oracle executor, as it stands, on the host cores: full passes over the DAG until
    about `budget_s` seconds are spent (at least one).  Returns (block, sink outputs)."""
    from oracle import executor
    sinks = wl.sinks()
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
    except Exception:
        threadpool_info = threadpool_limits = None
    times, out = [], None
    t_end = time.perf_counter() + budget_s
    while not times or time.perf_counter() < t_end:
        t0 = time.perf_counter()
        out = executor.run_dag(wl, keep=sinks)
        times.append(time.perf_counter() - t0)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1]) if threadpool_info else os.cpu_count()
    block = dict(value=percentile(times, 50) * 1e6, unit="us", cores=int(threads), kind="oracle",
                 sample=f"{len(times)} full pass(es) of the {wl.name} DAG (numpy fp64, all {len(wl.ops)} operators), median")
    if one_thread and threadpool_limits:
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            executor.run_dag(wl, keep=sinks)
            block["one_thread_us"] = (time.perf_counter() - t0) * 1e6
    return block, out


def bench_config(index, steps, warmup, zero_copy_concat="auto", cpu_budget_s=0.0, traffic=None):
    from paper_2312_10351_amd import binding as B
    from paper_2312_10351_amd.runtime import Session
    from paper_2312_10351_amd.roofline import dag_roofline
    from paper_2312_10351_amd.timeline import timeline_summary
    from workloads import build_config
    traffic = traffic or {}
    import torch
    wl = build_config(index)
    mem0 = torch.cuda.memory_allocated()
    s = Session(wl, zero_copy_concat=bool(zero_copy_concat))
    mem_session = torch.cuda.memory_allocated() - mem0          # inputs, weights, every operator's output buffer
    if zero_copy_concat == "auto":            # wherever the library finds a concatenation to remove
        zero_copy_concat = len(s.elided) > 0
    tag = "+zero_copy_concat" if zero_copy_concat else ""
    try:
        t0 = time.perf_counter()
        so, ns = B.opara_assign_streams(s.dag)
        t1 = time.perf_counter()
        B.opara_order_launch(s.dag)
        t2 = time.perf_counter()
        syncs = B.opara_sync_edges(s.dag)
        t3 = time.perf_counter()
        par = s.capture(B.PARALLEL)
        t4 = time.perf_counter()
        seq = s.capture(B.SEQUENTIAL)
        fus = s.capture(B.FUSED)
        t5 = time.perf_counter()
        # work-item order of the persistent executor: Alg. 2 queue or wave by wave, whichever a short
        # probe finds faster (static dealing of tiles favours level order on very wide DAGs)
        probe = {}
        for pol in (B.ORDER_ALG2, B.ORDER_LEVEL):
            probe[pol] = time_replays(s, s.capture_persistent(policy=pol), 40, 10)["median_us"]
        per_policy = min(probe, key=probe.get)
        per = s.capture_persistent(policy=per_policy)
        chn = s.capture_chained()
        runs = {"sequential": time_replays(s, seq, steps, warmup), "multi_stream_graph": time_replays(s, par, steps, warmup),
                "persistent": time_replays(s, per, steps, warmup), "chained": time_replays(s, chn, steps, warmup),
                "fused": time_replays(s, fus, steps, warmup)}
        if s.persistent_status(per) != 0 or s.persistent_status(chn) != 0:
            raise RuntimeError("persistent / chained executor: a wait ran out")
        r_seq = runs["sequential"]
        best = min(("multi_stream_graph", "persistent", "chained", "fused"), key=lambda k: runs[k]["median_us"])
        r_best = runs[best]
        roof = dag_roofline(wl)
        node_of, n_nodes = B.opara_fused_plan(fus, len(s.lib_ops))
        res = dict(workload=wl.name, dtype=wl.dtype, n_ops=len(wl.ops), zero_copy_concat=bool(zero_copy_concat),
                   n_ops_launched=len(s.lib_ops), n_streams=ns, n_sync_edges=len(syncs),
                   graph_nodes_edges=B.opara_exec_info(par), multi_stream_graph_validation=s.capture_log[0],
                   fused_nodes=n_nodes, waves=B.opara_wave_of(s.dag)[1],
                   assign_streams_ms=(t1 - t0) * 1e3, order_launch_ms=(t2 - t1) * 1e3, capture_ms=(t4 - t3) * 1e3,
                   sequential_and_fused_capture_ms=(t5 - t4) * 1e3, persistent_queue=B.ORDER_POLICY_NAMES[per_policy],
                   persistent_queue_probe_us={B.ORDER_POLICY_NAMES[k]: v for k, v in probe.items()},
                   sequential=r_seq, parallel=runs["multi_stream_graph"], persistent=runs["persistent"], chained=runs["chained"],
                   fused=runs["fused"], chained_blocks=B.opara_persistent_info(chn)[0],
                   persistent_timeline=timeline_summary(s, per), best_mode=best, best=r_best,
                   speedup_vs_sequential=r_seq["median_us"] / r_best["median_us"],
                   speedup_multi_stream_graph=r_seq["median_us"] / runs["multi_stream_graph"]["median_us"],
                   speedup_persistent=r_seq["median_us"] / runs["persistent"]["median_us"],
                   speedup_chained=r_seq["median_us"] / runs["chained"]["median_us"],
                   speedup_fused=r_seq["median_us"] / runs["fused"]["median_us"],
                   dag_flops=roof["flops"], dag_bytes=roof["bytes"],
                   roofline_us=dict(flops=roof["t_flops_us"], bytes=roof["t_bytes_us"], critical_path=roof["t_cp_us"],
                                    bound=roof["t_roof_us"]),
                   roofline_fraction=roof["t_roof_us"] / r_best["median_us"],
                   device_memory_bytes=dict(tensors=int(mem_session), with_executor_workspaces=int(torch.cuda.memory_allocated() - mem0),
                                            peak_during_run=int(torch.cuda.max_memory_allocated())))
        # ---- kernel-level roofline: the kernel that takes most of the best executor's time
        work = {v: roof["per_op"][s.lib_ops[v]] for v in range(len(s.lib_ops))}
        st = s.make_streams(1)
        t_iso = isolated_op_times(s)
        dem = B.opara_get_demands(s.dag)
        by = {}
        for v, (d, t) in enumerate(zip(dem, t_iso)):
            e = by.setdefault(B.opara_kernel_info(d.kernel_id)[0], dict(launches=0, time_us=0.0, flops=0, bytes=0))
            e["launches"] += 1; e["time_us"] += t; e["flops"] += work[v][0]; e["bytes"] += work[v][1]
        dom = max(by, key=lambda k: by[k]["time_us"])
        res["dominant_graph_kernel"] = kernel_block(dom, by[dom]["flops"], by[dom]["bytes"], by[dom]["launches"],
                                                    by[dom]["time_us"], wl.dtype, traffic.get((wl.name, dom + tag)))
        res["sum_isolated_us"] = float(sum(t_iso))
        finish = [0.0] * len(wl.ops)
        for op in wl.ops:                     # a removed concatenation takes no time of its own
            t_op = t_iso[s.lib_id[op.id]] if op.id in s.lib_id else 0.0
            finish[op.id] = max([finish[u] for u in op.inputs if u >= 0], default=0.0) + t_op
        res["critical_path_isolated_us"] = float(max(finish))
        res["kernels"] = {k: dict(launches=v["launches"], avg_us=v["time_us"] / v["launches"]) for k, v in by.items()}
        if best == "fused":
            # every node launched by itself between HIP events on the launch stream; nodes grouped by kernel
            us = B.opara_fused_time_nodes(fus, st.handles[0], max(20, min(steps, 200)))
            names = B.opara_fused_node_kernels(fus, wl.dtype)
            fk = {}
            for node, (name, t) in enumerate(zip(names, us)):
                e = fk.setdefault(name, dict(launches=0, time_us=0.0, flops=0, bytes=0, ops=0))
                members = [v for v in range(len(node_of)) if node_of[v] == node]
                e["launches"] += 1; e["time_us"] += t; e["ops"] += len(members)
                e["flops"] += sum(work[v][0] for v in members); e["bytes"] += sum(work[v][1] for v in members)
            dom = max(fk, key=lambda k: fk[k]["time_us"])
            kern = kernel_block(dom, fk[dom]["flops"], fk[dom]["bytes"], fk[dom]["launches"], fk[dom]["time_us"], wl.dtype,
                                traffic.get((wl.name, dom + tag)), operators_in_these_launches=fk[dom]["ops"],
                                share_of_node_time=fk[dom]["time_us"] / sum(us))
            res["fused_node_kernels"] = {k: dict(launches=v["launches"], avg_us=v["time_us"] / v["launches"], operators=v["ops"])
                                         for k, v in fk.items()}
            res["fused_sum_of_node_times_us"] = float(sum(us))
        elif best in ("persistent", "chained"):
            # one kernel runs the DAG behind its serial prefix: launched alone between HIP events on the
            # launch stream; its work is the operators inside it
            one = per if best == "persistent" else chn
            t_us = B.opara_persistent_time_kernel(one, st.handles[0], steps)
            if s.persistent_status(one) != 0:
                raise RuntimeError(best + " executor: a wait ran out")
            queue = B.opara_order_launch_policy(s.dag, per_policy if best == "persistent" else B.ORDER_ALG2)
            inside = queue[B.opara_persistent_prefix(one):]
            kern = kernel_block(("persist_" if best == "persistent" else "chain_") + wl.dtype, sum(work[v][0] for v in inside), sum(work[v][1] for v in inside), 1,
                                t_us, wl.dtype, traffic.get((wl.name, ("persist_" if best == "persistent" else "chain_") + wl.dtype + tag)),
                                operators_in_kernel=len(inside))
        else:
            kern = res["dominant_graph_kernel"]
        res["roofline"] = kern
        # ---- overlap measured inside the kernels (operator timeline: no profiler attached)
        from paper_2312_10351_amd.timeline import operator_overlap
        res["operator_overlap"] = {name: operator_overlap(s.operator_trace(mode))
                                   for name, mode in (("sequential", B.SEQUENTIAL), ("multi_stream_graph", B.PARALLEL), ("fused", B.FUSED))}
        # ---- the oracle on the host cores, and the timed executor's result against it
        if cpu_budget_s > 0:
            block, ref = oracle_pass(wl, cpu_budget_s, one_thread=index == 1)
            s.clear_outputs()
            s.replay({"multi_stream_graph": par, "persistent": per, "chained": chn, "fused": fus}[best])
            worst, ok = 0.0, True
            for v in wl.sinks():
                g, o = s.output(v).astype(np.float64), ref[v].astype(np.float64)
                err = np.abs(g - o)
                tol = (2e-2 * np.abs(o) + 1e-2) if wl.dtype == "f16" else (1e-4 * np.abs(o) + 1e-6 * np.abs(o).max())
                worst, ok = max(worst, float(err.max())), ok and bool((err <= tol).all())
            block["timed_executor_matches_oracle"] = dict(executor=best, sinks=len(wl.sinks()), max_abs_err=worst,
                                                          within_tolerance=ok)
            if not ok:
                raise RuntimeError(f"{wl.name}: the timed executor ({best}) misses the oracle, max |err| {worst:g}")
            res["cpu_baseline"] = block
        return res
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


MODE_TEXT = {
    "persistent": "persistent executor: one hipGraph replay = the serial stem as kernel nodes, then one kernel for the rest "
                  "(work items in launch-queue order, dependencies as completion flags)",
    "chained": "chained executor: one hipGraph replay = the serial stem as kernel nodes, then one launch whose workgroups each run "
               "one tile behind a wait for their operator's predecessors (blocks in launch-queue order)",
    "multi_stream_graph": "multi-stream hipGraph replay (Alg. 1 streams, Alg. 2 launch order)",
    "fused": "fused executor: one hipGraph replay = a chain of kernel nodes, one per wave of the Alg. 2 launch queue; a wave of "
             "several operators is ONE kernel whose grid is the sum of their grids"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--configs", type=str, default="0,2,3,4,5",
                    help="extra configs reported beside the headline one (5 = NASNet-cell-like DAG, not in BASELINE.json)")
    ap.add_argument("--layouts", default="both", choices=["both", "zero_copy", "explicit"],
                    help="concatenation layouts of the headline DAG to run (profiling runs take one)")
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
    traffic = load_traffic()
    cpu = 0.0 if a.no_cpu_baseline else 1.0
    heads = [bench_config(1, a.steps, a.warmup, zero_copy_concat=z, cpu_budget_s=(12.0 if i == 0 else 0.0) * cpu, traffic=traffic)
             for i, z in enumerate([True, False] if a.layouts == "both" else [a.layouts == "zero_copy"])]
    head = min(heads, key=lambda r: r["best"]["median_us"])
    alt = next((r for r in heads if r is not head), None)
    others = [bench_config(idx, max(100, a.steps // 4), a.warmup, cpu_budget_s=1.0 * cpu, traffic=traffic)
              for idx in [int(x) for x in a.configs.split(",") if x != ""]]
    line = {
        "metric": "batch1_dag_latency_us", "value": head["best"]["median_us"], "unit": "us",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["best"]["mean_us"] / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "googlenet_like fp16 batch 1, 1x3x224x224, 81 operators (configs[1])",
                   "concatenation": ("zero-copy: the branches write their channel slices of the concatenated tensor, "
                                     "%d of 81 operators are launched; the sequential baseline uses the same layout"
                                     % head["n_ops_launched"]) if head["zero_copy_concat"] else "explicit concatenation kernels",
                   "mode": MODE_TEXT[head["best_mode"]]},
        "throughput_inferences_per_s": 1e6 / head["best"]["back_to_back_us"],
        "speedup_vs_sequential_hipgraph": head["speedup_vs_sequential"],
        "speedup_by_executor": {k: head["speedup_" + k] for k in ("multi_stream_graph", "persistent", "chained", "fused")},
        "speedup_vs_sequential_hipgraph_all_configs": {r["workload"]: dict(best=r["best_mode"], speedup=r["speedup_vs_sequential"],
                                                                            multi_stream_graph=r["speedup_multi_stream_graph"],
                                                                            persistent=r["speedup_persistent"], chained=r["speedup_chained"],
                                                                            fused=r["speedup_fused"])
                                                       for r in [head] + others},
        "dag_roofline_fraction": head["roofline_fraction"],
        "roofline": head["roofline"],
        "headline": head,
        "headline_other_concatenation": alt,
        "other_configs": others,
    }
    if "cpu_baseline" in heads[0]:
        line["cpu_baseline"] = heads[0]["cpu_baseline"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
