"""Launch-order and interference ablations over the same kernels and graphs.

  python -m paper_2312_10351_amd.ablation [--configs 0,1,2,3,4] [--replays 300] [--batches 1,2,4,8,16,32] [--concat-configs 0,1,2] [--stream-configs 0,1,2,3,4] [--markdown]

Part 1 (paper Sec. 2.3, "GPU blocking"): the parallel graph is captured with each
launch-order policy of opara_order_launch_policy and replayed; only the queue differs.
Part 2 (paper Sec. 2.3, "Performance interference"): two independent operators are
replayed alone, back to back on one stream, and side by side on two streams, for a
compute-intensive + memory-intensive pair and for two pairs of one class.
Part 3 (paper Sec. 5.2): batch sweep of the Inception-v3-like DAG.
Part 4: zero-copy concatenation against explicit concatenation kernels (CNN configs).
Part 5: stream-allocation policies (Alg. 1 / fewest streams) with and without pruning of implied
        synchronisations: streams, synchronisations, host time, latency.
Prints one JSON object per line (and, with --markdown, the same records as tables at the end).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def replay_latency(session, exe, replays, warmup=30):
    from . import binding as B
    st = session.make_streams(1)
    h, ts = st.handles[0], st.torch_streams[0]
    for _ in range(warmup):
        B.opara_replay(exe, h)
    ts.synchronize()
    lat = []
    for _ in range(replays):
        t0 = time.perf_counter()
        B.opara_replay(exe, h)
        ts.synchronize()
        lat.append((time.perf_counter() - t0) * 1e6)
    return float(np.median(lat))


def order_ablation(index, replays):
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    wl = build_config(index)
    s = Session(wl)
    try:
        row = {"ablation": "launch_order", "workload": wl.name, "n_ops": len(wl.ops)}
        row["sequential_us"] = replay_latency(s, s.capture(B.SEQUENTIAL), replays)
        for pid, name in enumerate(B.ORDER_POLICY_NAMES):
            row[name + "_us"] = replay_latency(s, s.capture(B.PARALLEL, policy=pid), replays)
        for pid, name in enumerate(B.ORDER_POLICY_NAMES):      # the same queues as work-item orders
            row["persistent_" + name + "_us"] = replay_latency(s, s.capture_persistent(policy=pid), replays)
        for pid, name in enumerate(B.ORDER_POLICY_NAMES):      # ... and as the order inside the fused executor's waves
            row["fused_" + name + "_us"] = replay_latency(s, s.capture(B.FUSED, policy=pid), replays)
        return row
    finally:
        s.close()


def batch_sweep(batch, replays):
    """Inception-v3-like DAG at a given batch size: latency and images/s of the parallel and
    the sequential graph (paper Sec. 5.2, throughput under different batch sizes)."""
    from . import binding as B
    from .runtime import Session
    from workloads import inception_v3_like
    wl = inception_v3_like(batch=batch)
    s = Session(wl)
    try:
        seq = replay_latency(s, s.capture(B.SEQUENTIAL), replays)
        par = replay_latency(s, s.capture(B.PARALLEL), replays)
        per = replay_latency(s, s.capture_persistent(), replays)
        fus = replay_latency(s, s.capture(B.FUSED), replays)
        return {"ablation": "batch_sweep", "workload": wl.name, "batch": batch, "sequential_us": seq,
                "parallel_us": par, "persistent_us": per, "fused_us": fus, "speedup": seq / par, "speedup_persistent": seq / per,
                "speedup_fused": seq / fus, "fused_images_per_s": batch * 1e6 / fus,
                "parallel_images_per_s": batch * 1e6 / par, "persistent_images_per_s": batch * 1e6 / per,
                "sequential_images_per_s": batch * 1e6 / seq}
    finally:
        s.close()


def concat_ablation(index, replays):
    """Zero-copy concatenation (branches write channel slices in place, the concatenation
    operators disappear) against explicit concatenation kernels, per executor."""
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    wl = build_config(index)
    out = {"ablation": "zero_copy_concat", "workload": wl.name, "concats": sum(o.type == "concat" for o in wl.ops)}
    for tag, zc in (("explicit", False), ("zero_copy", True)):
        s = Session(wl, zero_copy_concat=zc)
        try:
            if zc:
                out["elided"] = len(s.elided)
            out[tag] = {"sequential_us": replay_latency(s, s.capture(B.SEQUENTIAL), replays),
                        "multi_stream_graph_us": replay_latency(s, s.capture(B.PARALLEL), replays),
                        "persistent_us": replay_latency(s, s.capture_persistent(), replays),
                        "fused_us": replay_latency(s, s.capture(B.FUSED), replays)}
        finally:
            s.close()
    return out


def stream_policy_ablation(index, replays):
    """Alg. 1 against the fewest-streams allocation (the matching-based policy the paper
    compares with, Sec. 5.2 / 5.4), each with all synchronisations and with the implied ones
    pruned: streams, synchronisations, graph edges, allocation time on the host, latency."""
    import time
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    wl = build_config(index)
    s = Session(wl)
    try:
        row = {"ablation": "stream_policy", "workload": wl.name, "n_ops": len(wl.ops),
               "sequential_us": replay_latency(s, s.capture(B.SEQUENTIAL), replays)}
        for name, pol in (("alg1", B.STREAMS_ALG1), ("min_streams", B.STREAMS_MIN)):
            best = 1e9
            for _ in range(5):
                t0 = time.perf_counter()
                _, ns = B.opara_assign_streams_policy(s.dag, pol)
                best = min(best, time.perf_counter() - t0)
            B.opara_order_launch(s.dag)
            r = {"n_streams": ns, "assign_ms": best * 1e3, "syncs": len(B.opara_sync_edges(s.dag)),
                 "syncs_pruned": len(B.opara_sync_edges_pruned(s.dag))}
            for tag, mode in (("graph", B.PARALLEL), ("graph_pruned", B.PARALLEL_PRUNED)):
                exe = s.capture(mode, stream_policy=pol)
                r[tag + "_edges"] = B.opara_exec_info(exe)[1]
                r[tag + "_us"] = replay_latency(s, exe, replays)
            row[name] = r
        return row
    finally:
        s.close()


def _pair(kind_a, kind_b):
    """Two independent operators of the given classes reading the same external tensor."""
    from workloads import Builder
    b = Builder(f"{kind_a}_{kind_b}", "f16")
    x = b.ext((512, 4096))
    big = b.ext((8192, 8192))
    for kind in (kind_a, kind_b):
        if kind == "comp":
            b.gemm(x, 512, 4096, 4096)                    # 17 GFLOP, 32 MB of weights
        else:
            b.rowwise("gelu", [big], 8192, 8192)          # 128 MB read + 128 MB written
    return b


def interference(kind_a, kind_b, replays):
    from . import binding as B
    from .runtime import Session
    from workloads import Builder
    row = {"ablation": "interference", "pair": f"{kind_a}||{kind_b}"}
    wl = _pair(kind_a, kind_b).build(3)
    s = Session(wl)
    try:
        row["sequential_us"] = replay_latency(s, s.capture(B.SEQUENTIAL), replays)
        row["parallel_us"] = replay_latency(s, s.capture(B.PARALLEL), replays)
        row["persistent_us"] = replay_latency(s, s.capture_persistent(), replays)
        row["fused_us"] = replay_latency(s, s.capture(B.FUSED), replays)
    finally:
        s.close()
    for tag, kind in (("a", kind_a), ("b", kind_b)):
        b = Builder("single", "f16")
        if kind == "comp":
            b.gemm(b.ext((512, 4096)), 512, 4096, 4096)
        else:
            b.rowwise("gelu", [b.ext((8192, 8192))], 8192, 8192)
        s = Session(b.build(3))
        try:
            row[f"alone_{tag}_us"] = replay_latency(s, s.capture(B.SEQUENTIAL), replays)
        finally:
            s.close()
    row["overlap_gain"] = row["sequential_us"] / row["parallel_us"]
    return row


def render_markdown(records):
    """The records of one run as markdown tables (microseconds), one section per ablation."""
    from . import binding as B
    out = []
    by = lambda kind: [r for r in records if r["ablation"] == kind]
    pol = list(B.ORDER_POLICY_NAMES)
    if by("launch_order"):
        for title, prefix in (("Launch order, multi-stream graph", ""), ("Launch order, persistent executor", "persistent_"),
                              ("Launch order, fused executor", "fused_")):
            out += ["", f"### {title}", "", "| workload | sequential graph | " + " | ".join(pol) + " |", "|---|---|" + "---|" * len(pol)]
            for r in by("launch_order"):
                out.append(f"| {r['workload']} ({r['n_ops']}) | {r['sequential_us']:.1f} | " +
                           " | ".join(f"{r[prefix + n + '_us']:.1f}" for n in pol) + " |")
    if by("interference"):
        out += ["", "### Interference pairs", "",
                "| pair | A alone | B alone | one stream, back to back | two streams (graph) | gain | persistent executor | fused executor (one kernel) |",
                "|---|---|---|---|---|---|---|---|"]
        for r in by("interference"):
            out.append(f"| {r['pair']} | {r['alone_a_us']:.1f} | {r['alone_b_us']:.1f} | {r['sequential_us']:.1f} | "
                       f"{r['parallel_us']:.1f} | {r['overlap_gain']:.2f}x | {r['persistent_us']:.1f} | {r['fused_us']:.1f} |")
    if by("batch_sweep"):
        out += ["", "### Batch sweep", "",
                "| batch | sequential us | multi-stream graph us | persistent us | fused us | graph speed-up | persistent speed-up | fused speed-up | best images/s |",
                "|---:|---:|---:|---:|---:|---:|---:|---:|---:|"]
        for r in by("batch_sweep"):
            best = max(r["parallel_images_per_s"], r["persistent_images_per_s"], r["sequential_images_per_s"], r["fused_images_per_s"])
            out.append(f"| {r['batch']} | {r['sequential_us']:.0f} | {r['parallel_us']:.0f} | {r['persistent_us']:.0f} | {r['fused_us']:.0f} | "
                       f"{r['speedup']:.2f} | {r['speedup_persistent']:.2f} | {r['speedup_fused']:.2f} | {best:,.0f} |")
    if by("zero_copy_concat"):
        out += ["", "### Zero-copy concatenation", "",
                "| workload | concats | elided | layout | sequential graph | multi-stream graph | persistent executor | fused executor |",
                "|---|---|---|---|---|---|---|---|"]
        for r in by("zero_copy_concat"):
            for tag in ("explicit", "zero_copy"):
                t = r[tag]
                out.append(f"| {r['workload']} | {r['concats']} | {r['elided']} | {tag} | {t['sequential_us']:.0f} | "
                           f"{t['multi_stream_graph_us']:.0f} | {t['persistent_us']:.0f} | {t['fused_us']:.0f} |")
    if by("stream_policy"):
        out += ["", "### Stream policies and synchronisation pruning", "",
                "| workload | ops | sequential | policy | streams | alloc us | syncs | after pruning | graph edges | graph us | pruned graph us |",
                "|---|---|---|---|---|---|---|---|---|---|---|"]
        for r in by("stream_policy"):
            for name in ("alg1", "min_streams"):
                q = r[name]
                out.append(f"| {r['workload']} | {r['n_ops']} | {r['sequential_us']:.0f} | {name} | {q['n_streams']} | "
                           f"{q['assign_ms'] * 1e3:.1f} | {q['syncs']} | {q['syncs_pruned']} | "
                           f"{q['graph_edges']} -> {q['graph_pruned_edges']} | {q['graph_us']:.0f} | {q['graph_pruned_us']:.0f} |")
    return "\n".join(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="0,1,2,3,4")
    ap.add_argument("--replays", type=int, default=300)
    ap.add_argument("--batches", default="1,2,4,8,16,32")
    ap.add_argument("--concat-configs", default="0,1,2")
    ap.add_argument("--stream-configs", default="0,1,2,3,4")
    ap.add_argument("--markdown", action="store_true", help="after the JSON lines, print the same records as tables")
    a = ap.parse_args()
    records = []

    def emit(r):
        records.append(r)
        print(json.dumps(r), flush=True)
    for idx in [int(x) for x in a.stream_configs.split(",") if x]:
        emit(stream_policy_ablation(idx, a.replays))
    for idx in [int(x) for x in a.concat_configs.split(",") if x]:
        emit(concat_ablation(idx, a.replays))
    for bsz in [int(x) for x in a.batches.split(",") if x]:
        emit(batch_sweep(bsz, max(50, a.replays // 3)))
    for idx in [int(x) for x in a.configs.split(",") if x]:
        emit(order_ablation(idx, a.replays))
    for pair in (("comp", "mem"), ("mem", "mem"), ("comp", "comp")):
        emit(interference(*pair, max(50, a.replays // 3)))
    if a.markdown:
        print(render_markdown(records))


if __name__ == "__main__":
    main()
