"""Replays one executor of one config a number of times and exits: the program to put
under a profiler (rocprofv3 --kernel-trace for a timeline of the multi-stream graph,
--pmc for counters of one executor's kernels).

  python -m paper_2312_10351_amd.replay --config 1 --mode par [--replays 20] [--zero-copy-concat]
  modes: seq (sequential graph), par (multi-stream graph), pruned, persist, fused, eager
Prints the number of kernels one replay launches and the median replay latency.
"""
import argparse
import time

import numpy as np


def main():
    from . import binding as B
    from .runtime import Session
    from workloads import build_config
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--mode", default="par", choices=["seq", "par", "pruned", "persist", "fused", "eager"])
    ap.add_argument("--replays", type=int, default=20)
    ap.add_argument("--policy", default="alg2", choices=list(B.ORDER_POLICY_NAMES))
    ap.add_argument("--zero-copy-concat", action="store_true")
    a = ap.parse_args()
    pol = list(B.ORDER_POLICY_NAMES).index(a.policy)
    s = Session(build_config(a.config), zero_copy_concat=a.zero_copy_concat)
    try:
        if a.mode == "persist":
            exe = s.capture_persistent(policy=pol)
        elif a.mode != "eager":
            exe = s.capture({"seq": B.SEQUENTIAL, "par": B.PARALLEL, "pruned": B.PARALLEL_PRUNED, "fused": B.FUSED}[a.mode], policy=pol)
        lat = []
        for _ in range(a.replays):
            t0 = time.perf_counter()
            s.run_eager() if a.mode == "eager" else s.replay(exe)
            lat.append((time.perf_counter() - t0) * 1e6)
        nodes = len(s.lib_ops) if a.mode == "eager" else B.opara_exec_info(exe)[0]
        print(f"{s.wl.name} [{a.mode}]: {nodes} kernels per replay, {a.replays} replays, median {np.median(lat):.1f} us "
              f"(host-timed launch + synchronise)")
    finally:
        s.close()


if __name__ == "__main__":
    main()
