"""Isolated HBM fraction of the streaming kernels (element-wise, row-wise, concatenation)
at the tensor sizes the configs draw (1-8 MB) and at 128 MB.

  python -m paper_2312_10351_amd.streaming [--sizes-mb 1,4,8,128] [--reps 50] [--cold]

Each operator is launched `reps` times back to back on one stream between two events on
that stream; achieved = algorithmic bytes (every input and the output once) / time per
launch, against the published 8 TB/s.  Tensors of up to 64 MB stay in the 256 MB memory-side
cache between launches, so the default figures are warm-cache ones; --cold runs each launch
after a 512 MB fill that evicts it.  Markdown table on stdout.
"""
import argparse

import numpy as np

PEAK = 8.0e12


def cases(mb, dtype="f16"):
    from workloads import Builder
    es = 2 if dtype == "f16" else 4
    cols = 4096
    rows = max(1, mb * 1024 * 1024 // es // cols)
    out = []
    for name, kind, n_in in (("relu", "relu", 1), ("gelu", "gelu", 1), ("add x2", "add", 2), ("add x3", "add", 3),
                             ("layernorm", "layernorm", 1), ("softmax", "softmax", 1), ("concat x2", "concat", 2)):
        b = Builder(name, dtype)
        if kind == "concat":
            xs = [b.ext((rows, cols // 2)), b.ext((rows, cols // 2))]
            b.add("concat", xs, [(rows, cols // 2)] * 2, (rows, cols), {"axis": 1})
            nbytes = 2 * rows * cols * es
        else:
            xs = [b.ext((rows, cols)) for _ in range(n_in)]
            b.rowwise(kind, xs, rows, cols, {"eps": 1e-5})
            nbytes = (n_in + 1) * rows * cols * es
        out.append((name, b.build(1), nbytes))
    return out


def time_op(session, reps, cold):
    import torch
    from . import binding as B
    st = session.make_streams(1)
    h, ts = st.handles[0], st.torch_streams[0]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        B.opara_launch_op(session.dag, 0, h)
    ts.synchronize()
    if not cold:
        e0.record(ts)
        for _ in range(reps):
            B.opara_launch_op(session.dag, 0, h)
        e1.record(ts)
        ts.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps
    junk = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device="cuda")
    t = []
    for _ in range(min(reps, 10)):
        with torch.cuda.stream(ts):
            junk.fill_(1)
        e0.record(ts)
        B.opara_launch_op(session.dag, 0, h)
        e1.record(ts)
        ts.synchronize()
        t.append(e0.elapsed_time(e1) * 1e3)
    return float(np.median(t))


def main():
    from . import binding as B
    from .runtime import Session
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes-mb", default="1,4,8,128")
    ap.add_argument("--reps", type=int, default=50)
    ap.add_argument("--cold", action="store_true")
    a = ap.parse_args()
    sizes = [int(x) for x in a.sizes_mb.split(",")]
    print("| operator (fp16, rows x 4096) | kernel | " + " | ".join(f"{mb} MB: us, GB/s, % of 8 TB/s" for mb in sizes) + " |")
    print("|---|---|" + "---|" * len(sizes))
    rows = {}
    for mb in sizes:
        for name, wl, nbytes in cases(mb):
            s = Session(wl)
            try:
                kernel = B.opara_kernel_info(B.opara_get_demands(s.dag)[0].kernel_id)[0]
                us = time_op(s, a.reps, a.cold)
            finally:
                s.close()
            rows.setdefault(name, [kernel])
            rows[name].append(f"{us:.1f}, {nbytes / us / 1e3:.0f}, {100 * nbytes / (us * 1e-6) / PEAK:.0f} %")
    for name, cells in rows.items():
        print(f"| {name} | {cells[0]} | " + " | ".join(cells[1:]) + " |")


if __name__ == "__main__":
    main()
