"""Algorithmic work of a workload and the DAG roofline bound (bookkeeping only).

Per operator: FLOPs = 2*M*N*K for the contractions (convolution through its GEMM view,
batched GEMM summed over the batch), 0 otherwise; bytes = every input read once +
weights read once + output written once.  The DAG bound is
    T_roof = max( sum FLOPs / P_mfma, sum bytes / B_hbm, T_cp )
with T_cp the longest dependency path when each operator costs
max(FLOPs/P_mfma, bytes/B_hbm).
"""
import numpy as np

HBM_BYTES_PER_S = 8.0e12                       # MI355X HBM3E, published
MFMA_FLOPS = {"f16": 2.5e15, "f32": 157.3e12}  # dense matrix peaks, published


def _numel(shape):
    return int(np.prod(shape))


def op_work(op, dtype):
    """(flops, bytes) of one operator."""
    es = 2 if dtype == "f16" else 4
    p = op.params
    flops = 0
    wbytes = 0
    if op.type == "conv2d":
        m = op.out_shape[1] * op.out_shape[2]
        k = p["cin"] * p["kh"] * p["kw"]
        flops = 2 * m * p["cout"] * k
        wbytes = p["cout"] * k * es
    elif op.type == "gemm":
        flops = 2 * p["m"] * p["n"] * p["k"]
        wbytes = p["k"] * p["n"] * es
    elif op.type == "bgemm":
        s, d, h = p["seq"], p["dhead"], p["heads"]
        flops = 2 * h * s * s * d
    nbytes = wbytes + _numel(op.out_shape) * es + sum(_numel(s) for s in op.in_shapes) * es
    return flops, nbytes


def dag_roofline(wl):
    dt = wl.dtype
    peak = MFMA_FLOPS[dt]
    work = [op_work(op, dt) for op in wl.ops]
    t_op = [max(f / peak, b / HBM_BYTES_PER_S) for f, b in work]
    finish = [0.0] * len(wl.ops)
    for op in wl.ops:                       # ids are a topological order
        start = max([finish[u] for u in op.inputs if u >= 0], default=0.0)
        finish[op.id] = start + t_op[op.id]
    flops = sum(f for f, _ in work)
    nbytes = sum(b for _, b in work)
    t_flops, t_bytes, t_cp = flops / peak, nbytes / HBM_BYTES_PER_S, max(finish)
    return dict(flops=flops, bytes=nbytes, t_flops_us=t_flops * 1e6, t_bytes_us=t_bytes * 1e6,
                t_cp_us=t_cp * 1e6, t_roof_us=max(t_flops, t_bytes, t_cp) * 1e6, per_op=work)
