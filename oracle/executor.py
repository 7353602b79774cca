"""Sequential DAG executor (test oracle; not used by the product path).

Runs every operator once, one at a time, in a topological order (Kahn, smallest id
first by default).  Any valid schedule of the DAG must reproduce this result, so
this is the definition the parallel GPU executor is compared with (paper Sec. 3.1:
the stream allocation plan changes how operators are parallelised, not what they
compute).  Precision reading: operators accumulate in fp64; every operator output
is rounded to the workload's storage type (fp32 or fp16, round-to-nearest-even)
before any consumer reads it.
"""
import heapq
import numpy as np
from . import ops as O


def kahn_order(n, edges, key=None):
    """Topological order choosing the ready operator with the smallest key (id)."""
    succ = [[] for _ in range(n)]
    indeg = [0] * n
    for u, v in edges:
        succ[u].append(v)
        indeg[v] += 1
    key = key or (lambda v: v)
    heap = [(key(v), v) for v in range(n) if indeg[v] == 0]
    heapq.heapify(heap)
    order = []
    while heap:
        _, v = heapq.heappop(heap)
        order.append(v)
        for s in succ[v]:
            indeg[s] -= 1
            if indeg[s] == 0:
                heapq.heappush(heap, (key(s), s))
    if len(order) != n:
        raise ValueError("graph has a cycle")
    return order


def _view(buf, shape):
    n = int(np.prod(shape))
    flat = buf.reshape(-1)
    assert flat.size >= n, "producer too small for the consumer's view"
    return flat[:n].reshape(shape)


_IMAGE_OPS = ("conv2d", "maxpool", "avgpool", "gavgpool")


_ELEMENTWISE_OPS = ("add", "relu", "gelu")


def is_image_op(op):
    """Operators whose tensors are [C, H, W] images (one per batch entry): the image
    operators proper, channel concatenation, and element-wise operators stated on 3-D shapes."""
    return op.type in _IMAGE_OPS or (op.type == "concat" and op.params.get("axis") == 0) \
        or (op.type in _ELEMENTWISE_OPS and len(op.out_shape) == 3)


def run_op(op, ins, wts):
    """ins: fp64 arrays already viewed in op.in_shapes; returns fp64 result."""
    p, t = op.params, op.type
    if t == "conv2d":
        return O.conv2d(ins[0], wts["w"].astype(np.float64), wts["b"].astype(np.float64),
                        (p["sh"], p["sw"]), (p["ph"], p["pw"]), p["relu"])
    if t == "gemm":
        return O.gemm(ins[0], wts["w"].astype(np.float64), wts["b"].astype(np.float64),
                      ins[1:], p.get("relu", False))
    if t == "bgemm":
        if p["mode"] == "qk":
            return O.bgemm_qk(ins[0], ins[1], p["heads"], p["alpha"])
        return O.bgemm_pv(ins[0], ins[1], p["heads"], p["alpha"])
    if t == "maxpool":
        return O.maxpool(ins[0], (p["kh"], p["kw"]), (p["sh"], p["sw"]), (p["ph"], p["pw"]))
    if t == "avgpool":
        return O.avgpool(ins[0], (p["kh"], p["kw"]), (p["sh"], p["sw"]), (p["ph"], p["pw"]))
    if t == "gavgpool":
        return O.gavgpool(ins[0])
    if t == "concat":
        return O.concat(ins, p["axis"])
    if t == "layernorm":
        return O.layernorm(ins, p["eps"])
    if t == "softmax":
        return O.softmax(ins)
    if t == "gelu":
        return O.gelu(ins)
    if t == "relu":
        return O.relu(ins)
    if t == "add":
        return O.add(ins)
    raise ValueError(f"unknown operator type {t}")


def run_dag(wl, order=None, keep=None):
    """Execute workload `wl`; returns {op id: output rounded to wl dtype (as stored)}.
    keep: iterable of op ids whose outputs to return (default: all)."""
    n = len(wl.ops)
    order = kahn_order(n, wl.edges()) if order is None else list(order)
    st = wl.np_dtype
    remaining = [0] * n
    for op in wl.ops:
        for u in op.inputs:
            if u >= 0:
                remaining[u] += 1
    keep = set(range(n)) if keep is None else set(keep)
    out = {}
    for v in order:
        op = wl.ops[v]
        batched = wl.batch > 1 and is_image_op(op)     # image operators act on each image alone
        ins = []
        for u, shp in zip(op.inputs, op.in_shapes):
            src = wl.ext_inputs[-u - 1] if u < 0 else out[u]
            ins.append(_view(src, ((wl.batch,) + tuple(shp)) if batched else shp).astype(np.float64))
        if batched:
            y = np.stack([run_op(op, [a[b] for a in ins], wl.weights.get(v)) for b in range(wl.batch)])
            assert y.shape[1:] == tuple(op.out_shape), (op.name, y.shape, op.out_shape)
        else:
            y = run_op(op, ins, wl.weights.get(v))
            assert y.shape == tuple(op.out_shape), (op.name, y.shape, op.out_shape)
        out[v] = y.astype(st)
        for u in op.inputs:
            if u >= 0:
                remaining[u] -= 1
                if remaining[u] == 0 and u not in keep:
                    del out[u]
    return {v: a for v, a in out.items() if v in keep}
