"""Plain data records for an operator DAG G=(V,E) (paper Sec. 3.1, "Definition of a model DAG").

Logical tensor conventions (both executors agree on these; physical layouts are
each executor's own business):
  * CNN activations: [C, H, W] per image; with Workload.batch = B > 1 every image
    tensor carries a leading batch axis [B, C, H, W] while operator records keep the
    per-image shapes.
  * matrices: [R, C] row-major.
  * an operator views each input as the leading prefix of its producer's flat
    row-major buffer, reshaped to the input shape the operator states.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple
import numpy as np

OP_TYPES = ("conv2d", "gemm", "bgemm", "maxpool", "avgpool", "gavgpool", "concat",
            "layernorm", "softmax", "gelu", "relu", "add")
# operator-table classes (paper Sec. 3.3: compute-intensive vs memory-intensive)
COMPUTE_TYPES = ("conv2d", "gemm", "bgemm")


@dataclass
class Op:
    id: int
    type: str
    inputs: List[int]                 # producer ids in argument order; -(slot+1) = external tensor
    in_shapes: List[Tuple[int, ...]]  # logical shape each input is viewed in
    out_shape: Tuple[int, ...]
    params: Dict = field(default_factory=dict)
    name: str = ""


@dataclass
class Workload:
    name: str
    dtype: str                        # "f32" | "f16"
    ops: List[Op]
    ext_inputs: List[np.ndarray]      # already rounded to dtype
    weights: Dict[int, Dict[str, np.ndarray]]  # op id -> {"w": ..., "b": ...}, rounded to dtype
    seed: int = 0
    batch: int = 1                    # images per pass; image tensors are then [batch, C, H, W]

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16

    def edges(self):
        """Operator-to-operator edges (u, v), deduplicated, in argument order."""
        out = []
        for op in self.ops:
            seen = set()
            for u in op.inputs:
                if u >= 0 and u not in seen:
                    seen.add(u)
                    out.append((u, op.id))
        return out

    def sinks(self):
        has_succ = set(u for u, _ in self.edges())
        return [op.id for op in self.ops if op.id not in has_succ]


def concat_elision_plan(wl):
    """Channel concatenations whose branches can write their slices in place (zero-copy
    concatenation): every input is the whole output of a distinct convolution that has no
    other consumer.  Returns {concat id: [(producer id, first channel, channels), ...]}.
    Pure graph bookkeeping; what is done with the plan is each executor's business."""
    consumers = {}
    for op in wl.ops:
        for u in op.inputs:
            if u >= 0:
                consumers.setdefault(u, []).append(op.id)
    plan = {}
    for op in wl.ops:
        if op.type != "concat" or op.params.get("axis") != 0:
            continue
        ok = len(set(op.inputs)) == len(op.inputs)
        parts, off = [], 0
        for u, shp in zip(op.inputs, op.in_shapes):
            ok = ok and u >= 0 and wl.ops[u].type == "conv2d" and consumers.get(u) == [op.id] \
                and tuple(wl.ops[u].out_shape) == tuple(shp)
            parts.append((u, off, shp[0]))
            off += shp[0]
        ok = ok and all(tuple(wl.ops[v].in_shapes[i]) == tuple(op.out_shape)
                        for v in consumers.get(op.id, []) for i, u in enumerate(wl.ops[v].inputs) if u == op.id)
        if ok:
            plan[op.id] = parts
    return plan


def reduced_dag(wl, plan):
    """The DAG without the concatenations in `plan`: an operator that read such a
    concatenation depends on its producers instead.  Returns (kept, preds): `kept[i]` is the
    workload id of reduced operator i; `preds[i]` its predecessors in reduced numbering,
    ordered as arguments that are operators first, then the producers standing in for each
    elided concatenation (argument order), without repeats."""
    kept = [op.id for op in wl.ops if op.id not in plan]
    new_id = {v: i for i, v in enumerate(kept)}
    preds = []
    for v in kept:
        op = wl.ops[v]
        direct = [u for u in op.inputs if u >= 0 and u not in plan]
        via = [p for u in op.inputs if u in plan for p, _, _ in plan[u]]
        seen, row = set(), []
        for u in direct + via:
            if u not in seen:
                seen.add(u)
                row.append(new_id[u])
        preds.append(row)
    return kept, preds
