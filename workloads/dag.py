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
