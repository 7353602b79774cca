"""Operator-parallel DAG executor for AMD MI355X (gfx950): Python binding of libopara.

`binding` mirrors the C ABI one to one (argument marshalling only); `runtime`
turns a workload description into device buffers plus operator descriptors and
drives build -> assign streams -> order launch -> capture -> replay.  Every step of
the method runs inside the native library; there is no CPU fallback.
"""
from . import binding  # noqa: F401
