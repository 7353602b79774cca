"""Seeded synthetic operator DAGs and tensors (data only).

This package describes workloads: which operators exist, how they are wired,
their shapes, and the seeded random tensors they consume.  It contains no
operator arithmetic and no scheduling logic, so both the CPU oracle and the
HIP path can consume it without sharing any of the method's code.
"""
from .dag import Op, Workload, OP_TYPES, COMPUTE_TYPES
from .configs import (Builder, build_config, CONFIG_NAMES, inception_block, googlenet_like,
                      inception_v3_like, bert_base_like, random_wide_dag, nasnet_like,
                      random_small_dag, appendix_example_edges)

__all__ = ["Builder", "Op", "Workload", "OP_TYPES", "COMPUTE_TYPES", "build_config", "CONFIG_NAMES",
           "inception_block", "googlenet_like", "inception_v3_like", "bert_base_like",
           "random_wide_dag", "nasnet_like", "random_small_dag", "appendix_example_edges"]
