// Interface between the kernel translation unit and the graph capturer.
#pragma once
#include <hip/hip_runtime.h>
#include "kernel_args.h"

namespace opara {
hipError_t launch_plan(const KernelPlan &p, hipStream_t s);
const void *kernel_symbol(int kernel_id);
hipError_t launch_noop(hipStream_t s);
// Explicit graph construction: one kernel node for a planned launch / for the kernel
// without work, depending on deps[0..n_deps).
hipError_t add_plan_node(hipGraph_t graph, const KernelPlan &p, const hipGraphNode_t *deps, size_t n_deps,
                         hipGraphNode_t *node);
hipError_t add_noop_node(hipGraph_t graph, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node);
}  // namespace opara
