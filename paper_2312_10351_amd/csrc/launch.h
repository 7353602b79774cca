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

// Dependency self-check (see opara_verify_dependencies): a token node marks its
// operator as done after a short delay and counts predecessors not yet marked.
constexpr int kVerifyMaxOps = 1 << 16;
constexpr int kVerifyMaxPreds = 8;
struct TokenArgs { int32_t epoch, self, n_preds, delay; int32_t preds[kVerifyMaxPreds]; };
hipError_t add_token_node(hipGraph_t graph, const TokenArgs &t, const hipGraphNode_t *deps, size_t n_deps,
                          hipGraphNode_t *node);
hipError_t verify_reset(hipStream_t s);            // clears tokens and the violation counter
hipError_t verify_read(hipStream_t s, int *viol);  // synchronises s, returns the counter
}  // namespace opara
