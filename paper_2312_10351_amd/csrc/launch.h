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

// Group nodes (fused executor): whether a kernel's body can run inside a group kernel at
// all (256-thread bodies) and inside the light flavour (at most 128 vector registers).
bool group_kernel_ok(int kernel_id, bool *light);
// Flavour of group kernel a body needs: 0 stream (at most 64 vector registers), 1 light (128), 2 heavy; -1 none.
int group_flavor(int kernel_id);
hipError_t add_group_node(hipGraph_t graph, bool f16, int flavor, const GroupArgs &ga, uint32_t n_blocks,
                          uint32_t lds_bytes, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node);
hipError_t launch_group(bool f16, int flavor, const GroupArgs &ga, uint32_t n_blocks, uint32_t lds_bytes, hipStream_t s);
hipError_t group_prepare(uint32_t max_lds_bytes);   // raises the dynamic LDS limit of the group kernels once

// Dependency self-check (see opara_verify_dependencies): a token node marks its
// operator as done after a short delay and counts predecessors not yet marked.
constexpr int kVerifyMaxOps = 1 << 16;
constexpr int kVerifyMaxPreds = 16;
struct TokenArgs { int32_t epoch, self, n_preds, delay; int32_t preds[kVerifyMaxPreds]; };
// What a token node is given.  The operator's own argument record sits at offset 0 and the
// record is as large as any kernel's: when the node of an instantiated graph is later
// switched to the operator's kernel, the argument block the runtime holds for the node is
// large enough and already valid for that kernel.
struct TokenNodeArgs { KernelArgs real; TokenArgs tok; };
hipError_t add_token_node(hipGraph_t graph, const TokenNodeArgs &t, const hipGraphNode_t *deps, size_t n_deps,
                          hipGraphNode_t *node);
// Switches a kernel node of an instantiated graph to the planned launch `p` (kernel, grid,
// workgroup size, arguments).  The node keeps its place and dependencies.
hipError_t set_exec_node_plan(hipGraphExec_t exec, hipGraphNode_t node, const KernelPlan &p);

// ---- Persistent executor: the whole DAG as one kernel -------------------------------
// Workgroups of one launch draw (operator, tile) work items from a ticket counter in
// launch-queue order; an item starts once the completion counters of its operator's
// predecessors have reached their tile counts.  Records live in a caller-owned
// workspace.  Positions ("pos") index operators in launch-queue order.
constexpr int kPersistMaxPreds = 8;
constexpr int kPersistItemAlign = 8;             // XCDs: workgroup w runs on XCD w % 8
constexpr int kPersistCounterStride = 64;        // uint32 words between completion counters: one per 256 bytes
constexpr int kPersistReplicas = 32;             // copies of each operator's "complete" flag, 128 bytes apart:
constexpr int kPersistFlagStride = 32;           // a workgroup polls copy (blockIdx % replicas), so that a
                                                 // flag has at most 1/32 of the waiting workgroups polling it
constexpr uint32_t kPersistBodyLds = 2 * (128 + 64) * 144;   // largest body: the 128x64 pipelined tile
constexpr uint32_t kPersistMaxLds = 160 * 1024;                // per workgroup on gfx950
constexpr uint32_t kPersistDefaultSpinLimit = 1u << 22;
constexpr int32_t kPersistActivationB = 0x100;   // added to a record's kernel id: the second
                                                 // operand of the contraction is an activation
struct PersistHeader {            // 64 bytes at the start of the workspace
  uint32_t reserved0;
  uint32_t exited;                // workgroups that have left; reset by the last one out
  uint32_t epoch;                 // launch number (starts at 1); the last workgroup out advances it
  uint32_t error;                 // sticky: 1 + pos of the operator whose wait ran out
  uint32_t spin_limit;            // polls one wait may take before it gives up
  uint64_t trace;                 // device address of the timeline buffer, 0 = off
  uint32_t reserved[9];
};
// Predecessors of one operator as every workgroup keeps them in workgroup memory.
struct PersistPredsLds {
  uint16_t n, tiles;               // predecessors; tiles of this operator
  uint16_t chunk, pad;             // consecutive tiles one work item runs (>= 1)
  uint16_t pos[kPersistMaxPreds];
};
constexpr uint32_t persist_lds_bytes(uint32_t n) {
  return kPersistBodyLds + 16 + 4 * (n + 1) + (uint32_t)sizeof(PersistPredsLds) * n;
}
struct PersistOp { int32_t kernel, gx, gy, gz; KernelArgs args; };
struct PersistArgs {
  PersistHeader *hdr;
  uint32_t *done;                 // [n * kPersistCounterStride] tiles finished per operator (every
                                  // kPersistCounterStride-th word); the workgroup that finishes the
                                  // last tile sets it back to 0 and raises the operator's flags
  uint32_t *flags;                // [n * kPersistReplicas * kPersistFlagStride]: copy r of operator p at
                                  // word (p * kPersistReplicas + r) * kPersistFlagStride holds the
                                  // number of the last launch in which p completed
  const int32_t *item_begin;      // [n + 1] first ticket of each operator
  const PersistPredsLds *preds;   // [n]
  const PersistOp *rec;           // [n]
  int32_t n, total;               // operators, work items
};
// Kernel ids the persistent kernel can run (256-thread bodies); others map through
// persist_kernel_id (the 8- and 16-wavefront contractions run their 4-wavefront form).
int persist_kernel_id(int kernel_id);              // -1: not available
bool kernel_is_f16(int kernel_id);
// Workgroups of the persistent kernel the device holds at once (all must be resident).
hipError_t persist_max_workgroups(bool f16, uint32_t lds_bytes, uint32_t *n_workgroups);
hipError_t add_persist_node(hipGraph_t graph, bool f16, const PersistArgs &a, uint32_t n_workgroups,
                            uint32_t lds_bytes, const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node);
// The same kernel as an ordinary launch on `s` (for timing it apart from the graph it belongs to).
hipError_t launch_persist(bool f16, const PersistArgs &a, uint32_t n_workgroups, uint32_t lds_bytes, hipStream_t s);

// ---- Chained executor: the persistent executor without a work-item loop ----------------
// One launch whose grid is the sum of all operators' grids in launch-queue order (each
// operator's block range padded to a multiple of the XCD count).  A workgroup runs exactly
// one tile: it looks up its operator, waits for the completion flags of the operator's
// predecessors, runs the tile and publishes it.  Workgroups are dispatched in increasing
// block order, predecessors have lower block numbers than their consumers, so the lowest
// unfinished block never waits for a block that has not been dispatched: the launch drains
// whatever number of workgroups the device holds at a time.
struct ChainRec {                 // one operator, read through the constant address space
  int32_t kernel, gx, gy, gz;     // body (KernelId, + kPersistActivationB for two-activation contractions) and grid
  int32_t begin, tiles;           // first block of the operator, gx * gy * gz
  uint16_t n_preds, reserved;
  uint16_t preds[kPersistMaxPreds];   // queue positions of the predecessors inside the kernel
  int32_t pad[3];
  KernelArgs args;
};
struct ChainArgs {
  PersistHeader *hdr;             // `exited` counts completed operators here
  uint32_t *done;                 // as in PersistArgs
  uint32_t *flags;
  const int32_t *block_op;        // [total] queue position of the operator a block belongs to, -1 = padding
  const ChainRec *rec;            // [n]
  int32_t n, total;
};
bool chain_kernel_ok(int kernel_id, bool *light);
hipError_t chain_max_lds(uint32_t lds_bytes);
hipError_t add_chain_node(hipGraph_t graph, bool f16, bool light, const ChainArgs &a, uint32_t lds_bytes,
                          const hipGraphNode_t *deps, size_t n_deps, hipGraphNode_t *node);
hipError_t launch_chain(bool f16, bool light, const ChainArgs &a, uint32_t lds_bytes, hipStream_t s);

// Operator timeline: device buffer of two 64-bit words per operator id, or nullptr to switch it off.
hipError_t set_op_trace(void *device_buffer);
void *current_op_trace();

hipError_t verify_reset(hipStream_t s);            // clears tokens and the violation counter
hipError_t verify_read(hipStream_t s, int *viol, int *op = nullptr, int *pred = nullptr);  // synchronises s; the counter and the last violation

// Workspace of the persistent executor for callers that cannot allocate: a static device
// array inside the library (one copy per GPU).  Returns its device address on the current
// device (looked up once per device) and its size.
constexpr int kStaticWorkspaceMaxOps = 512;
hipError_t static_workspace(void **ptr, size_t *bytes);
}  // namespace opara
