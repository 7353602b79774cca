// Internal representation behind the C ABI handles.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "../../include/opara.h"
#include "kernel_args.h"

namespace opara {
// Host copy of a persistent executor's workspace (header, counters, flags, item table,
// predecessor lists, operator records in launch-queue order) and what the launch needs.
struct PersistImage {
  std::vector<unsigned char> host;
  int32_t prefix = 0;               // leading queue operators launched as ordinary kernels
  int32_t np_ops = 0, total = 0;    // operators inside the kernel, work items
  uint32_t wgs = 0, lds_bytes = 0;  // workgroups of the launch, dynamic LDS per workgroup
  bool f16 = false;
};
}  // namespace opara

struct opara_dag {
  int32_t n = 0;
  std::vector<opara_op_desc> ops;
  std::vector<void *> ext;
  opara_limits lim{};
  // CSR adjacency over operator ids; predecessors in argument order, deduplicated.
  std::vector<int32_t> pred_off, pred, succ_off, succ;
  std::vector<int32_t> topo, tindex;
  std::vector<opara::KernelPlan> plan;          // graph executors (and the demand table)
  std::vector<opara::KernelPlan> plan_persist;  // persistent executor
  std::vector<opara::KernelPlan> plan_group;    // inside a group node of the fused executor (256-thread bodies)
  std::vector<opara_demand> dem;
  std::vector<int32_t> stream_of;   // empty until opara_assign_streams
  int32_t n_streams = 0;
  std::vector<int32_t> order;       // empty until opara_order_launch
  uint64_t order_gen = 0;           // counts the launch queues computed so far
  // Workspace image of the persistent executor as opara_run_persistent_noalloc last built it
  // (kept here so that the asynchronous upload reads memory that outlives the call).
  opara::PersistImage noalloc_image;
  uint64_t noalloc_gen = 0;         // order_gen the image belongs to, 0 = none
};

namespace opara {

struct KernelResource { const char *name; uint32_t vgprs, agprs, lds_bytes; };
extern const KernelResource kKernelResources[K_COUNT];

void set_error(const char *fmt, ...);

// One flag per entry of the opara_sync_edges list (same order): 0 = the dependency is
// implied by other ordering constraints and needs no synchronisation of its own.
int sync_keep_mask(const opara_dag *g, std::vector<uint8_t> *keep);

// Chooses the kernel, grid and arguments for operator `v`; `in[i]` are the resolved
// device pointers of its inputs.  kPlanGraph is the plan the graph executors launch and the
// demand table describes; kPlanPersistent the one the persistent executor runs (one
// workgroup size, fragment-loading contractions, its own hand-over point to the tiled
// kernel); kPlanGroup the one for operators inside a group kernel (one workgroup size,
// quad-coalesced contractions allowed).  Returns an opara_status.
enum { kPlanGraph = 0, kPlanPersistent = 1, kPlanGroup = 2 };
int plan_op(const opara_op_desc &op, const void *const *in, int kind, KernelPlan *out);

}  // namespace opara
