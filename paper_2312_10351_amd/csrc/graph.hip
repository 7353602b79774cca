// Graph capturer and replay (paper Sec. 3.4): one executable graph per DAG.  By default the
// graph is assembled node by node with the dependencies a multi-stream capture would record
// (previous operator of the stream in launch-queue order + every cross-stream predecessor)
// and is validated in place before it is handed out; stream capture itself, the paper's
// route, is kept for the DAG shapes it is known to serve.  Also here: the persistent
// executor's capture and the entry point for callers that cannot allocate.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <new>
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "launch.h"
#include "opara_internal.h"

struct opara_exec {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  std::vector<hipEvent_t> events;
  int32_t n_nodes = 0, n_edges = 0;
  int32_t validation = 0, attempts = 0;   // see opara_exec_validation
  // persistent executor only: caller-owned workspace and the size of its counter block
  void *workspace = nullptr;
  int32_t persist_ops = 0, persist_items = 0, persist_workgroups = 0, persist_prefix = 0;
  opara::PersistArgs persist_args{};   // the persistent kernel's launch: arguments, element type, LDS
  bool persist_f16 = false;
  uint32_t persist_lds = 0;
  // chained executor (the loop-free form of the persistent one): shares the fields above
  bool chained = false, chain_light = false;
  opara::ChainArgs chain_args{};
  // fused executor only: the chain of nodes (single operators and groups) and where each operator went
  struct FusedNode {
    bool is_group = false, f16 = false;
    int flavor = 0;                      // group kernel flavour: 0 stream, 1 light, 2 heavy
    int32_t op = -1;                     // single operator (ordinary kernel of the graph executors' plan)
    uint32_t blocks = 0, lds = 0;
    opara::GroupArgs ga;                 // group: the launch record
  };
  std::vector<FusedNode> fused;
  std::vector<int32_t> fused_node_of;
  const opara_dag *dag = nullptr;        // for launching single nodes again (timing aid); the DAG must outlive the exec
};

using namespace opara;

namespace {

void destroy_exec(opara_exec *e) {
  if (!e) return;
  if (e->exec) (void)hipGraphExecDestroy(e->exec);
  if (e->graph) (void)hipGraphDestroy(e->graph);
  for (hipEvent_t ev : e->events) (void)hipEventDestroy(ev);
  delete e;
}

#define HIP_TRY(call)                                                                   \
  do {                                                                                  \
    hipError_t err_ = (call);                                                           \
    if (err_ != hipSuccess) {                                                           \
      set_error("%s failed: %s", #call, hipGetErrorString(err_));                       \
      goto fail;                                                                        \
    }                                                                                   \
  } while (0)

constexpr int kCaptureAttempts = 4;      // instances of one graph tried before opara_capture gives up
constexpr int kValidationReplays = 2;
constexpr int64_t kFusedSplitLightBlocks = 2048;  // four times what a heavy group kernel keeps resident (2 workgroups per CU)
constexpr int kMaxGraphFanOut = 4;       // successors per node of the multi-stream graph; more go through relay nodes

// Stream capture is used for fork-join plans only: every stream other than the origin
// (the stream of the first queue entry) waits exactly once, at its first operator, on one
// event (which brings it into the capture), and is itself waited for; only the origin
// stream waits more than once.  Every DAG that captured cleanly has this shape (branch
// heads with one input each, joins on the origin stream); every capture that ended in a
// host-side crash of the runtime lacked it (streams that wait on each other again and again,
// as in chains of blocks whose heads read several branch tails, or random DAGs).
// On refusal *u -> *v is an offending dependency.
bool stream_capture_supported(const opara_dag *g, int32_t *u_out, int32_t *v_out) {
  const int32_t origin = g->stream_of[g->order[0]];
  std::vector<int32_t> first_of((size_t)g->n_streams, -1);
  for (int32_t i = 0; i < g->n; ++i) {
    const int32_t v = g->order[i];
    if (first_of[g->stream_of[v]] < 0) first_of[g->stream_of[v]] = v;
  }
  for (int32_t v = 0; v < g->n; ++v) {
    const int32_t sv = g->stream_of[v];
    const int32_t np = g->pred_off[v + 1] - g->pred_off[v];
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t u = g->pred[j], su = g->stream_of[u];
      if (su == sv || sv == origin) continue;                       // same stream, or a join on the origin
      if (first_of[sv] == v && np == 1) continue;                   // the one wait that opens stream sv
      *u_out = u; *v_out = v;
      return false;
    }
  }
  return true;
}

// Adds the nodes of the multi-stream plan to `graph` in launch-queue order: marker kernels
// (tokens) or the operators' kernels.  Markers know every predecessor of their operator,
// also those whose edge was pruned.
hipError_t assemble_parallel(const opara_dag *g, const std::vector<uint8_t> &keep_edge, bool tokens, hipGraph_t graph,
                             std::vector<hipGraphNode_t> *node_of) {
  const int32_t n = g->n;
  std::vector<hipGraphNode_t> last_on_stream((size_t)g->n_streams, nullptr), deps;
  int32_t n_sinks = 0;
  // No node gets more than kMaxGraphFanOut successors: the consumers of a producer with more
  // hang off a chain of relay nodes without work (producer -> 3 consumers + relay -> 3
  // consumers + relay ...).  Every instance of a graph in which some node had 7-15
  // successors either started a successor early or crashed the runtime on the host; graphs
  // whose nodes have at most 4 (the CNNs, BERT) never did, with or without relays.
  std::vector<int> outdeg(n, 0);
  {
    std::vector<int32_t> prev((size_t)g->n_streams, -1);
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = g->order[i], sv = g->stream_of[v];
      if (prev[sv] >= 0) ++outdeg[prev[sv]];
      prev[sv] = v;
      for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j)
        if (g->stream_of[g->pred[j]] != sv && keep_edge[j]) ++outdeg[g->pred[j]];
    }
  }
  const int fan_cap = kMaxGraphFanOut;
  std::vector<hipGraphNode_t> handle(n, nullptr);
  std::vector<int> fan(n, 0), left(outdeg);
  auto dep_on = [&](int32_t u, hipError_t *err) -> hipGraphNode_t {
    if (!handle[u]) handle[u] = (*node_of)[u];
    if (fan[u] == fan_cap - 1 && left[u] > 1) {     // the last free slot of this handle, and more than one consumer to go
      hipGraphNode_t r = nullptr;
      const hipError_t e2 = add_noop_node(graph, &handle[u], 1, &r);
      if (e2 != hipSuccess) *err = e2;
      handle[u] = r;
      fan[u] = 0;
    }
    ++fan[u];
    --left[u];
    return handle[u];
  };
  std::vector<int32_t> last_op_on_stream((size_t)g->n_streams, -1);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t v = g->order[i], sv = g->stream_of[v];
    deps.clear();
    hipError_t rerr = hipSuccess;
    if (last_on_stream[sv]) deps.push_back(dep_on(last_op_on_stream[sv], &rerr));
    last_op_on_stream[sv] = v;
    TokenNodeArgs t = {};
    t.real = g->plan[v].args;
    t.tok.epoch = 1; t.tok.self = v; t.tok.delay = 4;
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t u = g->pred[j];
      if (t.tok.n_preds < kVerifyMaxPreds) t.tok.preds[t.tok.n_preds++] = u;
      if (g->stream_of[u] != sv && keep_edge[j]) deps.push_back(dep_on(u, &rerr));
    }
    if (rerr != hipSuccess) return rerr;
    hipError_t err = tokens ? add_token_node(graph, t, deps.empty() ? nullptr : deps.data(), deps.size(), &(*node_of)[v])
                            : add_plan_node(graph, g->plan[v], deps.empty() ? nullptr : deps.data(), deps.size(), &(*node_of)[v]);
    if (err != hipSuccess) return err;
    last_on_stream[sv] = (*node_of)[v];
    n_sinks += (g->succ_off[v + 1] == g->succ_off[v]);
  }
  if (n_sinks > 1) {
    hipGraphNode_t leaf = nullptr;
    deps.clear();
    for (int32_t v = 0; v < n; ++v)
      if (g->succ_off[v + 1] == g->succ_off[v]) deps.push_back((*node_of)[v]);
    return add_noop_node(graph, deps.data(), deps.size(), &leaf);
  }
  return hipSuccess;
}

// Fused executor: the launch queue is cut into waves (every operator whose predecessors lie
// in earlier waves, in queue order); a wave of one operator is an ordinary kernel node with
// the graph executors' kernel, a wave of several becomes group nodes (one kernel whose grid
// is the sum of the members' grids); all nodes form one chain.
int capture_fused(opara_dag *g, opara_exec **out) {
  if (g->order.empty()) { set_error("opara_capture: call opara_order_launch first"); return OPARA_ESTATE; }
  const int32_t n = g->n;
  opara_exec *e = new (std::nothrow) opara_exec();
  if (!e) { set_error("out of memory"); return OPARA_ENOMEM; }
  e->dag = g;
  e->fused_node_of.assign(n, -1);
  std::vector<int32_t> indeg(n), wave;
  std::vector<char> done(n, 0);
  for (int32_t v = 0; v < n; ++v) indeg[v] = g->pred_off[v + 1] - g->pred_off[v];
  uint32_t max_lds = 0;
  int32_t placed = 0;
  while (placed < n) {
    wave.clear();
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = g->order[i];
      if (!done[v] && indeg[v] == 0) wave.push_back(v);
    }
    if (wave.empty()) { set_error("opara_capture: launch queue is not topological"); delete e; return OPARA_ESTATE; }
    for (int32_t v : wave) {
      done[v] = 1;
      ++placed;
      for (int32_t j = g->succ_off[v]; j < g->succ_off[v + 1]; ++j) --indeg[g->succ[j]];
    }
    // Operators that can share a group kernel: a 256-thread body, one element type.  The rest
    // (none with the present kernel set) and waves of one run as ordinary kernel nodes.
    std::vector<int32_t> members;
    auto flush = [&]() {
      if (members.empty()) return;
      opara_exec::FusedNode node;
      if (members.size() == 1) {
        node.op = members[0];
      } else {
        node.is_group = true;
        node.flavor = 0;
        std::memset(&node.ga, 0, sizeof node.ga);
        node.ga.n = (int32_t)members.size();
        node.ga.trace = (unsigned long long *)current_op_trace();
        for (int j = 0; j < kGroupMaxOps; ++j) node.ga.block_end[j] = INT32_MAX;
        int64_t end = 0;
        for (size_t i = 0; i < members.size(); ++i) {
          const KernelPlan &p = g->plan_group[members[i]];
          node.flavor = std::max(node.flavor, group_flavor(p.kernel));
          node.f16 = kernel_is_f16(p.kernel);
          const int64_t tiles = (int64_t)p.gx * p.gy * p.gz;
          end += (tiles + kGroupAlign - 1) / kGroupAlign * kGroupAlign;
          node.ga.meta[i].block_begin = i ? node.ga.block_end[i - 1] : 0;
          node.ga.block_end[i] = (int32_t)end;
          node.ga.meta[i].kernel = p.kernel;
          node.ga.meta[i].gx = (int32_t)p.gx; node.ga.meta[i].gy = (int32_t)p.gy;
          node.ga.meta[i].tiles = (int32_t)tiles;
          node.ga.meta[i].tag = members[i];
          node.ga.args[i] = p.args;
          node.lds = std::max(node.lds, kKernelResources[p.kernel].lds_bytes);
        }
        node.lds = std::max(node.lds, 16u);
        node.blocks = (uint32_t)end;
        max_lds = std::max(max_lds, node.lds);
      }
      for (int32_t v : members) e->fused_node_of[v] = (int32_t)e->fused.size();
      e->fused.push_back(node);
      members.clear();
    };
    int64_t blocks = 0;
    // A wave that mixes bodies of several flavours is cut between flavours, the heavier
    // members first, wherever the lighter side holds much work: inside a heavier group kernel
    // the lighter members would run at its occupancy (2 or 4 instead of 8 wavefronts per
    // SIMD), which streaming operators of several MB pay for dearly (random wide DAG: 3355 ->
    // 2740 us), while every extra node costs one more kernel boundary (Inception-v3-like:
    // 345 -> 358 us when every mixed wave is split).  The lighter side must hold more
    // workgroups than kFusedSplitLightBlocks.
    {
      std::vector<int32_t> by_flavor[3];
      bool groupable = wave.size() > 1;
      for (int32_t v : wave) {
        const KernelPlan &p = g->plan_group[v];
        const int f = group_flavor(p.kernel);
        groupable = groupable && f >= 0 && kernel_is_f16(p.kernel) == kernel_is_f16(g->plan_group[wave[0]].kernel) &&
                    (int64_t)p.gx * p.gy * p.gz < (1 << 24);
        if (f >= 0) by_flavor[f].push_back(v);
      }
      int64_t below[3] = {0, 0, 0};                    // workgroups of all members lighter than flavour f
      for (int f = 1; f < 3; ++f) {
        below[f] = below[f - 1];
        for (int32_t v : by_flavor[f - 1]) below[f] += (int64_t)g->plan_group[v].gx * g->plan_group[v].gy * g->plan_group[v].gz;
      }
      const bool cut2 = !by_flavor[2].empty() && below[2] > kFusedSplitLightBlocks;                       // heavy | rest
      const bool cut1 = !by_flavor[1].empty() && !by_flavor[0].empty() && below[1] > kFusedSplitLightBlocks &&
                        (cut2 || by_flavor[2].empty());                                                   // light | stream
      if (groupable && (cut1 || cut2)) {
        for (int f = 2; f >= 0; --f) {
          for (int32_t v : by_flavor[f]) {
            const int64_t tiles = (int64_t)g->plan_group[v].gx * g->plan_group[v].gy * g->plan_group[v].gz;
            if (members.size() == (size_t)kGroupMaxOps || blocks + tiles > (1 << 24)) { flush(); blocks = 0; }
            members.push_back(v);
            blocks += tiles + kGroupAlign;
          }
          if ((f == 2 && cut2) || (f == 1 && cut1)) { flush(); blocks = 0; }
        }
        flush();
        continue;
      }
    }
    for (int32_t v : wave) {
      const KernelPlan &p = g->plan_group[v];
      bool light = true;
      const int64_t tiles = (int64_t)p.gx * p.gy * p.gz;
      const bool fits = group_kernel_ok(p.kernel, &light) && wave.size() > 1 && tiles < (1 << 24);
      if (!fits) {                                    // on its own, before what follows it in the queue
        flush();
        members.push_back(v);
        flush();
        blocks = 0;
        continue;
      }
      if (!members.empty() && (members.size() == (size_t)kGroupMaxOps || blocks + tiles > (1 << 24) ||
                               kernel_is_f16(p.kernel) != kernel_is_f16(g->plan_group[members[0]].kernel))) {
        flush();
        blocks = 0;
      }
      members.push_back(v);
      blocks += tiles + kGroupAlign;
    }
    flush();
  }
  {
    hipGraphNode_t node = nullptr, last = nullptr;
    HIP_TRY(group_prepare(std::max(max_lds, 16u)));
    HIP_TRY(hipGraphCreate(&e->graph, 0));
    for (const opara_exec::FusedNode &fn : e->fused) {
      if (fn.is_group)
        HIP_TRY(add_group_node(e->graph, fn.f16, fn.flavor, fn.ga, fn.blocks, fn.lds, last ? &last : nullptr, last ? 1 : 0, &node));
      else
        HIP_TRY(add_plan_node(e->graph, g->plan[fn.op], last ? &last : nullptr, last ? 1 : 0, &node));
      last = node;
    }
    HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
    e->n_nodes = (int32_t)e->fused.size();
    e->n_edges = e->n_nodes - 1;
  }
  *out = e;
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  destroy_exec(e);
  return OPARA_EHIP;
}

}  // namespace

extern "C" int opara_capture(opara_dag *g, void *const *hip_streams, int32_t n_streams, int32_t mode,
                             opara_exec **out) {
  if (!g || !hip_streams || !out || n_streams < 1 || mode < OPARA_PARALLEL || mode > OPARA_FUSED) {
    set_error("opara_capture: bad argument");
    return OPARA_EINVAL;
  }
  *out = nullptr;
  if (mode == OPARA_FUSED) return capture_fused(g, out);
  const int32_t n = g->n;
  const bool parallel = mode != OPARA_SEQUENTIAL;
  if (parallel) {
    if (g->stream_of.empty() || g->order.empty()) {
      set_error("opara_capture: call opara_assign_streams and opara_order_launch first");
      return OPARA_ESTATE;
    }
    if (n_streams < g->n_streams) {
      set_error("opara_capture: %d streams given, the allocation plan needs %d", n_streams, g->n_streams);
      return OPARA_EINVAL;
    }
  }
  const int32_t ns = parallel ? g->n_streams : 1;
  for (int32_t s = 1; s < ns; ++s)
    for (int32_t r = 0; r < s; ++r)
      if (hip_streams[s] == hip_streams[r]) {
        set_error("opara_capture: streams %d and %d are the same handle", r, s);
        return OPARA_EINVAL;
      }
  const std::vector<int32_t> &q = parallel ? g->order : g->topo;
  opara_exec *e = new (std::nothrow) opara_exec();
  if (!e) { set_error("out of memory"); return OPARA_ENOMEM; }
  hipStream_t origin = (hipStream_t)hip_streams[0];
  bool capturing = false;
  int32_t n_roots = 0, n_sinks = 0;
  for (int32_t v = 0; v < n; ++v) {
    n_roots += (g->pred_off[v + 1] == g->pred_off[v]);
    n_sinks += (g->succ_off[v + 1] == g->succ_off[v]);
  }
  if (mode == OPARA_PARALLEL_CAPTURE && (n_roots > 1 || n_sinks > 1)) {
    set_error("opara_capture: stream capture serves DAGs with one root and one sink (this one has %d / %d)",
              n_roots, n_sinks);
    delete e;
    return OPARA_EUNSUPPORTED;
  }
  if (mode == OPARA_PARALLEL_CAPTURE) {
    int32_t u = -1, v = -1;
    if (!stream_capture_supported(g, &u, &v)) {
      set_error("opara_capture: stream capture serves fork-join plans only (every stream but the first waits once, at its "
                "first operator); dependency %d -> %d makes stream %d wait for stream %d otherwise", u, v,
                g->stream_of[v], g->stream_of[u]);
      delete e;
      return OPARA_EUNSUPPORTED;
    }
  }
  // Default: the graph is assembled node by node.  Each node depends on the previous
  // operator of its stream in launch-queue order and on every cross-stream predecessor;
  // one leaf node without work closes a DAG with several sinks.
  //
  // The graph runtime has been seen to start operators of irregular DAGs before a
  // predecessor had finished, depending on the instance (which one fails changes from
  // process to process).  So the graph is first instantiated with marker kernels as nodes
  // (each marks its operator done after a few microseconds and counts predecessors not yet
  // marked), that executable graph is replayed and must show no violation, and then every
  // node of the SAME executable graph is switched to its operator's kernel: the instance
  // that is handed out is the one that was checked.  A failed check is answered by a fresh
  // instance of the same graph (same streams, same launch queue), never by another plan.
  if (mode == OPARA_PARALLEL || mode == OPARA_PARALLEL_PRUNED) {
    // pruned: keep_edge[pred slot j] says whether the cross-stream dependency still needs an edge
    std::vector<uint8_t> keep_edge(g->pred.size(), 1);
    if (mode == OPARA_PARALLEL_PRUNED) {
      std::vector<uint8_t> keep;
      sync_keep_mask(g, &keep);
      size_t k = 0;
      for (int32_t v = 0; v < n; ++v)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j)
          if (g->stream_of[g->pred[j]] != g->stream_of[v]) keep_edge[j] = keep[k++];
    }
    if (n > kVerifyMaxOps) { set_error("opara_capture: more than %d operators", kVerifyMaxOps); delete e; return OPARA_EUNSUPPORTED; }
    std::vector<hipGraphNode_t> node_of(n, nullptr);
    bool swap_in_place = true;                     // false once the runtime has refused to switch a node's kernel
    int violations = 0, bad_op = -1, bad_pred = -1;
    for (int attempt = 1; attempt <= kCaptureAttempts; ++attempt) {
      e->attempts = attempt;
      if (e->exec) { (void)hipGraphExecDestroy(e->exec); e->exec = nullptr; }
      if (e->graph) { (void)hipGraphDestroy(e->graph); e->graph = nullptr; }
      HIP_TRY(hipGraphCreate(&e->graph, 0));
      HIP_TRY(assemble_parallel(g, keep_edge, /*tokens=*/true, e->graph, &node_of));
      HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
      violations = 0;
      for (int rep = 0; rep < kValidationReplays; ++rep) {
        int viol = 0, vop = -1, vpred = -1;
        HIP_TRY(verify_reset(origin));
        HIP_TRY(hipGraphLaunch(e->exec, origin));
        HIP_TRY(verify_read(origin, &viol, &vop, &vpred));
        violations += viol;
        if (viol) { bad_op = vop; bad_pred = vpred; }
      }
      if (violations != 0) continue;               // this instance drops a dependency: build another
      if (swap_in_place) {
        hipError_t err = hipSuccess;
        for (int32_t v = 0; v < n && err == hipSuccess; ++v) err = set_exec_node_plan(e->exec, node_of[v], g->plan[v]);
        if (err == hipSuccess) {
          e->validation = OPARA_VALIDATED_IN_PLACE;
          break;
        }
        (void)hipGetLastError();
        swap_in_place = false;                     // fall through: operators' graph beside the checked twin
      }
      (void)hipGraphExecDestroy(e->exec); e->exec = nullptr;
      (void)hipGraphDestroy(e->graph); e->graph = nullptr;
      HIP_TRY(hipGraphCreate(&e->graph, 0));
      HIP_TRY(assemble_parallel(g, keep_edge, /*tokens=*/false, e->graph, &node_of));
      HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
      e->validation = OPARA_SCREENED_ON_TWIN;
      break;
    }
    if (e->validation == OPARA_NOT_VALIDATED) {
      set_error("opara_capture: the graph runtime started operators before their predecessors in %d of %d instances "
                "of this graph (last one: %d violations, e.g. operator %d before its predecessor %d, which has %d "
                "successors); no graph is handed out", kCaptureAttempts, kCaptureAttempts, violations, bad_op, bad_pred,
                bad_pred >= 0 ? g->succ_off[bad_pred + 1] - g->succ_off[bad_pred] : 0);
      destroy_exec(e);
      return OPARA_EGRAPH;
    }
    size_t nn = 0, ne = 0;
    HIP_TRY(hipGraphGetNodes(e->graph, nullptr, &nn));
    HIP_TRY(hipGraphGetEdges(e->graph, nullptr, nullptr, &ne));
    e->n_nodes = (int32_t)nn;
    e->n_edges = (int32_t)ne;
    *out = e;
    return OPARA_OK;
  }
  {
    // Event plan: one per producer with a consumer on another stream, one join event
    // per non-origin stream.
    std::vector<int32_t> ev_of(n, -1);
    int32_t n_ev = 0;
    if (parallel)
      for (int32_t v = 0; v < n; ++v)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
          const int32_t u = g->pred[j];
          if (g->stream_of[u] != g->stream_of[v] && ev_of[u] < 0) ev_of[u] = n_ev++;
        }
    const int32_t join_ev0 = n_ev;
    n_ev += ns;
    e->events.reserve(n_ev);
    for (int32_t i = 0; i < n_ev; ++i) {
      hipEvent_t ev;
      HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
      e->events.push_back(ev);
    }
    // A stream enters the capture when it first waits on an event recorded inside it:
    // with a single root, the first operator of every other stream has cross-stream
    // predecessors only, so its own waits bring the stream in.
    HIP_TRY(hipStreamBeginCapture(origin, hipStreamCaptureModeRelaxed));
    capturing = true;
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = q[i];
      const int32_t sv = parallel ? g->stream_of[v] : 0;
      hipStream_t st = (hipStream_t)hip_streams[sv];
      if (parallel)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
          const int32_t u = g->pred[j];
          if (g->stream_of[u] != sv) HIP_TRY(hipStreamWaitEvent(st, e->events[ev_of[u]], 0));
        }
      HIP_TRY(launch_plan(g->plan[v], st));
      if (ev_of[v] >= 0) HIP_TRY(hipEventRecord(e->events[ev_of[v]], st));
    }
    for (int32_t s = 1; s < ns; ++s) {   // join every stream back into the origin
      HIP_TRY(hipEventRecord(e->events[join_ev0 + s], (hipStream_t)hip_streams[s]));
      HIP_TRY(hipStreamWaitEvent(origin, e->events[join_ev0 + s], 0));
    }
    capturing = false;
    {
      hipGraph_t captured = nullptr;
      HIP_TRY(hipStreamEndCapture(origin, &captured));   // on failure the runtime keeps ownership
      e->graph = captured;
    }
    HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
    size_t nn = 0, ne = 0;
    HIP_TRY(hipGraphGetNodes(e->graph, nullptr, &nn));
    HIP_TRY(hipGraphGetEdges(e->graph, nullptr, nullptr, &ne));
    e->n_nodes = (int32_t)nn;
    e->n_edges = (int32_t)ne;
  }
  *out = e;
  return OPARA_OK;
fail:
  if (capturing) {
    hipGraph_t partial = nullptr;
    if (hipStreamEndCapture(origin, &partial) == hipSuccess && partial) (void)hipGraphDestroy(partial);
  }
  (void)hipGetLastError();
  destroy_exec(e);
  return OPARA_EHIP;
}

// Builds a graph with the topology and node order opara_capture gives the parallel plan,
// but with marker kernels as nodes, replays it and counts operators that ran before one
// of their predecessors had finished.
extern "C" int opara_verify_dependencies(opara_dag *g, void *hip_stream, int32_t *n_violations) {
  if (!g || !n_violations) { set_error("opara_verify_dependencies: null pointer"); return OPARA_EINVAL; }
  if (g->stream_of.empty() || g->order.empty()) {
    set_error("opara_verify_dependencies: call opara_assign_streams and opara_order_launch first");
    return OPARA_ESTATE;
  }
  const int32_t n = g->n;
  if (n > kVerifyMaxOps) { set_error("opara_verify_dependencies: more than %d operators", kVerifyMaxOps); return OPARA_EUNSUPPORTED; }
  hipStream_t st = (hipStream_t)hip_stream;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  int total = 0;
  {
    std::vector<hipGraphNode_t> node_of(n, nullptr);
    const std::vector<uint8_t> keep_edge(g->pred.size(), 1);
    HIP_TRY(hipGraphCreate(&graph, 0));
    HIP_TRY(assemble_parallel(g, keep_edge, /*tokens=*/true, graph, &node_of));
    HIP_TRY(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    for (int rep = 0; rep < kValidationReplays; ++rep) {
      int viol = 0;
      HIP_TRY(verify_reset(st));
      HIP_TRY(hipGraphLaunch(exec, st));
      HIP_TRY(verify_read(st, &viol));
      total += viol;
    }
  }
  (void)hipGraphExecDestroy(exec);
  (void)hipGraphDestroy(graph);
  *n_violations = total;
  return OPARA_OK;
fail:
  if (exec) (void)hipGraphExecDestroy(exec);
  if (graph) (void)hipGraphDestroy(graph);
  (void)hipGetLastError();
  return OPARA_EHIP;
}

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct PersistLayout { size_t done, flags, begin, preds, rec, bytes; };

PersistLayout persist_layout(int32_t n) {
  PersistLayout l;
  l.done = align_up(sizeof(PersistHeader), 256);
  l.flags = align_up(l.done + sizeof(uint32_t) * (size_t)n * kPersistCounterStride, 256);
  l.begin = align_up(l.flags + sizeof(uint32_t) * (size_t)n * kPersistReplicas * kPersistFlagStride, 256);
  l.preds = align_up(l.begin + sizeof(int32_t) * ((size_t)n + 1), 256);
  l.rec = align_up(l.preds + sizeof(PersistPredsLds) * (size_t)n, 256);
  l.bytes = align_up(l.rec + sizeof(PersistOp) * (size_t)n, 256);
  return l;
}

// Number of leading launch-queue operators that nothing else can run beside: every other
// operator is a descendant of each of them (a network's stem).  They gain nothing from the
// persistent kernel's flags and lose its one-tile-shape restriction, so they are launched
// as ordinary kernel nodes ahead of it.  At least one operator is left for the kernel.
int32_t serial_prefix(const opara_dag *g) {
  const char *e = std::getenv("OPARA_PERSIST_SERIAL_PREFIX");
  if (e && std::atoi(e) == 0) return 0;
  const int32_t n = g->n;
  std::vector<char> seen((size_t)n);
  std::vector<int32_t> stack;
  int32_t prefix = 0;
  for (int32_t i = 0; i + 1 < n; ++i) {
    const int32_t v = g->order[i];
    std::fill(seen.begin(), seen.end(), 0);
    stack.assign(1, v);
    seen[v] = 1;
    int32_t reached = 0;
    while (!stack.empty()) {
      const int32_t u = stack.back(); stack.pop_back();
      for (int32_t j = g->succ_off[u]; j < g->succ_off[u + 1]; ++j) {
        const int32_t w = g->succ[j];
        if (!seen[w]) { seen[w] = 1; ++reached; stack.push_back(w); }
      }
    }
    // The earlier prefix operators are ancestors of v by the same test; the rest must be below it.
    if (reached != n - 1 - i) break;
    prefix = i + 1;
  }
  return prefix;
}

}  // namespace

extern "C" int opara_persistent_workspace_bytes(const opara_dag *g, uint64_t *bytes) {
  if (!g || !bytes) { set_error("opara_persistent_workspace_bytes: null pointer"); return OPARA_EINVAL; }
  *bytes = persist_layout(g->n).bytes;
  return OPARA_OK;
}

namespace {

// Builds the workspace image of the persistent executor for the current launch queue:
// records in launch-queue order, work items, predecessor lists.  Asks the runtime how many
// workgroups of the kernel the device holds at once (no allocation).  Returns an opara_status.
int build_persist_image(const opara_dag *g, int32_t n_workgroups, const char *who, PersistImage *img) {
  const int32_t n = g->n;
  const PersistLayout lay = persist_layout(n);
  const int32_t prefix = serial_prefix(g);                      // run as ordinary kernel nodes
  const int32_t np_ops = n - prefix;                            // operators inside the persistent kernel
  const uint32_t lds_bytes = persist_lds_bytes((uint32_t)np_ops);
  if (lds_bytes > kPersistMaxLds || n > 65535) {
    set_error("%s: %d operators exceed the ticket table held in workgroup memory", who, n);
    return OPARA_EUNSUPPORTED;
  }
  // Workgroups the device holds at once: the launch size, and the tiles per work item of
  // operators that have more tiles than that.
  const bool f16 = kernel_is_f16(persist_kernel_id(g->plan_persist[g->order[prefix]].kernel));
  uint32_t wgs = 0;
  {
    hipError_t err = persist_max_workgroups(f16, lds_bytes, &wgs);
    if (err != hipSuccess) {
      set_error("%s: occupancy query failed: %s", who, hipGetErrorString(err));
      (void)hipGetLastError();
      return OPARA_EHIP;
    }
  }
  if (wgs == 0) { set_error("%s: the kernel does not fit a compute unit", who); return OPARA_EHIP; }
  if (n_workgroups > 0 && (uint32_t)n_workgroups < wgs) wgs = (uint32_t)n_workgroups;
  // Records in launch-queue order.
  std::vector<unsigned char> &host = img->host;
  host.assign(lay.bytes, 0);
  PersistHeader *hdr = (PersistHeader *)host.data();
  hdr->spin_limit = kPersistDefaultSpinLimit;
  hdr->epoch = 1;
  int32_t *begin = (int32_t *)(host.data() + lay.begin);
  PersistPredsLds *preds = (PersistPredsLds *)(host.data() + lay.preds);
  PersistOp *rec = (PersistOp *)(host.data() + lay.rec);
  std::vector<int32_t> pos_of(n, -1);
  int64_t total = 0;
  std::vector<char> in_prefix((size_t)n, 0);                    // complete before the kernel starts
  for (int32_t q = 0; q < prefix; ++q) in_prefix[g->order[q]] = 1;
  for (int32_t i = 0; i < np_ops; ++i) {
    const int32_t v = g->order[prefix + i];
    const KernelPlan &p = g->plan_persist[v];
    const int kid = persist_kernel_id(p.kernel);
    if (kid < 0) { set_error("%s: operator %d has no persistent kernel", who, v); return OPARA_EUNSUPPORTED; }
    if (kernel_is_f16(kid) != f16) { set_error("%s: mixed element types", who); return OPARA_EUNSUPPORTED; }
    pos_of[v] = i;
    const int64_t t = (int64_t)p.gx * p.gy * p.gz;
    if (t < 1 || t > 65535 || total + t > INT32_MAX) { set_error("%s: work-item count out of range", who); return OPARA_EUNSUPPORTED; }
    begin[i] = (int32_t)total;
    const int64_t chunk = (t + wgs - 1) / wgs;                  // 1 unless the operator has more tiles than workgroups
    const int64_t items = (t + chunk - 1) / chunk;
    total += (items + kPersistItemAlign - 1) / kPersistItemAlign * kPersistItemAlign;
    rec[i].kernel = kid + (g->ops[v].op_type == OPARA_BGEMM ? kPersistActivationB : 0);
    rec[i].gx = (int32_t)p.gx; rec[i].gy = (int32_t)p.gy; rec[i].gz = (int32_t)p.gz;
    rec[i].args = p.args;
    const int32_t np = g->pred_off[v + 1] - g->pred_off[v];
    if (np > kPersistMaxPreds) { set_error("%s: operator %d has %d predecessors (limit %d)", who, v, np, kPersistMaxPreds); return OPARA_EUNSUPPORTED; }
    int32_t kept = 0;
    for (int32_t j = 0; j < np; ++j) {
      const int32_t pu = g->pred[g->pred_off[v] + j];
      const int32_t u = pos_of[pu];
      if (u >= 0) { preds[i].pos[kept++] = (uint16_t)u; continue; }
      if (!in_prefix[pu]) { set_error("%s: launch queue is not topological", who); return OPARA_ESTATE; }
    }
    preds[i].n = (uint16_t)kept;
    preds[i].tiles = (uint16_t)t;
    preds[i].chunk = (uint16_t)chunk;
  }
  begin[np_ops] = (int32_t)total;
  if ((int64_t)wgs > total) wgs = (uint32_t)total;
  if (wgs > (uint32_t)kPersistItemAlign) wgs -= wgs % kPersistItemAlign;
  img->prefix = prefix;
  img->np_ops = np_ops;
  img->total = (int32_t)total;
  img->wgs = wgs;
  img->lds_bytes = lds_bytes;
  img->f16 = f16;
  return OPARA_OK;
}

// Kernel arguments of an image that lives at device address `workspace`.
PersistArgs persist_args_at(const PersistImage &img, int32_t n_ops, void *workspace) {
  const PersistLayout lay = persist_layout(n_ops);
  PersistArgs pa;
  unsigned char *ws = (unsigned char *)workspace;
  pa.hdr = (PersistHeader *)ws;
  pa.done = (uint32_t *)(ws + lay.done);
  pa.flags = (uint32_t *)(ws + lay.flags);
  pa.item_begin = (const int32_t *)(ws + lay.begin);
  pa.preds = (const PersistPredsLds *)(ws + lay.preds);
  pa.rec = (const PersistOp *)(ws + lay.rec);
  pa.n = img.np_ops;
  pa.total = img.total;
  return pa;
}

}  // namespace

extern "C" int opara_capture_persistent(opara_dag *g, void *workspace, uint64_t workspace_bytes,
                                        int32_t n_workgroups, opara_exec **out) {
  if (!g || !workspace || !out || n_workgroups < 0) { set_error("opara_capture_persistent: bad argument"); return OPARA_EINVAL; }
  *out = nullptr;
  if (g->order.empty()) { set_error("opara_capture_persistent: call opara_order_launch first"); return OPARA_ESTATE; }
  const int32_t n = g->n;
  const PersistLayout lay = persist_layout(n);
  if (workspace_bytes < lay.bytes || ((uintptr_t)workspace & 255u)) {
    set_error("opara_capture_persistent: workspace of %llu bytes (need %llu, 256-byte aligned)",
              (unsigned long long)workspace_bytes, (unsigned long long)lay.bytes);
    return OPARA_EINVAL;
  }
  PersistImage img;
  {
    const int rc = build_persist_image(g, n_workgroups, "opara_capture_persistent", &img);
    if (rc != OPARA_OK) return rc;
  }
  opara_exec *e = new (std::nothrow) opara_exec();
  if (!e) { set_error("out of memory"); return OPARA_ENOMEM; }
  {
    HIP_TRY(hipMemcpy(workspace, img.host.data(), lay.bytes, hipMemcpyHostToDevice));
    const PersistArgs pa = persist_args_at(img, n, workspace);
    hipGraphNode_t node = nullptr, last = nullptr;
    HIP_TRY(hipGraphCreate(&e->graph, 0));
    for (int32_t q = 0; q < img.prefix; ++q) {                  // the serial prefix: a chain of ordinary launches
      HIP_TRY(add_plan_node(e->graph, g->plan[g->order[q]], last ? &last : nullptr, last ? 1 : 0, &node));
      last = node;
    }
    HIP_TRY(add_persist_node(e->graph, img.f16, pa, img.wgs, img.lds_bytes, last ? &last : nullptr, last ? 1 : 0, &node));
    HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
    e->n_nodes = img.prefix + 1;
    e->n_edges = img.prefix;
    e->workspace = workspace;
    e->persist_prefix = img.prefix;
    e->persist_args = pa;
    e->persist_f16 = img.f16;
    e->persist_lds = img.lds_bytes;
    e->persist_ops = n;
    e->persist_items = img.total;
    e->persist_workgroups = (int32_t)img.wgs;
  }
  *out = e;
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  destroy_exec(e);
  return OPARA_EHIP;
}

// One pass over the DAG through the persistent executor without a graph and without any
// allocation: the workspace is the library's static device array, the image is uploaded on
// the caller's stream, the serial prefix and the persistent kernel are ordinary launches.
extern "C" int opara_run_persistent_noalloc(opara_dag *g, void *hip_stream, uint32_t *error_word) {
  if (!g) { set_error("opara_run_persistent_noalloc: null handle"); return OPARA_EINVAL; }
  if (g->order.empty()) { set_error("opara_run_persistent_noalloc: call opara_order_launch first"); return OPARA_ESTATE; }
  const int32_t n = g->n;
  const PersistLayout lay = persist_layout(n);
  hipStream_t st = (hipStream_t)hip_stream;
  void *ws = nullptr;
  size_t ws_bytes = 0;
  HIP_TRY(static_workspace(&ws, &ws_bytes));
  if (n > kStaticWorkspaceMaxOps || lay.bytes > ws_bytes) {
    set_error("opara_run_persistent_noalloc: %d operators need %llu bytes of workspace; the static workspace serves up to "
              "%d operators (%llu bytes)", n, (unsigned long long)lay.bytes, kStaticWorkspaceMaxOps,
              (unsigned long long)ws_bytes);
    return OPARA_EUNSUPPORTED;
  }
  if (g->noalloc_gen != g->order_gen) {
    // A new launch queue: an earlier upload may still be reading the old image.
    HIP_TRY(hipStreamSynchronize(st));
    g->noalloc_gen = 0;
    const int rc = build_persist_image(g, 0, "opara_run_persistent_noalloc", &g->noalloc_image);
    if (rc != OPARA_OK) return rc;
    g->noalloc_gen = g->order_gen;
  }
  {
    const PersistImage &img = g->noalloc_image;
    // The whole image every time: counters, flags, launch number and error word start clean
    // whatever the previous call (of this or another DAG) left in the array.
    HIP_TRY(hipMemcpyAsync(ws, img.host.data(), lay.bytes, hipMemcpyHostToDevice, st));
    for (int32_t q = 0; q < img.prefix; ++q) HIP_TRY(launch_plan(g->plan[g->order[q]], st));
    HIP_TRY(launch_persist(img.f16, persist_args_at(img, n, ws), img.wgs, img.lds_bytes, st));
    if (error_word) {
      PersistHeader h;
      HIP_TRY(hipMemcpyAsync(&h, ws, sizeof(h), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      *error_word = h.error;
    }
  }
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  return OPARA_EHIP;
}

namespace {

struct ChainLayout { size_t block_op, rec, bytes; };

// Header, counters and flags sit where the persistent executor has them (persist_layout),
// so status, reset and tracing serve both; then the block table and the operator records.
ChainLayout chain_layout(int32_t n, int64_t total_blocks) {
  ChainLayout l;
  l.block_op = persist_layout(n).begin;
  l.rec = align_up(l.block_op + sizeof(int32_t) * (size_t)total_blocks, 256);
  l.bytes = align_up(l.rec + sizeof(ChainRec) * (size_t)n, 256);
  return l;
}

int64_t chain_blocks_of(const KernelPlan &p) {
  const int64_t t = (int64_t)p.gx * p.gy * p.gz;
  return (t + kGroupAlign - 1) / kGroupAlign * kGroupAlign;
}

}  // namespace

extern "C" int opara_chained_workspace_bytes(const opara_dag *g, uint64_t *bytes) {
  if (!g || !bytes) { set_error("opara_chained_workspace_bytes: null pointer"); return OPARA_EINVAL; }
  int64_t total = 0;
  for (int32_t v = 0; v < g->n; ++v) total += chain_blocks_of(g->plan_group[v]);
  *bytes = chain_layout(g->n, total).bytes;
  return OPARA_OK;
}

extern "C" int opara_capture_chained(opara_dag *g, void *workspace, uint64_t workspace_bytes, opara_exec **out) {
  if (!g || !workspace || !out) { set_error("opara_capture_chained: bad argument"); return OPARA_EINVAL; }
  *out = nullptr;
  if (g->order.empty()) { set_error("opara_capture_chained: call opara_order_launch first"); return OPARA_ESTATE; }
  const int32_t n = g->n;
  const int32_t prefix = serial_prefix(g);
  const int32_t np_ops = n - prefix;
  if (n > 65535) { set_error("opara_capture_chained: more than 65535 operators"); return OPARA_EUNSUPPORTED; }
  int64_t total = 0;
  for (int32_t i = 0; i < np_ops; ++i) total += chain_blocks_of(g->plan_group[g->order[prefix + i]]);
  if (total > (int64_t)1 << 30) { set_error("opara_capture_chained: %lld workgroups in one launch", (long long)total); return OPARA_EUNSUPPORTED; }
  const ChainLayout lay = chain_layout(n, total);
  const PersistLayout play = persist_layout(n);
  if (workspace_bytes < lay.bytes || ((uintptr_t)workspace & 255u)) {
    set_error("opara_capture_chained: workspace of %llu bytes (need %llu, 256-byte aligned)",
              (unsigned long long)workspace_bytes, (unsigned long long)lay.bytes);
    return OPARA_EINVAL;
  }
  std::vector<unsigned char> host(lay.bytes, 0);
  PersistHeader *hdr = (PersistHeader *)host.data();
  hdr->spin_limit = kPersistDefaultSpinLimit;
  hdr->epoch = 1;
  int32_t *block_op = (int32_t *)(host.data() + lay.block_op);
  ChainRec *rec = (ChainRec *)(host.data() + lay.rec);
  std::vector<int32_t> pos_of(n, -1);
  std::vector<char> in_prefix((size_t)n, 0);
  for (int32_t q = 0; q < prefix; ++q) in_prefix[g->order[q]] = 1;
  bool all_light = true, f16 = false;
  uint32_t lds = 16;
  int64_t at = 0;
  for (int32_t i = 0; i < np_ops; ++i) {
    const int32_t v = g->order[prefix + i];
    const KernelPlan &p = g->plan_group[v];
    bool light = true;
    if (!chain_kernel_ok(p.kernel, &light)) { set_error("opara_capture_chained: operator %d has no 256-thread kernel", v); return OPARA_EUNSUPPORTED; }
    if (i == 0) f16 = kernel_is_f16(p.kernel);
    if (kernel_is_f16(p.kernel) != f16) { set_error("opara_capture_chained: mixed element types"); return OPARA_EUNSUPPORTED; }
    all_light = all_light && light;
    lds = std::max(lds, kKernelResources[p.kernel].lds_bytes);
    pos_of[v] = i;
    const int64_t tiles = (int64_t)p.gx * p.gy * p.gz, blocks = chain_blocks_of(p);
    ChainRec &r = rec[i];
    r.kernel = p.kernel + (g->ops[v].op_type == OPARA_BGEMM ? kPersistActivationB : 0);
    r.gx = (int32_t)p.gx; r.gy = (int32_t)p.gy; r.gz = (int32_t)p.gz;
    r.begin = (int32_t)at;
    r.tiles = (int32_t)tiles;
    r.args = p.args;
    for (int64_t b = 0; b < blocks; ++b) block_op[at + b] = b < tiles ? i : -1;
    at += blocks;
    const int32_t np = g->pred_off[v + 1] - g->pred_off[v];
    if (np > kPersistMaxPreds) { set_error("opara_capture_chained: operator %d has %d predecessors (limit %d)", v, np, kPersistMaxPreds); return OPARA_EUNSUPPORTED; }
    int32_t kept = 0;
    for (int32_t j = 0; j < np; ++j) {
      const int32_t pu = g->pred[g->pred_off[v] + j];
      if (pos_of[pu] >= 0) { r.preds[kept++] = (uint16_t)pos_of[pu]; continue; }
      if (!in_prefix[pu]) { set_error("opara_capture_chained: launch queue is not topological"); return OPARA_ESTATE; }
    }
    r.n_preds = (uint16_t)kept;
  }
  opara_exec *e = new (std::nothrow) opara_exec();
  if (!e) { set_error("out of memory"); return OPARA_ENOMEM; }
  {
    HIP_TRY(chain_max_lds(lds));
    HIP_TRY(hipMemcpy(workspace, host.data(), lay.bytes, hipMemcpyHostToDevice));
    unsigned char *ws = (unsigned char *)workspace;
    ChainArgs ca;
    ca.hdr = (PersistHeader *)ws;
    ca.done = (uint32_t *)(ws + play.done);
    ca.flags = (uint32_t *)(ws + play.flags);
    ca.block_op = (const int32_t *)(ws + lay.block_op);
    ca.rec = (const ChainRec *)(ws + lay.rec);
    ca.n = np_ops;
    ca.total = (int32_t)total;
    hipGraphNode_t node = nullptr, last = nullptr;
    HIP_TRY(hipGraphCreate(&e->graph, 0));
    for (int32_t q = 0; q < prefix; ++q) {
      HIP_TRY(add_plan_node(e->graph, g->plan[g->order[q]], last ? &last : nullptr, last ? 1 : 0, &node));
      last = node;
    }
    HIP_TRY(add_chain_node(e->graph, f16, all_light, ca, lds, last ? &last : nullptr, last ? 1 : 0, &node));
    HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
    e->n_nodes = prefix + 1;
    e->n_edges = prefix;
    e->workspace = workspace;
    e->persist_prefix = prefix;
    e->persist_f16 = f16;
    e->persist_lds = lds;
    e->persist_ops = n;
    e->persist_items = (int32_t)total;
    e->persist_workgroups = (int32_t)total;
    e->chained = true;
    e->chain_light = all_light;
    e->chain_args = ca;
  }
  *out = e;
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  destroy_exec(e);
  return OPARA_EHIP;
}

extern "C" int opara_persistent_status(opara_exec *e, void *hip_stream, uint32_t *error_word) {
  if (!e || !e->workspace || !error_word) { set_error("opara_persistent_status: not a persistent executor"); return OPARA_EINVAL; }
  hipStream_t st = (hipStream_t)hip_stream;
  PersistHeader h;
  HIP_TRY(hipMemcpyAsync(&h, e->workspace, sizeof(h), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  *error_word = h.error;
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  return OPARA_EHIP;
}

extern "C" int opara_persistent_info(const opara_exec *e, int32_t *n_items, int32_t *n_workgroups) {
  if (!e || !e->workspace) { set_error("opara_persistent_info: not a persistent executor"); return OPARA_EINVAL; }
  if (n_items) *n_items = e->persist_items;
  if (n_workgroups) *n_workgroups = e->persist_workgroups;
  return OPARA_OK;
}

extern "C" int opara_persistent_prefix(const opara_exec *e, int32_t *n_prefix) {
  if (!e || !e->workspace || !n_prefix) { set_error("opara_persistent_prefix: not a persistent executor"); return OPARA_EINVAL; }
  *n_prefix = e->persist_prefix;
  return OPARA_OK;
}

extern "C" int opara_persistent_time_kernel(opara_exec *e, void *hip_stream, int32_t launches, float *avg_us) {
  if (!e || !e->workspace || !avg_us || launches < 1) { set_error("opara_persistent_time_kernel: bad argument"); return OPARA_EINVAL; }
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t t0 = nullptr, t1 = nullptr;
  float ms = 0.f;
  HIP_TRY(hipEventCreate(&t0));
  HIP_TRY(hipEventCreate(&t1));
  HIP_TRY(hipStreamSynchronize(st));
  HIP_TRY(hipEventRecord(t0, st));
  for (int32_t i = 0; i < launches; ++i) {
    if (e->chained) HIP_TRY(launch_chain(e->persist_f16, e->chain_light, e->chain_args, e->persist_lds, st));
    else HIP_TRY(launch_persist(e->persist_f16, e->persist_args, (uint32_t)e->persist_workgroups, e->persist_lds, st));
  }
  HIP_TRY(hipEventRecord(t1, st));
  HIP_TRY(hipEventSynchronize(t1));
  HIP_TRY(hipEventElapsedTime(&ms, t0, t1));
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  *avg_us = ms * 1e3f / (float)launches;
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  return OPARA_EHIP;
}

extern "C" int opara_persistent_set_trace(opara_exec *e, void *hip_stream, void *trace, uint64_t trace_bytes) {
  if (!e || !e->workspace) { set_error("opara_persistent_set_trace: not a persistent executor"); return OPARA_EINVAL; }
  if (trace && (trace_bytes < 32ull * (uint64_t)e->persist_items || ((uintptr_t)trace & 7u))) {
    set_error("opara_persistent_set_trace: buffer of %llu bytes, need %llu (8-byte aligned)",
              (unsigned long long)trace_bytes, 32ull * (unsigned long long)e->persist_items);
    return OPARA_EINVAL;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const uint64_t addr = (uint64_t)(uintptr_t)trace;
  HIP_TRY(hipStreamSynchronize(st));
  HIP_TRY(hipMemcpyAsync((unsigned char *)e->workspace + offsetof(PersistHeader, trace), &addr, sizeof(addr),
                         hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  return OPARA_EHIP;
}

extern "C" int opara_persistent_reset(opara_exec *e, void *hip_stream, uint32_t spin_limit) {
  if (!e || !e->workspace) { set_error("opara_persistent_reset: not a persistent executor"); return OPARA_EINVAL; }
  hipStream_t st = (hipStream_t)hip_stream;
  const PersistLayout lay = persist_layout(e->persist_ops);
  PersistHeader h = {};
  HIP_TRY(hipStreamSynchronize(st));
  HIP_TRY(hipMemcpyAsync(&h, e->workspace, sizeof(h), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  h.exited = 0;
  h.error = 0;
  h.epoch = 1;
  h.spin_limit = spin_limit ? spin_limit : kPersistDefaultSpinLimit;
  HIP_TRY(hipMemcpyAsync(e->workspace, &h, sizeof(h), hipMemcpyHostToDevice, st));
  HIP_TRY(hipMemsetAsync((unsigned char *)e->workspace + lay.done, 0, lay.begin - lay.done, st));   // counters and flags
  HIP_TRY(hipStreamSynchronize(st));
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  return OPARA_EHIP;
}

extern "C" int opara_replay(opara_exec *e, void *hip_stream) {
  if (!e || !e->exec) { set_error("opara_replay: null handle"); return OPARA_EINVAL; }
  hipError_t err = hipGraphLaunch(e->exec, (hipStream_t)hip_stream);
  if (err != hipSuccess) { set_error("hipGraphLaunch failed: %s", hipGetErrorString(err)); return OPARA_EHIP; }
  return OPARA_OK;
}

extern "C" int opara_fused_plan(const opara_exec *e, int32_t *node_of, int32_t *n_nodes, int32_t *node_kernel) {
  if (!e || e->fused.empty()) { set_error("opara_fused_plan: not a fused executor"); return OPARA_EINVAL; }
  if (node_of) std::memcpy(node_of, e->fused_node_of.data(), sizeof(int32_t) * e->fused_node_of.size());
  if (n_nodes) *n_nodes = (int32_t)e->fused.size();
  if (node_kernel)
    for (size_t i = 0; i < e->fused.size(); ++i) {
      const opara_exec::FusedNode &fn = e->fused[i];
      node_kernel[i] = fn.is_group ? (fn.flavor == 0 ? OPARA_GROUP_KERNEL_STREAM : fn.flavor == 1 ? OPARA_GROUP_KERNEL_LIGHT : OPARA_GROUP_KERNEL_HEAVY) : e->dag->plan[fn.op].kernel;
    }
  return OPARA_OK;
}

extern "C" int opara_fused_time_nodes(opara_exec *e, void *hip_stream, int32_t launches, float *us) {
  if (!e || e->fused.empty() || !us || launches < 1) { set_error("opara_fused_time_nodes: bad argument"); return OPARA_EINVAL; }
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t t0 = nullptr, t1 = nullptr;
  HIP_TRY(hipEventCreate(&t0));
  HIP_TRY(hipEventCreate(&t1));
  for (size_t i = 0; i < e->fused.size(); ++i) {
    const opara_exec::FusedNode &fn = e->fused[i];
    float ms = 0.f;
    for (int32_t k = -2; k < launches; ++k) {       // two untimed launches first
      if (k == 0) HIP_TRY(hipEventRecord(t0, st));
      if (fn.is_group) HIP_TRY(launch_group(fn.f16, fn.flavor, fn.ga, fn.blocks, fn.lds, st));
      else HIP_TRY(launch_plan(e->dag->plan[fn.op], st));
    }
    HIP_TRY(hipEventRecord(t1, st));
    HIP_TRY(hipEventSynchronize(t1));
    HIP_TRY(hipEventElapsedTime(&ms, t0, t1));
    us[i] = ms * 1e3f / (float)launches;
  }
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  return OPARA_OK;
fail:
  (void)hipGetLastError();
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  return OPARA_EHIP;
}

extern "C" int opara_set_operator_trace(void *device_buffer) {
  hipError_t err = set_op_trace(device_buffer);
  if (err != hipSuccess) { set_error("opara_set_operator_trace: %s", hipGetErrorString(err)); (void)hipGetLastError(); return OPARA_EHIP; }
  return OPARA_OK;
}

extern "C" int opara_exec_validation(const opara_exec *e, int32_t *kind, int32_t *attempts) {
  if (!e) { set_error("opara_exec_validation: null handle"); return OPARA_EINVAL; }
  if (kind) *kind = e->validation;
  if (attempts) *attempts = e->attempts;
  return OPARA_OK;
}

extern "C" int opara_exec_info(const opara_exec *e, int32_t *n_nodes, int32_t *n_edges) {
  if (!e) { set_error("opara_exec_info: null handle"); return OPARA_EINVAL; }
  if (n_nodes) *n_nodes = e->n_nodes;
  if (n_edges) *n_edges = e->n_edges;
  return OPARA_OK;
}

extern "C" void opara_exec_destroy(opara_exec *e) { destroy_exec(e); }

extern "C" int opara_launch_op(opara_dag *g, int32_t op, void *hip_stream) {
  if (!g || op < 0 || op >= g->n) { set_error("opara_launch_op: bad argument"); return OPARA_EINVAL; }
  hipError_t err = launch_plan(g->plan[op], (hipStream_t)hip_stream);
  if (err != hipSuccess) { set_error("kernel launch failed: %s", hipGetErrorString(err)); return OPARA_EHIP; }
  return OPARA_OK;
}

extern "C" int opara_run_eager(opara_dag *g, void *hip_stream) {
  if (!g) { set_error("opara_run_eager: null handle"); return OPARA_EINVAL; }
  for (int32_t i = 0; i < g->n; ++i) {
    hipError_t err = launch_plan(g->plan[g->topo[i]], (hipStream_t)hip_stream);
    if (err != hipSuccess) { set_error("kernel launch failed: %s", hipGetErrorString(err)); return OPARA_EHIP; }
  }
  return OPARA_OK;
}

extern "C" int opara_kernel_device_attrs(int32_t id, uint32_t *vgprs, uint32_t *lds_bytes) {
  const void *sym = kernel_symbol(id);
  if (!sym) { set_error("opara_kernel_device_attrs: id %d out of range", id); return OPARA_EINVAL; }
  hipFuncAttributes attr;
  hipError_t err = hipFuncGetAttributes(&attr, sym);
  if (err != hipSuccess) { set_error("hipFuncGetAttributes failed: %s", hipGetErrorString(err)); return OPARA_EHIP; }
  if (vgprs) *vgprs = (uint32_t)attr.numRegs;
  if (lds_bytes) *lds_bytes = (uint32_t)attr.sharedSizeBytes;
  return OPARA_OK;
}
