// Graph capturer and replay (paper Sec. 3.4): every stream handed in by the caller is
// pulled into one stream capture, operators are launched on their streams in launch-
// queue order, cross-stream dependencies become event record / wait pairs, and the
// result is instantiated as a single executable graph.
#include <hip/hip_runtime.h>
#include <new>
#include <vector>
#include "launch.h"
#include "opara_internal.h"

struct opara_exec {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  std::vector<hipEvent_t> events;
  int32_t n_nodes = 0, n_edges = 0;
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

}  // namespace

extern "C" int opara_capture(opara_dag *g, void *const *hip_streams, int32_t n_streams, int32_t mode,
                             opara_exec **out) {
  if (!g || !hip_streams || !out || n_streams < 1 || (mode != OPARA_PARALLEL && mode != OPARA_SEQUENTIAL && mode != OPARA_PARALLEL_CAPTURE)) {
    set_error("opara_capture: bad argument");
    return OPARA_EINVAL;
  }
  *out = nullptr;
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
  // Default: the graph is assembled node by node.  Each node depends on the previous
  // operator of its stream in launch-queue order and on every cross-stream predecessor;
  // one leaf node without work closes a DAG with several sinks.
  if (mode == OPARA_PARALLEL) {
    std::vector<hipGraphNode_t> node_of(n, nullptr), last_on_stream(ns, nullptr), deps;
    hipGraphNode_t leaf = nullptr;
    HIP_TRY(hipGraphCreate(&e->graph, 0));
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = q[i], sv = g->stream_of[v];
      deps.clear();
      if (last_on_stream[sv]) deps.push_back(last_on_stream[sv]);
      for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
        const int32_t u = g->pred[j];
        if (g->stream_of[u] != sv) deps.push_back(node_of[u]);
      }
      HIP_TRY(add_plan_node(e->graph, g->plan[v], deps.empty() ? nullptr : deps.data(), deps.size(), &node_of[v]));
      last_on_stream[sv] = node_of[v];
    }
    if (n_sinks > 1) {
      deps.clear();
      for (int32_t v = 0; v < n; ++v)
        if (g->succ_off[v + 1] == g->succ_off[v]) deps.push_back(node_of[v]);
      HIP_TRY(add_noop_node(e->graph, deps.data(), deps.size(), &leaf));
    }
    HIP_TRY(hipGraphInstantiate(&e->exec, e->graph, nullptr, nullptr, 0));
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
    std::vector<hipGraphNode_t> node_of(n, nullptr), last_on_stream(g->n_streams, nullptr), deps;
    HIP_TRY(hipGraphCreate(&graph, 0));
    int32_t n_sinks = 0;
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = g->order[i], sv = g->stream_of[v];
      TokenArgs t = {};
      t.epoch = 1; t.self = v; t.delay = 4;
      deps.clear();
      if (last_on_stream[sv]) deps.push_back(last_on_stream[sv]);
      for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
        const int32_t u = g->pred[j];
        if (t.n_preds < kVerifyMaxPreds) t.preds[t.n_preds++] = u;
        if (g->stream_of[u] != sv) deps.push_back(node_of[u]);
      }
      HIP_TRY(add_token_node(graph, t, deps.empty() ? nullptr : deps.data(), deps.size(), &node_of[v]));
      last_on_stream[sv] = node_of[v];
      n_sinks += (g->succ_off[v + 1] == g->succ_off[v]);
    }
    if (n_sinks > 1) {
      hipGraphNode_t leaf = nullptr;
      deps.clear();
      for (int32_t v = 0; v < n; ++v)
        if (g->succ_off[v + 1] == g->succ_off[v]) deps.push_back(node_of[v]);
      HIP_TRY(add_noop_node(graph, deps.data(), deps.size(), &leaf));
    }
    HIP_TRY(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    for (int rep = 0; rep < 2; ++rep) {
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

extern "C" int opara_replay(opara_exec *e, void *hip_stream) {
  if (!e || !e->exec) { set_error("opara_replay: null handle"); return OPARA_EINVAL; }
  hipError_t err = hipGraphLaunch(e->exec, (hipStream_t)hip_stream);
  if (err != hipSuccess) { set_error("hipGraphLaunch failed: %s", hipGetErrorString(err)); return OPARA_EHIP; }
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
