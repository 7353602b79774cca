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
  if (!g || !hip_streams || !out || n_streams < 1 || (mode != OPARA_PARALLEL && mode != OPARA_SEQUENTIAL)) {
    set_error("opara_capture: bad argument");
    return OPARA_EINVAL;
  }
  *out = nullptr;
  const int32_t n = g->n;
  if (mode == OPARA_PARALLEL) {
    if (g->stream_of.empty() || g->order.empty()) {
      set_error("opara_capture: call opara_assign_streams and opara_order_launch first");
      return OPARA_ESTATE;
    }
    if (n_streams < g->n_streams) {
      set_error("opara_capture: %d streams given, the allocation plan needs %d", n_streams, g->n_streams);
      return OPARA_EINVAL;
    }
  }
  const int32_t ns = mode == OPARA_PARALLEL ? g->n_streams : 1;
  for (int32_t s = 1; s < ns; ++s)
    for (int32_t r = 0; r < s; ++r)
      if (hip_streams[s] == hip_streams[r]) {
        set_error("opara_capture: streams %d and %d are the same handle", r, s);
        return OPARA_EINVAL;
      }
  const std::vector<int32_t> &q = mode == OPARA_PARALLEL ? g->order : g->topo;
  opara_exec *e = new (std::nothrow) opara_exec();
  if (!e) { set_error("out of memory"); return OPARA_ENOMEM; }
  hipStream_t origin = (hipStream_t)hip_streams[0];
  bool capturing = false;
  {
    // Event plan: one per producer with a consumer on another stream, one fork event,
    // one join event per non-origin stream.
    std::vector<int32_t> ev_of(n, -1);
    std::vector<uint8_t> entered(ns, 0);
    int32_t n_ev = 0;
    if (mode == OPARA_PARALLEL)
      for (int32_t v = 0; v < n; ++v)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
          const int32_t u = g->pred[j];
          if (g->stream_of[u] != g->stream_of[v] && ev_of[u] < 0) ev_of[u] = n_ev++;
        }
    const int32_t fork_ev = n_ev++;
    const int32_t join_ev0 = n_ev;
    n_ev += ns;
    e->events.reserve(n_ev);
    for (int32_t i = 0; i < n_ev; ++i) {
      hipEvent_t ev;
      HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
      e->events.push_back(ev);
    }
    HIP_TRY(hipStreamBeginCapture(origin, hipStreamCaptureModeRelaxed));
    capturing = true;
    entered[0] = 1;
    if (ns > 1) HIP_TRY(hipEventRecord(e->events[fork_ev], origin));
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = q[i];
      const int32_t sv = mode == OPARA_PARALLEL ? g->stream_of[v] : 0;
      hipStream_t st = (hipStream_t)hip_streams[sv];
      if (!entered[sv]) {   // first operator of this stream: fork it off the origin
        HIP_TRY(hipStreamWaitEvent(st, e->events[fork_ev], 0));
        entered[sv] = 1;
      }
      if (mode == OPARA_PARALLEL)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
          const int32_t u = g->pred[j];
          if (g->stream_of[u] != sv) HIP_TRY(hipStreamWaitEvent(st, e->events[ev_of[u]], 0));
        }
      HIP_TRY(launch_plan(g->plan[v], st));
      if (ev_of[v] >= 0) HIP_TRY(hipEventRecord(e->events[ev_of[v]], st));
    }
    for (int32_t s = 1; s < ns; ++s) {   // join every stream back into the origin
      if (!entered[s]) continue;
      HIP_TRY(hipEventRecord(e->events[join_ev0 + s], (hipStream_t)hip_streams[s]));
      HIP_TRY(hipStreamWaitEvent(origin, e->events[join_ev0 + s], 0));
    }
    capturing = false;
    HIP_TRY(hipStreamEndCapture(origin, &e->graph));
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
    (void)hipStreamEndCapture(origin, &partial);
    if (partial) (void)hipGraphDestroy(partial);
  }
  (void)hipGetLastError();
  destroy_exec(e);
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
