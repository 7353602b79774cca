// Host-side scheduler core: DAG construction, stream allocation (paper Alg. 1),
// launch ordering (paper Alg. 2) and synchronisation-edge placement.  No HIP calls.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <queue>
#include "opara_internal.h"

namespace opara {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

static const opara_limits kMi355x = {256u, 2048u, 163840u, 4u * 512u * 64u};

static uint64_t ceil_div_u64(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Workgroup's share of one compute unit, in units of 2^-16, times the number of
// workgroups: "amount of GPU resources" an operator asks for (paper Sec. 3.2/3.3:
// threads, shared memory and registers of a block; Sec. 2.3: number of blocks).
static uint64_t demand_scalar(const opara_demand &d, const opara_limits &lim) {
  const uint64_t t = d.block_threads;
  uint64_t share = ceil_div_u64(65536ull * t, lim.threads_per_cu);
  share = std::max(share, ceil_div_u64(65536ull * d.lds_bytes, lim.lds_bytes_per_cu));
  share = std::max(share, ceil_div_u64(65536ull * t * d.vgprs, lim.vgpr_lanes_per_cu));
  return (uint64_t)d.grid_blocks * share;
}

static int default_class(int32_t op_type) {
  return (op_type == OPARA_CONV2D || op_type == OPARA_GEMM || op_type == OPARA_BGEMM)
             ? OPARA_COMP : OPARA_MEM;
}

}  // namespace opara

using namespace opara;

extern "C" const char *opara_last_error(void) { return g_err; }

extern "C" int opara_build_dag(const opara_op_desc *ops, int32_t n_ops, void *const *ext_inputs,
                               int32_t n_ext, const opara_limits *lim, opara_dag **out) {
  if (!ops || !out || n_ops <= 0 || n_ext < 0 || (n_ext > 0 && !ext_inputs)) {
    set_error("opara_build_dag: null pointer or non-positive operator count");
    return OPARA_EINVAL;
  }
  *out = nullptr;
  opara_dag *g = new (std::nothrow) opara_dag();
  if (!g) { set_error("out of memory"); return OPARA_ENOMEM; }
  int rc = OPARA_OK;
  try {
    g->n = n_ops;
    g->ops.assign(ops, ops + n_ops);
    g->ext.assign(ext_inputs, ext_inputs + n_ext);
    g->lim = lim ? *lim : kMi355x;
    if (!g->lim.threads_per_cu || !g->lim.lds_bytes_per_cu || !g->lim.vgpr_lanes_per_cu) {
      set_error("opara_build_dag: zero in opara_limits");
      delete g;
      return OPARA_EINVAL;
    }
    // ---- validate ids, build deduplicated predecessor lists in argument order
    g->pred_off.assign(n_ops + 1, 0);
    for (int v = 0; v < n_ops && rc == OPARA_OK; ++v) {
      const opara_op_desc &op = g->ops[v];
      if (op.op_type < 0 || op.op_type >= OPARA_N_OP_TYPES) {
        set_error("operator %d: unknown op_type %d", v, op.op_type); rc = OPARA_EINVAL; break;
      }
      if (op.dtype != OPARA_F32 && op.dtype != OPARA_F16) {
        set_error("operator %d: unknown dtype %d", v, op.dtype); rc = OPARA_EINVAL; break;
      }
      if (op.op_class != OPARA_CLASS_DEFAULT && op.op_class != OPARA_MEM && op.op_class != OPARA_COMP) {
        set_error("operator %d: unknown op_class %d", v, op.op_class); rc = OPARA_EINVAL; break;
      }
      if (op.n_inputs < 1 || op.n_inputs > OPARA_MAX_INPUTS) {
        set_error("operator %d: n_inputs %d outside 1..%d", v, op.n_inputs, OPARA_MAX_INPUTS);
        rc = OPARA_EINVAL; break;
      }
      if (!op.out) { set_error("operator %d: null output pointer", v); rc = OPARA_EINVAL; break; }
      if (op.n_deps < 0 || op.n_deps > OPARA_MAX_INPUTS) {
        set_error("operator %d: n_deps %d outside 0..%d", v, op.n_deps, OPARA_MAX_INPUTS);
        rc = OPARA_EINVAL; break;
      }
      for (int i = 0; i < op.n_inputs + op.n_deps; ++i) {
        const bool is_dep = i >= op.n_inputs;
        const int32_t u = is_dep ? op.deps[i - op.n_inputs] : op.inputs[i];
        if (u == v) { set_error("operator %d reads its own output", v); rc = OPARA_ECYCLE; break; }
        if (u >= n_ops || (u < 0 && (is_dep || -(int64_t)u - 1 >= n_ext))) {
          set_error("operator %d: %s %d refers to %d, out of range", v, is_dep ? "dependency" : "input",
                    is_dep ? i - op.n_inputs : i, u);
          rc = OPARA_EINVAL; break;
        }
        if (u < 0) continue;
        bool dup = false;
        for (int32_t j = g->pred_off[v]; j < (int32_t)g->pred.size(); ++j) dup |= (g->pred[j] == u);
        if (!dup) g->pred.push_back(u);
      }
      if (rc != OPARA_OK) break;
      g->pred_off[v + 1] = (int32_t)g->pred.size();
    }
    if (rc != OPARA_OK) { delete g; return rc; }
    // ---- successors (CSR), in increasing consumer id
    std::vector<int32_t> outdeg(n_ops, 0), indeg(n_ops, 0);
    for (int v = 0; v < n_ops; ++v)
      for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) { ++outdeg[g->pred[j]]; ++indeg[v]; }
    g->succ_off.assign(n_ops + 1, 0);
    for (int v = 0; v < n_ops; ++v) g->succ_off[v + 1] = g->succ_off[v] + outdeg[v];
    g->succ.assign(g->pred.size(), 0);
    {
      std::vector<int32_t> fill(g->succ_off.begin(), g->succ_off.end() - 1);
      for (int v = 0; v < n_ops; ++v)
        for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) g->succ[fill[g->pred[j]]++] = v;
    }
    // ---- topological order: ready operator with the smallest id first
    {
      std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> ready;
      for (int v = 0; v < n_ops; ++v) if (indeg[v] == 0) ready.push(v);
      g->topo.reserve(n_ops);
      while (!ready.empty()) {
        const int32_t v = ready.top(); ready.pop();
        g->topo.push_back(v);
        for (int32_t j = g->succ_off[v]; j < g->succ_off[v + 1]; ++j)
          if (--indeg[g->succ[j]] == 0) ready.push(g->succ[j]);
      }
      if ((int32_t)g->topo.size() != n_ops) {
        set_error("operator graph has a cycle (%d of %d operators sortable)", (int)g->topo.size(), n_ops);
        delete g;
        return OPARA_ECYCLE;
      }
      g->tindex.assign(n_ops, 0);
      for (int i = 0; i < n_ops; ++i) g->tindex[g->topo[i]] = i;
    }
    // ---- kernel plan + demand record per operator
    g->plan.resize(n_ops);
    g->plan_persist.resize(n_ops);
    g->plan_group.resize(n_ops);
    g->dem.resize(n_ops);
    for (int v = 0; v < n_ops; ++v) {
      const opara_op_desc &op = g->ops[v];
      const void *in[OPARA_MAX_INPUTS];
      for (int i = 0; i < op.n_inputs; ++i) {
        const int32_t u = op.inputs[i];
        in[i] = u < 0 ? g->ext[-(int64_t)u - 1] : g->ops[u].out;
        if (!in[i]) { set_error("operator %d: input %d resolves to a null pointer", v, i); delete g; return OPARA_EINVAL; }
      }
      rc = plan_op(op, in, kPlanGraph, &g->plan[v]);
      if (rc == OPARA_OK) rc = plan_op(op, in, kPlanPersistent, &g->plan_persist[v]);
      if (rc == OPARA_OK) rc = plan_op(op, in, kPlanGroup, &g->plan_group[v]);
      if (rc != OPARA_OK) { delete g; return rc; }
      g->plan[v].tag = g->plan_persist[v].tag = g->plan_group[v].tag = v;
      const KernelPlan &p = g->plan[v];
      const KernelResource &r = kKernelResources[p.kernel];
      opara_demand &d = g->dem[v];
      d.kernel_id = p.kernel;
      d.op_class = op.op_class == OPARA_CLASS_DEFAULT ? default_class(op.op_type) : op.op_class;
      if (op.grid_blocks | op.block_threads | op.lds_bytes | op.vgprs) {
        d.grid_blocks = op.grid_blocks; d.block_threads = op.block_threads;
        d.lds_bytes = op.lds_bytes; d.vgprs = op.vgprs;
      } else {
        d.grid_blocks = p.gx * p.gy * p.gz; d.block_threads = p.block;
        d.lds_bytes = r.lds_bytes; d.vgprs = r.vgprs + r.agprs;
      }
      d.demand = demand_scalar(d, g->lim);
    }
  } catch (const std::bad_alloc &) {
    set_error("out of memory");
    delete g;
    return OPARA_ENOMEM;
  }
  *out = g;
  return OPARA_OK;
}

extern "C" int opara_assign_streams(opara_dag *g, int32_t *stream_of, int32_t *n_streams) {
  if (!g || !stream_of || !n_streams) { set_error("opara_assign_streams: null pointer"); return OPARA_EINVAL; }
  const int32_t n = g->n;
  std::vector<uint8_t> claimed(n, 0);      // the paper's SYNC flag
  g->stream_of.assign(n, -1);
  int32_t ns = 0;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t v = g->topo[i];
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t p = g->pred[j];
      if (!claimed[p]) { g->stream_of[v] = g->stream_of[p]; claimed[p] = 1; break; }
    }
    if (g->stream_of[v] < 0) g->stream_of[v] = ns++;
  }
  g->n_streams = ns;
  std::memcpy(stream_of, g->stream_of.data(), sizeof(int32_t) * n);
  *n_streams = ns;
  return OPARA_OK;
}

namespace {

// Bit matrix: row u holds the operators reachable from u.
struct Reach {
  int32_t n = 0, words = 0;
  std::vector<uint64_t> bits;
  void init(int32_t n_) { n = n_; words = (n_ + 63) / 64; bits.assign((size_t)n * words, 0); }
  uint64_t *row(int32_t u) { return bits.data() + (size_t)u * words; }
  const uint64_t *row(int32_t u) const { return bits.data() + (size_t)u * words; }
  bool get(int32_t u, int32_t v) const { return row(u)[v >> 6] >> (v & 63) & 1; }
  void set(int32_t u, int32_t v) { row(u)[v >> 6] |= 1ull << (v & 63); }
  void merge(int32_t u, int32_t v) { uint64_t *a = row(u); const uint64_t *b = row(v); for (int32_t w = 0; w < words; ++w) a[w] |= b[w]; }
};

// Kuhn's augmenting path over "v is a descendant of u"; match_r[v] = the operator v follows.
bool augment(const Reach &r, int32_t u, std::vector<int32_t> &match_r, std::vector<uint8_t> &seen) {
  for (int32_t v = 0; v < r.n; ++v) {
    if (!r.get(u, v) || seen[v]) continue;
    seen[v] = 1;
    if (match_r[v] < 0 || augment(r, match_r[v], match_r, seen)) { match_r[v] = u; return true; }
  }
  return false;
}

}  // namespace

// Fewest streams: a stream can hold any set of operators totally ordered by the dependency
// relation, so the minimum is a minimum chain cover = n - maximum matching between
// operators and their descendants (the matching-based allocation the paper compares
// Alg. 1 with, Sec. 5.2 and 5.4: cubic in n).
static int assign_min_streams(opara_dag *g) {
  const int32_t n = g->n;
  Reach r;
  r.init(n);
  for (int32_t i = n - 1; i >= 0; --i) {
    const int32_t u = g->topo[i];
    for (int32_t j = g->succ_off[u]; j < g->succ_off[u + 1]; ++j) { r.set(u, g->succ[j]); r.merge(u, g->succ[j]); }
  }
  std::vector<int32_t> match_r(n, -1);
  std::vector<uint8_t> seen(n);
  for (int32_t i = 0; i < n; ++i) {
    std::fill(seen.begin(), seen.end(), 0);
    augment(r, g->topo[i], match_r, seen);
  }
  g->stream_of.assign(n, -1);
  int32_t ns = 0;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t v = g->topo[i];
    g->stream_of[v] = match_r[v] < 0 ? ns++ : g->stream_of[match_r[v]];
  }
  g->n_streams = ns;
  return OPARA_OK;
}

extern "C" int opara_assign_streams_policy(opara_dag *g, int32_t policy, int32_t *stream_of, int32_t *n_streams) {
  if (policy == OPARA_STREAMS_ALG1) return opara_assign_streams(g, stream_of, n_streams);
  if (!g || !stream_of || !n_streams) { set_error("opara_assign_streams_policy: null pointer"); return OPARA_EINVAL; }
  if (policy != OPARA_STREAMS_MIN) { set_error("opara_assign_streams_policy: unknown policy %d", policy); return OPARA_EINVAL; }
  try {
    assign_min_streams(g);
  } catch (const std::bad_alloc &) {
    set_error("out of memory");
    return OPARA_ENOMEM;
  }
  std::memcpy(stream_of, g->stream_of.data(), sizeof(int32_t) * g->n);
  *n_streams = g->n_streams;
  return OPARA_OK;
}

// keep[k] for the k-th entry of the opara_sync_edges list: false if the dependency is implied
// by a longer chain of ordering constraints (dependencies + stream order in the queue).
int opara::sync_keep_mask(const opara_dag *g, std::vector<uint8_t> *keep) {
  const int32_t n = g->n;
  std::vector<std::vector<int32_t>> succ(n);
  for (int32_t v = 0; v < n; ++v)
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) succ[g->pred[j]].push_back(v);
  {
    std::vector<int32_t> last(g->n_streams, -1);
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = g->order[i], sv = g->stream_of[v];
      if (last[sv] >= 0) succ[last[sv]].push_back(v);
      last[sv] = v;
    }
  }
  Reach r;
  r.init(n);
  for (int32_t i = n - 1; i >= 0; --i) {
    const int32_t u = g->order[i];
    for (int32_t v : succ[u]) { r.set(u, v); r.merge(u, v); }
  }
  keep->clear();
  for (int32_t v = 0; v < n; ++v)
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t u = g->pred[j];
      if (g->stream_of[u] == g->stream_of[v]) continue;
      bool implied = false;
      for (int32_t w : succ[u]) implied = implied || (w != v && r.get(w, v));
      keep->push_back(!implied);
    }
  return OPARA_OK;
}

extern "C" int opara_sync_edges_pruned(const opara_dag *g, int32_t *uv, int32_t cap, int32_t *n_edges) {
  if (!g || !n_edges || cap < 0 || (cap > 0 && !uv)) { set_error("opara_sync_edges_pruned: bad argument"); return OPARA_EINVAL; }
  if (g->stream_of.empty() || g->order.empty()) {
    set_error("opara_sync_edges_pruned: call opara_assign_streams and opara_order_launch first");
    return OPARA_ESTATE;
  }
  std::vector<uint8_t> keep;
  try {
    sync_keep_mask(g, &keep);
  } catch (const std::bad_alloc &) {
    set_error("out of memory");
    return OPARA_ENOMEM;
  }
  int32_t k = 0, e = 0;
  for (int32_t v = 0; v < g->n; ++v)
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t u = g->pred[j];
      if (g->stream_of[u] == g->stream_of[v]) continue;
      if (keep[e++]) {
        if (k < cap) { uv[2 * k] = u; uv[2 * k + 1] = v; }
        ++k;
      }
    }
  *n_edges = k;
  return OPARA_OK;
}

extern "C" int opara_order_launch_policy(opara_dag *g, int32_t policy, int32_t *order) {
  if (!g || !order) { set_error("opara_order_launch: null pointer"); return OPARA_EINVAL; }
  if (policy < 0 || policy >= OPARA_N_ORDER_POLICIES) {
    set_error("opara_order_launch_policy: unknown policy %d", policy);
    return OPARA_EINVAL;
  }
  const int32_t n = g->n;
  // Ready lists as min-heaps; the pop is the argmin of the policy's key.  The paper's
  // Alg. 2 keeps two lists (memory- / compute-intensive) keyed by (demand, topological
  // index) and alternates between them; the other policies use a single list.
  typedef std::pair<uint64_t, int32_t> Key;
  std::priority_queue<Key, std::vector<Key>, std::greater<Key>> ready[2];
  const bool two_lists = policy == OPARA_ORDER_ALG2 || policy == OPARA_ORDER_ALG2_COMP_FIRST;
  std::vector<int32_t> indeg(n), level(n, 0);
  for (int32_t v = 0; v < n; ++v) indeg[v] = g->pred_off[v + 1] - g->pred_off[v];
  if (policy == OPARA_ORDER_LEVEL)
    for (int32_t i = 0; i < n; ++i) {
      const int32_t v = g->topo[i];
      for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) level[v] = std::max(level[v], level[g->pred[j]] + 1);
    }
  auto push = [&](int32_t v) {
    switch (policy) {
      case OPARA_ORDER_ALG2: case OPARA_ORDER_ALG2_COMP_FIRST:
        ready[g->dem[v].op_class].push(Key(g->dem[v].demand, g->tindex[v])); break;
      case OPARA_ORDER_LEAST_DEMAND: ready[0].push(Key(g->dem[v].demand, g->tindex[v])); break;
      case OPARA_ORDER_MOST_DEMAND: ready[0].push(Key(~g->dem[v].demand, g->tindex[v])); break;
      case OPARA_ORDER_LEVEL: ready[0].push(Key((uint64_t)level[v], g->tindex[v])); break;
      default: ready[0].push(Key(0, g->tindex[v])); break;   // OPARA_ORDER_TOPO
    }
  };
  for (int32_t v = 0; v < n; ++v) if (indeg[v] == 0) push(v);
  g->order.clear();
  g->order.reserve(n);
  int pref = policy == OPARA_ORDER_ALG2_COMP_FIRST ? OPARA_COMP : OPARA_MEM;
  while (!ready[0].empty() || !ready[1].empty()) {
    const int cls = two_lists ? (!ready[pref].empty() ? pref : 1 - pref) : 0;
    const int32_t v = g->topo[ready[cls].top().second];
    ready[cls].pop();
    g->order.push_back(v);
    pref = 1 - cls;
    for (int32_t j = g->succ_off[v]; j < g->succ_off[v + 1]; ++j) {
      const int32_t s = g->succ[j];
      if (--indeg[s] == 0) push(s);
    }
  }
  ++g->order_gen;
  std::memcpy(order, g->order.data(), sizeof(int32_t) * n);
  return OPARA_OK;
}

extern "C" int opara_order_launch(opara_dag *g, int32_t *order) {
  return opara_order_launch_policy(g, OPARA_ORDER_ALG2, order);
}

extern "C" int opara_sync_edges(const opara_dag *g, int32_t *uv, int32_t cap, int32_t *n_edges) {
  if (!g || !n_edges || cap < 0 || (cap > 0 && !uv)) { set_error("opara_sync_edges: bad argument"); return OPARA_EINVAL; }
  if (g->stream_of.empty()) { set_error("opara_sync_edges: call opara_assign_streams first"); return OPARA_ESTATE; }
  int32_t k = 0;
  for (int32_t v = 0; v < g->n; ++v)
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) {
      const int32_t u = g->pred[j];
      if (g->stream_of[u] == g->stream_of[v]) continue;
      if (k < cap) { uv[2 * k] = u; uv[2 * k + 1] = v; }
      ++k;
    }
  *n_edges = k;
  return OPARA_OK;
}

// Wave of every operator: 0 for operators without predecessors, else one more than the
// largest wave among its predecessors.  These are the groups the fused executor launches
// together (it takes, again and again, every operator whose predecessors have all run).
extern "C" int opara_wave_of(const opara_dag *g, int32_t *wave_of, int32_t *n_waves) {
  if (!g || !wave_of) { set_error("opara_wave_of: null pointer"); return OPARA_EINVAL; }
  int32_t deepest = -1;
  for (int32_t i = 0; i < g->n; ++i) {
    const int32_t v = g->topo[i];
    int32_t w = 0;
    for (int32_t j = g->pred_off[v]; j < g->pred_off[v + 1]; ++j) w = std::max(w, wave_of[g->pred[j]] + 1);
    wave_of[v] = w;
    deepest = std::max(deepest, w);
  }
  if (n_waves) *n_waves = deepest + 1;
  return OPARA_OK;
}

extern "C" int opara_get_demands(const opara_dag *g, opara_demand *out) {
  if (!g || !out) { set_error("opara_get_demands: null pointer"); return OPARA_EINVAL; }
  std::memcpy(out, g->dem.data(), sizeof(opara_demand) * g->n);
  return OPARA_OK;
}

extern "C" int opara_topo_order(const opara_dag *g, int32_t *order) {
  if (!g || !order) { set_error("opara_topo_order: null pointer"); return OPARA_EINVAL; }
  std::memcpy(order, g->topo.data(), sizeof(int32_t) * g->n);
  return OPARA_OK;
}

extern "C" int32_t opara_num_ops(const opara_dag *g) { return g ? g->n : 0; }

extern "C" void opara_dag_destroy(opara_dag *g) { delete g; }

extern "C" int32_t opara_kernel_count(void) { return K_COUNT; }

extern "C" int opara_persistent_plan(const opara_dag *g, int32_t *tiles, int32_t *kernel_ids) {
  if (!g) { set_error("opara_persistent_plan: null graph"); return OPARA_EINVAL; }
  for (int32_t v = 0; v < g->n; ++v) {
    const KernelPlan &p = g->plan_persist[v];
    if (tiles) tiles[v] = (int32_t)((int64_t)p.gx * p.gy * p.gz);
    if (kernel_ids) kernel_ids[v] = p.kernel;
  }
  return OPARA_OK;
}

extern "C" int opara_kernel_info(int32_t id, const char **name, uint32_t *vgprs, uint32_t *lds_bytes) {
  if (id < 0 || id >= K_COUNT) { set_error("opara_kernel_info: id %d out of range", id); return OPARA_EINVAL; }
  const KernelResource &r = kKernelResources[id];
  if (name) *name = r.name;
  if (vgprs) *vgprs = r.vgprs + r.agprs;
  if (lds_bytes) *lds_bytes = r.lds_bytes;
  return OPARA_OK;
}
