"""The paper's two scheduling algorithms, step by step (test oracle; not used by
the product path).

  * assign_streams : stream allocation, paper Algorithm 1 (Sec. 3.1) and the four
    placement rules of the appendix example.
  * order_launch   : operator launch order, paper Algorithm 2 (Sec. 3.3).
  * sync_edges     : the dependencies that need a synchronisation operator
    (Sec. 3.1 "synchronization operators", Sec. 4 event record / wait).
  * check_schedule : validity of (stream map, launch queue, sync list).
  * min_streams    : the fewest streams any allocation can use - the comparison system's
    policy the paper sets Alg. 1 against (Sec. 5.2: 28 streams against 4 on GoogLeNet;
    Sec. 5.4: cubic matching against the linear greedy pass).
  * waves          : the groups of operators that can run together once all earlier groups
    have run (the level-synchronous schedule the paper's comparison systems use, Sec. 5.1;
    this build launches each group as one kernel).
  * prune_syncs    : the synchronisations that remain once those implied by other
    dependencies are dropped (Sec. 3.1: every synchronisation costs t_overhead, Eq. 3).

Readings where the paper is silent (all repeated in the design notes):
  - topological order = Kahn with the smallest operator id first;
  - predecessors are visited in argument order, duplicates dropped keeping the first;
  - streams get dense ids in creation order and are never reused;
  - external tensors are not operators;
  - "alternately choose": preference starts at the memory list; the preferred list
    is used when non-empty, otherwise the other; after a pick the preference is the
    class opposite to the one just picked;
  - "least amount of GPU resources": demand = grid_blocks * share, where share is the
    largest of the workgroup's fractions of a compute unit's thread slots, LDS and
    vector registers, each in units of 2^-16, rounded up;
  - argmin ties: smaller topological index first.
"""
from .executor import kahn_order

MEM, COMP = 0, 1


def dedup_preds(inputs_per_op):
    """Operator predecessors in argument order, externals (<0) and repeats dropped."""
    preds = []
    for ins in inputs_per_op:
        seen, lst = set(), []
        for u in ins:
            if u >= 0 and u not in seen:
                seen.add(u)
                lst.append(u)
        preds.append(lst)
    return preds


def _edges(preds):
    return [(u, v) for v, ps in enumerate(preds) for u in ps]


def assign_streams(preds):
    """Algorithm 1.  Returns (stream_of, n_streams)."""
    n = len(preds)
    topo = kahn_order(n, _edges(preds))
    sync_flag = [False] * n
    stream_of = [None] * n
    n_streams = 0
    for v in topo:
        for p in preds[v]:
            if not sync_flag[p]:
                stream_of[v] = stream_of[p]
                sync_flag[p] = True
                break
        if stream_of[v] is None:
            stream_of[v] = n_streams
            n_streams += 1
    return stream_of, n_streams


def _ceil_div(a, b):
    return -(-a // b)


def demand_scalar(rec, limits):
    """rec = (grid_blocks, block_threads, lds_bytes, vgprs); limits = dict with
    threads_per_cu, lds_bytes_per_cu, vgpr_lanes_per_cu.  One integer in units of
    2^-16 of a compute unit."""
    g, t, lds, vg = rec
    share = max(_ceil_div(65536 * t, limits["threads_per_cu"]),
                _ceil_div(65536 * lds, limits["lds_bytes_per_cu"]),
                _ceil_div(65536 * t * vg, limits["vgpr_lanes_per_cu"]))
    return g * share


def order_launch(preds, op_class, demand):
    """Algorithm 2.  op_class[v] in {MEM, COMP}; demand[v] integer.  Returns Q."""
    n = len(preds)
    topo = kahn_order(n, _edges(preds))
    tindex = [0] * n
    for i, v in enumerate(topo):
        tindex[v] = i
    succ = [[] for _ in range(n)]
    indeg = [0] * n
    for v, ps in enumerate(preds):
        for u in ps:
            succ[u].append(v)
            indeg[v] += 1
    lists = {MEM: [], COMP: []}
    for v in topo:
        if indeg[v] == 0:
            lists[op_class[v]].append(v)
    q = []
    pref = MEM
    while lists[MEM] or lists[COMP]:
        cls = pref if lists[pref] else (COMP if pref == MEM else MEM)
        lst = lists[cls]
        vmin = min(lst, key=lambda u: (demand[u], tindex[u]))
        lst.remove(vmin)
        q.append(vmin)
        pref = COMP if cls == MEM else MEM
        for s in succ[vmin]:
            indeg[s] -= 1
            if indeg[s] == 0:
                lists[op_class[s]].append(s)
    return q


POLICIES = ("alg2", "alg2_comp_first", "least_demand", "most_demand", "topo", "level")


def order_launch_policy(preds, op_class, demand, policy):
    """Launch-order variants for the order ablation (paper Sec. 2.3 compares launch
    orders).  "alg2" is Algorithm 2; "alg2_comp_first" starts its alternation at the
    compute list; "least_demand"/"most_demand" keep one ready list ordered by demand;
    "topo" is Kahn smallest id; "level" goes wave by wave (depth, then id)."""
    n = len(preds)
    topo = kahn_order(n, _edges(preds))
    tindex = {v: i for i, v in enumerate(topo)}
    if policy == "alg2":
        return order_launch(preds, op_class, demand)
    if policy == "topo":
        return topo
    if policy == "level":
        depth = [0] * n
        for v in topo:
            for u in preds[v]:
                depth[v] = max(depth[v], depth[u] + 1)
        return sorted(range(n), key=lambda v: (depth[v], tindex[v]))
    succ = [[] for _ in range(n)]
    indeg = [len(p) for p in preds]
    for v, ps in enumerate(preds):
        for u in ps:
            succ[u].append(v)
    ready = [v for v in topo if indeg[v] == 0]
    q, pref = [], COMP
    while ready:
        if policy == "alg2_comp_first":
            pool = [v for v in ready if op_class[v] == pref] or ready
            key = lambda u: (demand[u], tindex[u])
        elif policy == "least_demand":
            pool, key = ready, (lambda u: (demand[u], tindex[u]))
        elif policy == "most_demand":
            pool, key = ready, (lambda u: (-demand[u], tindex[u]))
        else:
            raise ValueError(policy)
        v = min(pool, key=key)
        ready.remove(v)
        q.append(v)
        pref = MEM if op_class[v] == COMP else COMP
        for s in succ[v]:
            indeg[s] -= 1
            if indeg[s] == 0:
                ready.append(s)
    return q


def waves(preds):
    """Wave of every operator: 0 without predecessors, else 1 + the largest wave among its
    predecessors, i.e. the length of the longest dependency chain that ends in it.  Taking,
    again and again, every operator whose predecessors have all run yields these groups."""
    n = len(preds)
    wave = [None] * n
    left = set(range(n))
    k = 0
    while left:
        ready = [v for v in left if all(wave[u] is not None and wave[u] < k for u in preds[v])]
        if not ready:
            raise ValueError("graph has a cycle")
        for v in ready:
            wave[v] = k
        left -= set(ready)
        k += 1
    return wave


def sync_edges(preds, stream_of):
    """All dependencies whose endpoints sit on different streams, sorted by (v, arg position)."""
    return [(u, v) for v, ps in enumerate(preds) for u in ps if stream_of[u] != stream_of[v]]


def check_schedule(preds, stream_of, q, syncs):
    """Raise AssertionError unless q is a topological permutation and every edge is
    either same-stream (ordered by q) or listed in syncs."""
    n = len(preds)
    assert sorted(q) == list(range(n)), "Q is not a permutation"
    pos = [0] * n
    for i, v in enumerate(q):
        pos[v] = i
    sset = set(syncs)
    for v, ps in enumerate(preds):
        for u in ps:
            assert pos[u] < pos[v], f"edge {u}->{v} violates launch order"
            if stream_of[u] != stream_of[v]:
                assert (u, v) in sset, f"cross-stream edge {u}->{v} has no sync"
    for (u, v) in syncs:
        assert u in preds[v] and stream_of[u] != stream_of[v], f"spurious sync {u}->{v}"
    return True


def _reach(preds):
    """reach[u] = set of operators reachable from u by one or more edges."""
    n = len(preds)
    succ = [[] for _ in range(n)]
    for v, ps in enumerate(preds):
        for u in ps:
            succ[u].append(v)
    topo = kahn_order(n, _edges(preds))
    reach = [set() for _ in range(n)]
    for u in reversed(topo):
        for v in succ[u]:
            reach[u].add(v)
            reach[u] |= reach[v]
    return reach


def min_streams(preds):
    """Fewest streams: a stream may hold any set of operators that are totally ordered by
    the dependency relation (a chain), so the minimum is a minimum chain cover, found as
    n minus a maximum matching between operators and their descendants (Dilworth /
    Fulkerson).  Returns (stream_of, n_streams); streams are numbered by their first
    operator in topological order.  The matching is not unique, the count is."""
    n = len(preds)
    reach = _reach(preds)
    topo = kahn_order(n, _edges(preds))
    match_r = [None] * n          # descendant -> the operator it follows on its stream

    def augment(u, seen):
        for v in sorted(reach[u]):
            if v in seen:
                continue
            seen.add(v)
            if match_r[v] is None or augment(match_r[v], seen):
                match_r[v] = u
                return True
        return False

    for u in topo:
        augment(u, set())
    stream_of = [None] * n
    n_streams = 0
    for v in topo:                # a predecessor on the chain comes earlier in topological order
        if match_r[v] is None:
            stream_of[v] = n_streams
            n_streams += 1
        else:
            stream_of[v] = stream_of[match_r[v]]
    return stream_of, n_streams


def execution_edges(preds, stream_of, q):
    """Ordering constraints of a multi-stream run: every dependency, plus consecutive
    operators of one stream in launch-queue order."""
    edges = set(_edges(preds))
    last = {}
    for v in q:
        s = stream_of[v]
        if s in last:
            edges.add((last[s], v))
        last[s] = v
    return edges


def prune_syncs(preds, stream_of, q):
    """Cross-stream dependencies that still need a synchronisation when every one that is
    implied by a longer chain of constraints (dependencies and stream order) is dropped.
    Sorted like sync_edges."""
    edges = execution_edges(preds, stream_of, q)
    n = len(preds)
    succ = [[] for _ in range(n)]
    for u, v in edges:
        succ[u].append(v)
    pos = {v: i for i, v in enumerate(q)}
    reach = [set() for _ in range(n)]
    for u in sorted(range(n), key=lambda x: -pos[x]):
        for v in succ[u]:
            reach[u].add(v)
            reach[u] |= reach[v]
    keep = []
    for (u, v) in sync_edges(preds, stream_of):
        implied = any(w != v and v in reach[w] for w in succ[u])
        if not implied:
            keep.append((u, v))
    return keep
