"""Pins for the oracle scheduler (Alg. 1, Alg. 2, sync edges): the values the paper
prints, the appendix placement rules, closed forms and invariants on random DAGs."""
import json
import os
import numpy as np
import pytest
from oracle import sched
from oracle.executor import kahn_order
from workloads import (googlenet_like, inception_block, inception_v3_like, bert_base_like,
                       appendix_example_edges, COMPUTE_TYPES)

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def preds_of(wl):
    return sched.dedup_preds([o.inputs for o in wl.ops])


def preds_from_edges(n, edges):
    p = [[] for _ in range(n)]
    for u, v in edges:
        p[v].append(u)
    return p


def random_preds(rng, n, max_fan_in=3, p_root=0.2):
    preds = [[]]
    for v in range(1, n):
        if rng.random() < p_root:
            preds.append([])
            continue
        k = int(rng.integers(1, max_fan_in + 1))
        preds.append([int(u) for u in rng.choice(v, size=min(k, v), replace=False)])
    return preds


def test_googlenet_opens_28_streams():
    so, ns = sched.assign_streams(preds_of(googlenet_like()))
    assert ns == GOLD["googlenet_streams"]["value"]


def test_appendix_rules():
    edges = [(u - 1, v - 1) for u, v in appendix_example_edges()]
    preds = preds_from_edges(13, edges)
    so, ns = sched.assign_streams(preds)
    s = lambda i: so[i - 1]
    r = GOLD["appendix_rules"]
    # an operator opens a new stream exactly when the rules say so
    openers = sorted(i for i in range(1, 14) if all(s(i) != s(j) for j in range(1, i)))
    assert openers == r["new_stream"] and ns == len(openers)
    for i in r["same_stream_as_only_pred"] + r["first_successor_joins_pred"]:
        (p,) = preds[i - 1]
        assert s(i) == so[p]
    assert s(8) == s(5) and s(13) == s(10)      # first predecessor whose flag is still False
    assert [s(i) for i in (1, 2, 5, 8, 9, 11)] == [s(1)] * 6
    assert s(3) == s(6) and s(4) == s(7) and len({s(1), s(3), s(4), s(10), s(12)}) == 5
    # swapping the argument order of operator 13 changes which predecessor it joins
    preds2 = [list(p) for p in preds]
    preds2[12] = [11, 10, 9]
    so2, _ = sched.assign_streams(preds2)
    assert so2[12] == so2[11]


def test_closed_forms():
    chain = [[]] + [[i] for i in range(9)]
    so, ns = sched.assign_streams(chain)
    assert ns == 1 and so == [0] * 10 and sched.sync_edges(chain, so) == []
    k = 5                                     # root -> k branches -> join
    fj = [[]] + [[0]] * k + [list(range(1, k + 1))]
    so, ns = sched.assign_streams(fj)
    assert ns == k and so[1] == so[0] and so[k + 1] == so[1]
    assert len(sched.sync_edges(fj, so)) == 2 * (k - 1)
    # independent roots each open a stream
    assert sched.assign_streams([[], [], []]) == ([0, 1, 2], 3)


@pytest.mark.parametrize("builder,n_streams,n_sync", [
    (inception_block, 4, 3), (googlenet_like, 28, None), (inception_v3_like, 36, None),
    (bert_base_like, 25, None)])
def test_config_stream_counts(builder, n_streams, n_sync):
    wl = builder()
    preds = preds_of(wl)
    so, ns = sched.assign_streams(preds)
    assert ns == n_streams
    if n_sync is not None:
        assert len(sched.sync_edges(preds, so)) == n_sync
    if builder is inception_block:
        # only the non-first branch tails into the concat need an event
        assert sched.sync_edges(preds, so) == [(2, 7), (4, 7), (6, 7)]


@pytest.mark.parametrize("seed", range(40))
def test_invariants_random(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    preds = random_preds(rng, n)
    so, ns = sched.assign_streams(preds)
    assert sorted(set(so)) == list(range(ns))
    # each stream is a path; each operator is claimed at most once; n_streams = n - #claims
    topo = kahn_order(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    last, claims, claimed = {}, 0, set()
    for v in topo:
        s = so[v]
        if s in last:
            assert last[s] in preds[v]
            assert last[s] not in claimed
            claimed.add(last[s]); claims += 1
        last[s] = v
    assert ns == n - claims
    cls = [int(rng.integers(0, 2)) for _ in range(n)]
    dem = [int(rng.integers(1, 50)) for _ in range(n)]
    q = sched.order_launch(preds, cls, dem)
    syncs = sched.sync_edges(preds, so)
    assert sched.check_schedule(preds, so, q, syncs)
    # within a stream the launch queue follows the path order
    pos = {v: i for i, v in enumerate(q)}
    tpos = {v: i for i, v in enumerate(topo)}
    for a in range(n):
        for b in range(n):
            if so[a] == so[b] and tpos[a] < tpos[b]:
                assert pos[a] < pos[b]
    # a missing sync edge or a non-topological queue is caught
    if syncs:
        with pytest.raises(AssertionError):
            sched.check_schedule(preds, so, q, syncs[1:])
    if any(preds):
        v = next(i for i in range(n) if preds[i])
        bad = [x for x in q if x != v]
        bad.insert(0, v)
        with pytest.raises(AssertionError):
            sched.check_schedule(preds, so, bad, syncs)


def replay_alg2(preds, cls, dem, q):
    """Re-walk Q with independent ready-set bookkeeping and check every pick."""
    n = len(preds)
    topo = kahn_order(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    tidx = {v: i for i, v in enumerate(topo)}
    done, prev_cls = set(), None
    for i, v in enumerate(q):
        ready = [u for u in range(n) if u not in done and all(p in done for p in preds[u])]
        rc = {c: [u for u in ready if cls[u] == c] for c in (0, 1)}
        assert v in ready
        if rc[0] and rc[1]:
            want = sched.MEM if prev_cls is None else 1 - prev_cls
            assert cls[v] == want, "classes must alternate while both lists are non-empty"
        best = min(rc[cls[v]], key=lambda u: (dem[u], tidx[u]))
        assert v == best, "least-demand operator of the chosen list first"
        done.add(v)
        prev_cls = cls[v]


@pytest.mark.parametrize("seed", range(30))
def test_alg2_pick_by_pick(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(2, 30))
    preds = random_preds(rng, n, p_root=0.35)
    cls = [int(rng.integers(0, 2)) for _ in range(n)]
    dem = [int(rng.integers(1, 6)) for _ in range(n)]     # many ties
    replay_alg2(preds, cls, dem, sched.order_launch(preds, cls, dem))


def test_alg2_special_cases():
    rng = np.random.default_rng(7)
    preds = random_preds(rng, 25)
    n = len(preds)
    topo = kahn_order(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    # one class, equal demand: reduces to Kahn smallest-id order
    assert sched.order_launch(preds, [1] * n, [3] * n) == topo
    # four independent roots: memory list first, then strict alternation, small before large
    q = sched.order_launch([[], [], [], []], [1, 1, 0, 0], [5, 2, 9, 4])
    assert q == [3, 1, 2, 0]
    # GoogLeNet block: the pool-headed branch (memory-intensive) is launched first
    wl = inception_block()
    p = sched.dedup_preds([o.inputs for o in wl.ops])
    cls = [1 if o.type in COMPUTE_TYPES else 0 for o in wl.ops]
    q = sched.order_launch(p, cls, [1] * len(p))
    assert wl.ops[q[0]].type == "maxpool"


def test_demand_scalar():
    lim = dict(threads_per_cu=2048, lds_bytes_per_cu=163840, vgpr_lanes_per_cu=131072)
    assert sched.demand_scalar((10, 256, 0, 0), lim) == 10 * 8192          # 1/8 of the thread slots
    assert sched.demand_scalar((3, 64, 81920, 16), lim) == 3 * 32768       # LDS binds: half a CU
    assert sched.demand_scalar((1, 256, 1024, 128), lim) == 16384          # registers bind: a quarter
    assert sched.demand_scalar((2, 100, 1, 1), lim) == 2 * 3200            # rounds up


# ---------------------------------------------------------------- fewest streams, sync pruning
def closure(n, edges):
    """Reachability by Warshall's algorithm (independent of the oracle's traversal)."""
    r = np.zeros((n, n), dtype=bool)
    for u, v in edges:
        r[u, v] = True
    for k in range(n):
        r |= np.outer(r[:, k], r[k, :])
    return r


def test_googlenet_needs_4_streams_at_least():
    ms, n = sched.min_streams(preds_of(googlenet_like()))
    assert n == GOLD["googlenet_min_streams"]["value"]
    assert sched.min_streams(preds_of(inception_block()))[1] == 4      # four branches
    chain = [[]] + [[i] for i in range(9)]
    assert sched.min_streams(chain)[1] == 1
    assert sched.min_streams([[] for _ in range(5)])[1] == 5           # no edges: one stream each


@pytest.mark.parametrize("seed", range(60))
def test_min_streams_is_the_width_of_the_dag(seed):
    """Dilworth: the fewest chains covering a partial order equal its largest antichain
    (brute force over all subsets), and every stream must be a chain."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 11))
    preds = random_preds(rng, n, p_root=0.35)
    so, ns = sched.min_streams(preds)
    r = closure(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    comparable = r | r.T
    width = 0
    for mask in range(1, 1 << n):
        idx = [i for i in range(n) if mask >> i & 1]
        if len(idx) > width and not any(comparable[a, b] for a in idx for b in idx if a < b):
            width = len(idx)
    assert ns == width
    assert sorted(set(so)) == list(range(ns))
    for s_ in range(ns):
        members = [v for v in range(n) if so[v] == s_]
        assert all(comparable[a, b] for a in members for b in members if a < b)
    assert ns <= sched.assign_streams(preds)[1]


@pytest.mark.parametrize("seed", range(60))
def test_pruned_syncs_keep_every_ordering_and_are_minimal(seed):
    rng = np.random.default_rng(2000 + seed)
    n = int(rng.integers(2, 14))
    preds = random_preds(rng, n, max_fan_in=4)
    cls = [int(rng.integers(0, 2)) for _ in range(n)]
    dem = [int(rng.integers(1, 50)) for _ in range(n)]
    q = sched.order_launch(preds, cls, dem)
    for so in (sched.assign_streams(preds)[0], sched.min_streams(preds)[0]):
        full = sched.sync_edges(preds, so)
        kept = sched.prune_syncs(preds, so, q)
        assert set(kept) <= set(full) and kept == [e for e in full if e in set(kept)]
        order_edges = sched.execution_edges(preds, so, q) - set(full)      # stream order + same-stream dependencies
        want = closure(n, list(order_edges) + full)
        assert np.array_equal(closure(n, list(order_edges) + kept), want)
        for e in kept:                                                     # none of the kept ones is implied
            rest = [x for x in kept if x != e]
            assert not closure(n, list(order_edges) + rest)[e[0], e[1]]


def test_pruning_special_cases():
    # diamond on two streams with a shortcut edge 0->3: the shortcut is implied by 0->1->3
    preds = [[], [0], [0], [1, 2, 0]]
    so = [0, 0, 1, 0]
    q = [0, 1, 2, 3]
    assert sched.sync_edges(preds, so) == [(0, 2), (2, 3)]
    assert sched.prune_syncs(preds, so, q) == [(0, 2), (2, 3)]
    so = [0, 1, 2, 3]                     # every operator on its own stream
    assert sched.sync_edges(preds, so) == [(0, 1), (0, 2), (1, 3), (2, 3), (0, 3)]
    assert sched.prune_syncs(preds, so, q) == [(0, 1), (0, 2), (1, 3), (2, 3)]
    # stream order implies a dependency: 0 and 1 on stream A in queue order, 2 on B needs both
    preds = [[], [], [0, 1]]
    assert sched.prune_syncs(preds, [0, 0, 1], [0, 1, 2]) == [(1, 2)]
    assert sched.prune_syncs(preds, [0, 0, 1], [1, 0, 2]) == [(0, 2)]


# ---------------------------------------------------------------- launch-order policies (Sec. 2.3 order comparison)
# Hand-worked example.  Seven operators, Kahn order = id order:
#   0 -> 2, 3     1 -> 4     2, 3 -> 5     4, 3 -> 6
# classes (M memory-, C compute-intensive) and demands (ties on purpose: 0/1 and 2/4):
#   id      0  1  2  3  4  5  6
#   class   C  M  M  C  C  M  C
#   demand  5  5  3  6  3  4  1
HAND_PREDS = [[], [], [0], [0], [1], [2, 3], [4, 3]]
HAND_CLS = [1, 0, 0, 1, 1, 0, 1]
HAND_DEM = [5, 5, 3, 6, 3, 4, 1]
# Each queue below was written out by hand from the policy's one-line definition:
#  alg2            start at M: 1 | C{0:5,4:3} -> 4 | M empty -> 0 | M{2} -> 2 | C{3} -> 3 | M{5} -> 5 | 6
#  alg2_comp_first start at C: 0 | M{1:5,2:3} -> 2 | C{3} -> 3 | M{1:5,5:4} -> 5 | C empty -> 1 | C{4} -> 4 | 6
#  least_demand    {0,1} tie -> 0 | {1:5,2:3,3:6} -> 2 | {1:5,3:6} -> 1 | {3:6,4:3} -> 4 | 3 | {5:4,6:1} -> 6 | 5
#  most_demand     {0,1} tie -> 0 | {1:5,2:3,3:6} -> 3 | {1:5,2:3} -> 1 | {2:3,4:3} tie -> 2 | {4:3,5:4} -> 5 | 4 | 6
HAND_QUEUES = {
    "alg2": [1, 4, 0, 2, 3, 5, 6],
    "alg2_comp_first": [0, 2, 3, 5, 1, 4, 6],
    "least_demand": [0, 2, 1, 4, 3, 6, 5],
    "most_demand": [0, 3, 1, 2, 5, 4, 6],
    "topo": [0, 1, 2, 3, 4, 5, 6],
    "level": [0, 1, 2, 3, 4, 5, 6],
}


@pytest.mark.parametrize("policy", sched.POLICIES)
def test_policy_queues_on_the_hand_worked_example(policy):
    assert sched.order_launch_policy(HAND_PREDS, HAND_CLS, HAND_DEM, policy) == HAND_QUEUES[policy]
    assert sched.order_launch(HAND_PREDS, HAND_CLS, HAND_DEM) == HAND_QUEUES["alg2"]


def test_level_and_trace_order_differ_where_ids_do_not_follow_depth():
    # 0 -> 3 -> 1 -> 5, 2 -> 4 -> 5.  Kahn smallest id: 0, 2, 3, 1, 4, 5 (1 becomes ready before 4 is taken);
    # depths 0:0 2:0 3:1 4:1 1:2 5:3, so wave by wave 4 comes before 1.
    preds = [[], [3], [], [0], [2], [1, 4]]
    cls, dem = [0] * 6, [1] * 6
    assert sched.order_launch_policy(preds, cls, dem, "topo") == [0, 2, 3, 1, 4, 5]
    assert sched.order_launch_policy(preds, cls, dem, "level") == [0, 2, 3, 4, 1, 5]


def replay_policy(preds, cls, dem, q, policy):
    """Independent pick-by-pick check of a one-list policy or of the compute-first Alg. 2:
    the ready set is recomputed from scratch before every pick."""
    n = len(preds)
    topo = kahn_order(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    tidx = {v: i for i, v in enumerate(topo)}
    done, prev_cls = set(), None
    assert sorted(q) == list(range(n))
    for v in q:
        ready = [u for u in range(n) if u not in done and all(p in done for p in preds[u])]
        assert v in ready
        if policy == "alg2_comp_first":
            want = sched.COMP if prev_cls is None else 1 - prev_cls
            same = [u for u in ready if cls[u] == want]
            pool = same if same else ready
            best = min(pool, key=lambda u: (dem[u], tidx[u]))
        elif policy == "least_demand":
            best = min(ready, key=lambda u: (dem[u], tidx[u]))
        else:
            best = min(ready, key=lambda u: (-dem[u], tidx[u]))
        assert v == best, (policy, v, best)
        done.add(v)
        prev_cls = cls[v]


@pytest.mark.parametrize("policy", ["alg2_comp_first", "least_demand", "most_demand"])
@pytest.mark.parametrize("seed", range(20))
def test_policy_pick_by_pick(seed, policy):
    rng = np.random.default_rng(3000 + seed)
    n = int(rng.integers(2, 30))
    preds = random_preds(rng, n, p_root=0.35)
    cls = [int(rng.integers(0, 2)) for _ in range(n)]
    dem = [int(rng.integers(1, 6)) for _ in range(n)]     # many ties
    replay_policy(preds, cls, dem, sched.order_launch_policy(preds, cls, dem, policy), policy)


@pytest.mark.parametrize("seed", range(20))
def test_level_order_is_depth_then_trace_order(seed):
    rng = np.random.default_rng(4000 + seed)
    n = int(rng.integers(2, 40))
    preds = random_preds(rng, n, p_root=0.3)
    q = sched.order_launch_policy(preds, [0] * n, [1] * n, "level")
    topo = sched.order_launch_policy(preds, [0] * n, [1] * n, "topo")
    assert topo == kahn_order(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
    # depth = length of the longest path from a root, from powers of the adjacency matrix
    a = np.zeros((n, n), dtype=np.int64)
    for v, ps in enumerate(preds):
        for u in ps:
            a[u, v] = 1
    depth, p = np.zeros(n, dtype=int), np.eye(n, dtype=np.int64)
    for k in range(1, n):
        p = np.minimum(p @ a, 1)
        depth[p.sum(0) > 0] = k
    tidx = {v: i for i, v in enumerate(topo)}
    assert sorted(q) == list(range(n))
    keys = [(int(depth[v]), tidx[v]) for v in q]
    assert keys == sorted(keys)


# ---------------------------------------------------------------- waves
def test_waves_hand_worked_and_longest_chain():
    # the hand-worked DAG above: 0, 1 | 2, 3, 4 | 5, 6
    assert sched.waves(HAND_PREDS) == [0, 0, 1, 1, 1, 2, 2]
    # ids that do not follow depth: 0 -> 3 -> 1 -> 5, 2 -> 4 -> 5
    assert sched.waves([[], [3], [], [0], [2], [1, 4]]) == [0, 2, 0, 1, 1, 3]
    assert sched.waves([[]] + [[i] for i in range(6)]) == list(range(7))        # a chain
    assert sched.waves([[], [], []]) == [0, 0, 0]
    with pytest.raises(ValueError):
        sched.waves([[1], [0]])


@pytest.mark.parametrize("seed", range(20))
def test_waves_are_longest_path_lengths(seed):
    rng = np.random.default_rng(5000 + seed)
    n = int(rng.integers(2, 40))
    preds = random_preds(rng, n, p_root=0.3)
    a = np.zeros((n, n), dtype=np.int64)
    for v, ps in enumerate(preds):
        for u in ps:
            a[u, v] = 1
    depth, p = np.zeros(n, dtype=int), np.eye(n, dtype=np.int64)
    for k in range(1, n):
        p = np.minimum(p @ a, 1)
        depth[p.sum(0) > 0] = k
    assert sched.waves(preds) == [int(d) for d in depth]
