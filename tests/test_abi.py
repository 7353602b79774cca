"""Host-side tests of the C ABI (no GPU needed): the library loads and exports every
declared symbol, rejects malformed graphs, and its scheduler agrees bit for bit with
the oracle scheduler on the configs and on thousands of random tiny DAGs."""
import ctypes as C
import os
import re
import numpy as np
import pytest
from oracle import sched
from paper_2312_10351_amd import binding as B
from paper_2312_10351_amd.runtime import Session
from workloads import (Builder, inception_block, googlenet_like, inception_v3_like, bert_base_like,
                       random_small_dag, random_wide_dag, nasnet_like)
from util import LIMITS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "opara.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(opara_\w+)\s*\(", header))
    assert {"opara_build_dag", "opara_assign_streams", "opara_order_launch", "opara_capture",
            "opara_replay"} <= declared
    lib = B.load()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in opara.h but not exported"
    assert declared == set(B.EXPORTS)


def test_struct_layouts_match_header():
    # sizes the C compiler gives the same records (natural alignment, no packing)
    assert C.sizeof(B.OpParams) == 16 * 4 + 6 * 8 + 8 * 4 + 3 * 4 + 4
    assert C.sizeof(B.OpDesc) == 4 * 4 + 8 * 4 + 4 * 4 + C.sizeof(B.OpParams) + 3 * 8 + 4 + 8 * 4 + 4
    assert C.sizeof(B.Demand) == 32
    assert C.sizeof(B.Limits) == 16


def chain_descs(n, inputs):
    descs = []
    for v in range(n):
        d = B.OpDesc()
        d.op_type, d.op_class, d.dtype = B.ADD, B.CLASS_DEFAULT, B.F16
        d.n_inputs = len(inputs[v])
        for i, u in enumerate(inputs[v]):
            d.inputs[i] = u
        d.params.m, d.params.n = 4, 64
        d.out = 0x10000 + 0x1000 * v
        descs.append(d)
    return descs


def build_status(descs, ext=(0x1000,)):
    try:
        dag = B.opara_build_dag(descs, list(ext))
    except B.OparaError as e:
        return e.status, str(e)
    B.opara_dag_destroy(dag)
    return B.OK, ""


def test_error_paths():
    assert build_status(chain_descs(3, [[-1], [0], [1]]))[0] == B.OK
    st, msg = build_status(chain_descs(3, [[2], [0], [1]]))
    assert st == B.ECYCLE and "cycle" in msg
    assert build_status(chain_descs(2, [[-1], [1]]))[0] == B.ECYCLE          # self-loop
    assert build_status(chain_descs(2, [[-1], [5]]))[0] == B.EINVAL          # producer out of range
    assert build_status(chain_descs(2, [[-2], [0]]))[0] == B.EINVAL          # external slot out of range
    assert build_status([])[0] == B.EINVAL                                   # n_ops == 0
    d = chain_descs(1, [[-1]]); d[0].n_inputs = 0
    assert build_status(d)[0] == B.EINVAL
    d = chain_descs(1, [[-1]]); d[0].out = None
    assert build_status(d)[0] == B.EINVAL
    d = chain_descs(1, [[-1]]); d[0].op_type = 99
    assert build_status(d)[0] == B.EINVAL
    d = chain_descs(1, [[-1]]); d[0].params.m = 0
    assert build_status(d)[0] == B.EINVAL
    lib = B.load()
    assert lib.opara_build_dag(None, 1, None, 0, None, None) == B.EINVAL
    assert lib.opara_assign_streams(None, None, None) == B.EINVAL
    assert lib.opara_replay(None, None) == B.EINVAL
    # calls out of order
    dag = B.opara_build_dag(chain_descs(2, [[-1], [0]]), [0x1000])
    with pytest.raises(B.OparaError) as e:
        B.opara_sync_edges(dag)
    assert e.value.status == B.ESTATE
    handles = (C.c_void_p * 1)(0x1)
    out = C.c_void_p()
    assert lib.opara_capture(dag, handles, 1, B.PARALLEL, C.byref(out)) == B.ESTATE
    assert b"opara_assign_streams" in lib.opara_last_error()
    assert lib.opara_capture(dag, handles, 1, B.FUSED, C.byref(out)) == B.ESTATE        # needs a launch queue
    assert lib.opara_capture(dag, handles, 1, 99, C.byref(out)) == B.EINVAL
    ws = C.c_uint64()
    assert lib.opara_chained_workspace_bytes(dag, C.byref(ws)) == B.OK and ws.value % 256 == 0
    assert lib.opara_capture_chained(dag, C.c_void_p(0x100000), ws.value, C.byref(out)) == B.ESTATE
    assert lib.opara_wave_of(dag, None, None) == B.EINVAL
    assert lib.opara_elide_concats(None, 1, None, 0, None, None, None, None, None) == B.EINVAL
    assert lib.opara_run_persistent_noalloc(dag, None, None) == B.ESTATE
    B.opara_dag_destroy(dag)


def test_bad_shapes_rejected():
    b = Builder("bad", "f16")
    x = b.ext((8, 6, 6))
    b.conv(x, 8, 3, pad=1)
    wl = b.build(0)
    wl.ops[0].out_shape = (8, 5, 6)          # does not match the floor formula
    with pytest.raises(B.OparaError) as e:
        Session(wl, device=None)
    assert e.value.status == B.EINVAL


def oracle_schedule(wl, dem):
    preds = sched.dedup_preds([o.inputs for o in wl.ops])
    so, ns = sched.assign_streams(preds)
    scal = [sched.demand_scalar((d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs), LIMITS) for d in dem]
    q = sched.order_launch(preds, [d.op_class for d in dem], scal)
    return preds, so, ns, q, sched.sync_edges(preds, so), scal


@pytest.mark.parametrize("builder", [inception_block, googlenet_like, inception_v3_like, bert_base_like,
                                     random_wide_dag, nasnet_like])
def test_scheduler_matches_oracle_on_configs(builder):
    wl = builder()
    s = Session(wl, device=None)
    try:
        so, ns, q, syncs = s.schedule()
        dem = B.opara_get_demands(s.dag)
        preds, oso, ons, oq, osync, scal = oracle_schedule(wl, dem)
        assert (so, ns) == (oso, ons)
        assert [d.demand for d in dem] == scal
        assert q == oq
        assert syncs == osync
        assert sched.check_schedule(preds, so, q, syncs)
        assert B.opara_wave_of(s.dag) == (sched.waves(preds), max(sched.waves(preds)) + 1)
        if builder is random_wide_dag:       # the figures the design notes quote for the 400-operator DAG
            assert (len(wl.ops), ns, len(syncs)) == (400, 182, 562)
        from oracle.executor import kahn_order
        assert B.opara_topo_order(s.dag) == kahn_order(len(wl.ops), wl.edges())
        # operator table: contractions are compute-intensive, the rest memory-intensive
        for op, d in zip(wl.ops, dem):
            assert d.op_class == (B.COMP if op.type in ("conv2d", "gemm", "bgemm") else B.MEM)
            name, vg, lds = B.opara_kernel_info(d.kernel_id)
            assert (d.vgprs, d.lds_bytes) == (vg, lds) and d.grid_blocks > 0
    finally:
        s.close()


@pytest.mark.parametrize("builder,kw", [(inception_block, {}), (googlenet_like, {}), (inception_v3_like, {}),
                                        (googlenet_like, dict(batch=2))])
def test_zero_copy_concat_dag_matches_oracle_scheduler(builder, kw):
    """Zero-copy concatenation: opara_elide_concats removes the concatenations of convolution
    branches; readers depend on the branches through dependency-only predecessors.  Which
    operators go, and the streams, launch queue and synchronisation edges of what is left,
    must be what the checker's own reading of the rewrite and the oracle scheduler give."""
    from util import expected_elision
    wl = builder(**kw)
    removed, kept, preds = expected_elision(wl)
    assert len(removed) >= 1
    s = Session(wl, device=None, zero_copy_concat=True)
    try:
        assert s.elided == removed and s.lib_ops == kept and B.opara_num_ops(s.dag) == len(kept)
        so, ns, q, syncs = s.schedule()
        dem = B.opara_get_demands(s.dag)
        oso, ons = sched.assign_streams(preds)
        scal = [sched.demand_scalar((d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs), LIMITS) for d in dem]
        oq = sched.order_launch(preds, [d.op_class for d in dem], scal)
        assert (so, ns) == (oso, ons) and q == oq and syncs == sched.sync_edges(preds, so)
        assert sched.check_schedule(preds, so, q, syncs)
        # every branch that fills a slice is a predecessor of every reader of the concatenation,
        # and writes at its channel offset with the concatenation's pixel stride
        es = 2 if wl.dtype == "f16" else 4
        for c in removed:
            base, off = s._ptr(s.out_dev[c]), 0
            for r in [op.id for op in wl.ops if c in op.inputs]:
                assert set(s.lib_id[b] for b in wl.ops[c].inputs) <= set(preds[s.lib_id[r]])
            for b_, shp in zip(wl.ops[c].inputs, wl.ops[c].in_shapes):
                d = s.descs[s.lib_id[b_]]
                assert d.out == base + off * es and d.params.c_row_stride == wl.ops[c].out_shape[0]
                off += shp[0]
    finally:
        s.close()


def test_elide_concats_leaves_other_concatenations_alone():
    """A concatenation with a pooled branch, or whose branch has a second reader, stays; a
    DAG without candidates comes back unchanged."""
    b = Builder("mixed", "f16")
    x = b.ext((16, 8, 8))
    c1, c2 = b.conv(x, 8, 1), b.conv(x, 24, 3, pad=1)
    p = b.pool("maxpool", x, 3, 1, 1)
    cat_pool = b.concat_c([c1, p])               # a pooling branch: stays
    c3, c4 = b.conv(cat_pool, 8, 1), b.conv(cat_pool, 8, 1)
    cat_ok = b.concat_c([c3, c4])                # goes
    c5 = b.conv(cat_ok, 16, 1)
    cat_shared = b.concat_c([c5, c2])            # c5 is also read by the pooling below: stays
    b.pool("avgpool", c5, 3, 1, 1)
    b.gavgpool(cat_shared)
    s = Session(b.build(3), device=None, zero_copy_concat=True)
    try:
        assert s.elided == [cat_ok]
        d = s.descs[s.lib_id[c5]]
        assert d.n_deps == 2 and [d.deps[0], d.deps[1]] == [s.lib_id[c3], s.lib_id[c4]] and d.inputs[0] < 0
    finally:
        s.close()
    s = Session(bert_base_like(layers=1), device=None, zero_copy_concat=True)
    try:
        assert s.elided == [] and s.lib_ops == list(range(14))
    finally:
        s.close()


def _capture_status(session, mode):
    """opara_capture with made-up stream handles: only what is decided before the first HIP call."""
    _, ns, _, _ = session.schedule()
    handles = (C.c_void_p * ns)(*[0x1000 + 16 * i for i in range(ns)])
    out = C.c_void_p()
    return B.load().opara_capture(session.dag, handles, ns, mode, C.byref(out)), B.opara_last_error()


@pytest.mark.parametrize("builder,zero_copy", [(googlenet_like, True), (inception_v3_like, True), (nasnet_like, False),
                                               (bert_base_like, False), (random_wide_dag, False)])
def test_stream_capture_is_refused_outside_fork_join_plans(builder, zero_copy):
    """Stream capture crashed the host process for plans whose streams wait on each other
    repeatedly (the zero-copy GoogLeNet-like chain of blocks among them); the library refuses
    those before it touches the runtime.  No GPU is needed to see the refusal."""
    s = Session(builder(), device=None, zero_copy_concat=zero_copy)
    try:
        rc, msg = _capture_status(s, B.PARALLEL_CAPTURE)
        assert rc == B.EUNSUPPORTED, (rc, msg)
        assert "fork-join" in msg or "one root and one sink" in msg
    finally:
        s.close()


def test_static_workspace_serves_512_operators():
    """The no-allocation entry point's static workspace (2.5 MiB) holds the image of 512 operators."""
    dag = B.opara_build_dag(chain_descs(512, [[-1]] + [[i] for i in range(511)]), [0x1000])
    assert B.opara_persistent_workspace_bytes(dag) <= 2560 * 1024
    B.opara_dag_destroy(dag)
    dag = B.opara_build_dag(chain_descs(600, [[-1]] + [[i] for i in range(599)]), [0x1000])
    assert B.opara_persistent_workspace_bytes(dag) > 2560 * 1024
    B.opara_dag_destroy(dag)


def test_dependency_only_predecessors_are_validated():
    descs = chain_descs(3, [[-1], [0], [-1]])
    descs[2].n_deps = 2
    descs[2].deps[0], descs[2].deps[1] = 1, 0
    dag = B.opara_build_dag(descs, [0x1000])
    so, ns = B.opara_assign_streams(dag)
    assert B.opara_topo_order(dag) == [0, 1, 2] and (so, ns) == sched.assign_streams([[], [0], [1, 0]])
    B.opara_dag_destroy(dag)
    for bad in (3, -1, 2):                      # out of range, external slot, itself
        descs[2].deps[0] = bad
        assert build_status(descs)[0] in (B.EINVAL, B.ECYCLE)
    descs[2].deps[0] = 1
    descs[2].n_deps = 9
    assert build_status(descs)[0] == B.EINVAL


def _closure(n, edges):
    r = np.zeros((n, n), dtype=bool)
    for u, v in edges:
        r[u, v] = True
    for k in range(n):
        r |= np.outer(r[:, k], r[k, :])
    return r


@pytest.mark.parametrize("builder", [inception_block, googlenet_like, inception_v3_like, bert_base_like, nasnet_like])
def test_min_streams_and_pruned_syncs_match_oracle_on_configs(builder):
    wl = builder()
    s = Session(wl, device=None)
    try:
        preds = sched.dedup_preds([o.inputs for o in wl.ops])
        n = len(preds)
        q = B.opara_order_launch(s.dag)
        for policy, oracle_fn in ((B.STREAMS_ALG1, sched.assign_streams), (B.STREAMS_MIN, sched.min_streams)):
            so, ns = B.opara_assign_streams_policy(s.dag, policy)
            oso, ons = oracle_fn(preds)
            assert ns == ons                                   # the count is unique
            if policy == B.STREAMS_ALG1:
                assert so == oso
            else:                                              # the matching is not: check it is a chain cover
                reach = _closure(n, [(u, v) for v, ps in enumerate(preds) for u in ps])
                assert sorted(set(so)) == list(range(ns))
                for st in range(ns):
                    m = [v for v in range(n) if so[v] == st]
                    assert all(reach[a, b] or reach[b, a] for a in m for b in m if a < b)
            assert B.opara_sync_edges(s.dag) == sched.sync_edges(preds, so)
            assert B.opara_sync_edges_pruned(s.dag) == sched.prune_syncs(preds, so, q)
    finally:
        s.close()


def test_min_streams_and_pruned_syncs_match_oracle_on_random_dags():
    rng = np.random.default_rng(77)
    for trial in range(300):
        n = int(rng.integers(1, 60))
        inputs = [[-1]]
        for v in range(1, n):
            k = int(rng.integers(0, 4))
            ins = [int(u) for u in rng.choice(v, size=min(k, v), replace=False)] or [-1]
            inputs.append(ins)
        dag = B.opara_build_dag(chain_descs(n, inputs), [0x1000])
        try:
            preds = sched.dedup_preds(inputs)
            pol = int(rng.integers(0, len(B.ORDER_POLICY_NAMES)))
            q = B.opara_order_launch_policy(dag, pol)
            for policy, oracle_fn in ((B.STREAMS_ALG1, sched.assign_streams), (B.STREAMS_MIN, sched.min_streams)):
                so, ns = B.opara_assign_streams_policy(dag, policy)
                assert ns == oracle_fn(preds)[1]
                assert B.opara_sync_edges_pruned(dag) == sched.prune_syncs(preds, so, q)
                assert sched.check_schedule(preds, so, q, B.opara_sync_edges(dag))
        finally:
            B.opara_dag_destroy(dag)


def test_scheduler_matches_oracle_on_random_dags():
    """>= 10^4 seeded random DAGs with n <= 12 and caller-supplied demand records."""
    rng = np.random.default_rng(20231210)
    for trial in range(10000):
        n = int(rng.integers(1, 13))
        inputs = []
        for v in range(n):
            if v == 0 or rng.random() < 0.25:
                inputs.append([-1])
            else:
                k = int(rng.integers(1, 4))
                inputs.append([int(u) for u in rng.integers(0, v, size=k)])   # repeats allowed
        descs = chain_descs(n, inputs)
        for d in descs:
            d.op_class = int(rng.integers(-1, 2))
            d.grid_blocks = int(rng.integers(1, 5))
            d.block_threads = int(rng.choice([64, 128, 256]))
            d.lds_bytes = int(rng.choice([0, 1024, 65536]))
            d.vgprs = int(rng.choice([16, 64, 128]))
        dag = B.opara_build_dag(descs, [0x1000])
        so, ns = B.opara_assign_streams(dag)
        q = B.opara_order_launch(dag)
        syncs = B.opara_sync_edges(dag)
        dem = B.opara_get_demands(dag)
        B.opara_dag_destroy(dag)
        preds = sched.dedup_preds(inputs)
        oso, ons = sched.assign_streams(preds)
        cls = [d.op_class for d in dem]
        for d, desc in zip(dem, descs):
            assert d.op_class == (desc.op_class if desc.op_class >= 0 else B.MEM)   # ADD is memory-intensive
        scal = [sched.demand_scalar((d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs), LIMITS) for d in descs]
        assert [d.demand for d in dem] == scal
        assert (so, ns) == (oso, ons), (trial, inputs)
        assert q == sched.order_launch(preds, cls, scal), (trial, inputs)
        assert syncs == sched.sync_edges(preds, oso)


def test_order_policies_match_oracle():
    rng = np.random.default_rng(99)
    for trial in range(300):
        n = int(rng.integers(1, 25))
        inputs = [[-1] if v == 0 or rng.random() < 0.3 else [int(u) for u in rng.integers(0, v, size=int(rng.integers(1, 4)))]
                  for v in range(n)]
        descs = chain_descs(n, inputs)
        for d in descs:
            d.op_class = int(rng.integers(0, 2))
            d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs = int(rng.integers(1, 4)), 256, 0, 32
        dag = B.opara_build_dag(descs, [0x1000])
        preds = sched.dedup_preds(inputs)
        cls = [d.op_class for d in descs]
        dem = [sched.demand_scalar((d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs), LIMITS) for d in descs]
        so, ns = sched.assign_streams(preds)
        B.opara_assign_streams(dag)
        for pid, name in enumerate(sched.POLICIES):
            q = B.opara_order_launch_policy(dag, pid)
            assert q == sched.order_launch_policy(preds, cls, dem, name), (trial, name, inputs)
            assert sched.check_schedule(preds, so, q, sched.sync_edges(preds, so))
        assert B.opara_order_launch_policy(dag, B.ORDER_ALG2) == B.opara_order_launch(dag)
        assert B.opara_wave_of(dag)[0] == sched.waves(preds)
        with pytest.raises(B.OparaError):
            B.opara_order_launch_policy(dag, 17)
        B.opara_dag_destroy(dag)
    assert B.ORDER_POLICY_NAMES == sched.POLICIES


def test_random_small_workloads_schedule():
    for seed in range(5):
        wl = random_small_dag(seed, n_ops=60)
        s = Session(wl, device=None)
        so, ns, q, syncs = s.schedule()
        dem = B.opara_get_demands(s.dag)
        preds, oso, ons, oq, osync, _ = oracle_schedule(wl, dem)
        assert (so, ns, q, syncs) == (oso, ons, oq, osync)
        s.close()


@pytest.mark.parametrize("builder", [inception_block, googlenet_like, bert_base_like, random_wide_dag])
def test_planner_gives_each_executor_kind_its_kernels(builder):
    """Host logic, no GPU: the graph executors' plan uses the quad-coalesced kernels for deep K and 64 x 64 tiles
    for large GEMM-shaped operands; the persistent executor's plan never does (one workgroup size, the
    fragment-loading bodies), keeps 32 x 32 tiles for them, and reports a positive tile count per operator."""
    wl = builder()
    s = Session(wl, device=None)
    try:
        dem = B.opara_get_demands(s.dag)
        tiles, kernels = B.opara_persistent_plan(s.dag)
        assert len(tiles) == len(kernels) == len(wl.ops)
        graph_names = [B.opara_kernel_info(d.kernel_id)[0] for d in dem]
        persist_names = [B.opara_kernel_info(k)[0] for k in kernels]
        assert all(t > 0 for t in tiles)
        assert not any("quad" in n for n in persist_names)
        for op, d, gname, pname, t in zip(wl.ops, dem, graph_names, persist_names, tiles):
            if not gname.startswith("igemm"):
                assert pname == gname and t == d.grid_blocks         # same kernel, same grid
            elif "quad64" in gname:                                  # 64 x 64 tiles against 32 x 32 or the tiled kernel
                assert pname.split("_")[-1] in ("direct4", "direct8", "t128x64") and t != d.grid_blocks
            elif "quad" in gname:                                    # same 32 x 32 tiles, fragment-loading body
                assert pname.split("_")[-1] in ("direct4", "direct8", "t128x64")
        if wl.name == "bert_base_like":
            assert any("quad" in n for n in graph_names)
        if wl.name == "random_wide_dag":
            assert any("quad64x4" in n for n in graph_names) and any("t128x64" in n for n in persist_names)
    finally:
        s.close()


def test_kernel_table():
    n = B.opara_kernel_count()
    names = [B.opara_kernel_info(i)[0] for i in range(n)]
    assert len(set(names)) == n and "igemm_f16_t64x64" in names
    for i in range(n):
        name, vg, lds = B.opara_kernel_info(i)
        assert 0 < vg <= 512 and lds <= 163840
        if name.startswith("igemm"):
            assert lds > 0
    with pytest.raises(B.OparaError):
        B.opara_kernel_info(n)
