"""GPU parity of the persistent executor (whole DAG in one kernel, dependencies through
completion flags in device memory) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch
from oracle import executor
from paper_2312_10351_amd import binding as B
from paper_2312_10351_amd.runtime import Session
from workloads import (Builder, inception_block, googlenet_like, inception_v3_like, bert_base_like,
                       random_wide_dag, random_small_dag)
from util import compare_all
from test_gpu_parity import run_modes

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("builder,kw", [
    (inception_block, dict(random_bias=True)), (inception_block, dict(dtype="f16", batch=3)),
    (googlenet_like, dict(he_init=True)), (inception_v3_like, dict(he_init=True)), (bert_base_like, {}),
    (googlenet_like, dict(he_init=True, batch=2))])
def test_model_configs_persistent(builder, kw):
    run_modes(builder(**kw), modes=("persist",), outlier_frac=1e-3)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_random_small_dags_persistent(seed, dtype):
    run_modes(random_small_dag(seed, dtype), modes=("persist",), outlier_frac=1e-3)


def test_random_wide_dag_persistent():
    run_modes(random_wide_dag(), modes=("persist",), outlier_frac=1e-3)


@pytest.mark.parametrize("wgs", [1, 3, 17, 100])
def test_any_number_of_workgroups(wgs):
    """Work items are dealt in a topological order, so the launch drains with any number of
    workgroups, down to one."""
    run_modes(inception_block(random_bias=True), modes=(f"persist:{wgs}",))
    run_modes(random_small_dag(3, "f16"), modes=(f"persist:{wgs}",), outlier_frac=1e-3)


def test_replays_are_identical_and_rewrite_every_output():
    wl = googlenet_like(he_init=True)
    ref = executor.run_dag(wl)
    s = Session(wl)
    try:
        exe = s.capture_persistent()
        bits = []
        for rep in range(4):
            for t in s.out_dev:
                t.fill_(float("nan"))            # a skipped tile or a read before its producer shows up as NaN
            torch.cuda.synchronize()
            s.replay(exe)
            assert s.persistent_status(exe) == 0
            assert not compare_all(s, ref, outlier_frac=1e-3)
            bits.append([t.clone().view(torch.int16) for t in s.out_dev])
        for other in bits[1:]:
            assert all(torch.equal(a, b) for a, b in zip(bits[0], other))
        # back-to-back replays without host synchronisation in between
        for _ in range(20):
            s.replay(exe, sync=False)
        s.make_streams(1).torch_streams[0].synchronize()
        assert s.persistent_status(exe) == 0
        assert all(torch.equal(a, t.view(torch.int16)) for a, t in zip(bits[0], s.out_dev))
        prefix = B.opara_persistent_prefix(exe)               # ordinary kernel nodes in a chain, then the one kernel
        assert B.opara_exec_info(exe) == (prefix + 1, prefix)
        items, wgs = B.opara_persistent_info(exe)
        tiles, _ = B.opara_persistent_plan(s.dag)
        # an operator with more tiles than workgroups runs ceil(tiles / workgroups) tiles per item;
        # every operator's item range is padded to the XCD count
        order = B.opara_order_launch_policy(s.dag, B.ORDER_ALG2)
        inside = order[B.opara_persistent_prefix(exe):]      # the serial prefix runs as ordinary kernel nodes
        per_op = [-(-tiles[v] // -(-tiles[v] // wgs)) for v in inside]
        assert items == sum((i + 7) // 8 * 8 for i in per_op) and 1 <= wgs <= items
    finally:
        s.close()


def test_all_launch_orders_persistent():
    """Any topological queue is a valid work-item order (Alg. 2 is only the default)."""
    wl = random_small_dag(1, "f32", n_ops=60, max_width=8)
    ref = executor.run_dag(wl)
    s = Session(wl)
    try:
        for pol in range(len(B.ORDER_POLICY_NAMES)):
            exe = s.capture_persistent(policy=pol)
            for t in s.out_dev:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            s.replay(exe)
            assert s.persistent_status(exe) == 0
            assert not compare_all(s, ref), B.ORDER_POLICY_NAMES[pol]
    finally:
        s.close()


def test_bounded_wait_reports_and_recovers():
    """Failure handling: with a spin limit of one poll the waits run out; every workgroup
    leaves, the error word names a queue position, and after a reset the executor is
    usable again.  The kernel exits normally in both cases."""
    wl = googlenet_like(he_init=True)
    ref = executor.run_dag(wl)
    s = Session(wl)
    try:
        exe = s.capture_persistent()
        s.persistent_reset(exe, spin_limit=1)
        s.replay(exe)
        word = s.persistent_status(exe)
        assert 1 <= word <= len(wl.ops)
        s.replay(exe)                                  # sticky: the word stays set (any wait that ran out may name itself)
        assert 1 <= s.persistent_status(exe) <= len(wl.ops)
        s.persistent_reset(exe)
        for t in s.out_dev:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        s.replay(exe)
        assert s.persistent_status(exe) == 0
        assert not compare_all(s, ref, outlier_frac=1e-3)
    finally:
        s.close()


def test_timeline_is_consistent_with_the_dag():
    """The in-kernel timeline covers every tile once, and no tile of an operator became
    ready before all tiles of each predecessor had started and (up to the delay between a
    publication and its time stamp) finished."""
    wl = inception_v3_like()
    s = Session(wl)
    try:
        exe = s.capture_persistent()
        s.replay(exe)
        tr = s.persistent_trace(exe)
        assert s.persistent_status(exe) == 0
        order = B.opara_order_launch_policy(s.dag, B.ORDER_ALG2)
        pos_of = {v: i for i, v in enumerate(order)}
        plan_tiles, _ = B.opara_persistent_plan(s.dag)
        _, wgs = B.opara_persistent_info(exe)
        assert np.all(tr[:, 0] <= tr[:, 1]) and np.all(tr[:, 1] <= tr[:, 2])
        first_ready, last_start, last_end = {}, {}, {}
        prefix = B.opara_persistent_prefix(exe)
        assert not np.any(tr[:, 3] < prefix)
        for p in range(prefix, len(order)):
            m = tr[:, 3] == p
            tiles = plan_tiles[order[p]]
            assert m.sum() == -(-tiles // -(-tiles // wgs))            # items = ceil(tiles / chunk)
            first_ready[p], last_start[p], last_end[p] = tr[m, 1].min(), tr[m, 1].max(), tr[m, 2].max()
        stamp_delay_ns = 3000
        for u, v in wl.edges():
            if pos_of[u] < prefix:         # a kernel node ahead of the persistent kernel: complete before it starts
                continue
            assert first_ready[pos_of[v]] >= last_start[pos_of[u]]
            assert first_ready[pos_of[v]] + stamp_delay_ns >= last_end[pos_of[u]]
    finally:
        s.close()


def test_serial_prefix_runs_as_kernel_nodes(monkeypatch):
    """The stem of a network (operators every other operator depends on) is launched as ordinary kernel nodes
    ahead of the persistent kernel; DAGs that start with a fork have no such prefix; the switch keeps everything
    inside the kernel.  Results hold either way."""
    expect = {"googlenet_like": 5, "inception_block": 0, "bert_base_like": 0}
    for make in (lambda: googlenet_like(he_init=True), inception_block, lambda: bert_base_like(layers=2)):
        wl = make()
        ref = executor.run_dag(wl)
        for switch in ("1", "0"):
            monkeypatch.setenv("OPARA_PERSIST_SERIAL_PREFIX", switch)
            s = Session(wl)
            try:
                exe = s.capture_persistent()
                prefix = B.opara_persistent_prefix(exe)
                assert prefix == (expect[wl.name] if switch == "1" else 0), (wl.name, switch, prefix)
                assert B.opara_exec_info(exe) == (prefix + 1, prefix)
                for t in s.out_dev:
                    t.fill_(float("nan"))
                torch.cuda.synchronize()
                s.replay(exe)
                assert s.persistent_status(exe) == 0
                assert not compare_all(s, ref, outlier_frac=1e-3)
            finally:
                s.close()


def test_kernel_alone_can_be_timed():
    """The measurement aid launches the persistent kernel by itself: plausible time, no error, same outputs."""
    wl = googlenet_like(he_init=True)
    s = Session(wl)
    try:
        exe = s.capture_persistent()
        s.replay(exe)
        before = [t.clone() for t in s.out_dev]
        h = s.make_streams(1).handles[0]
        us = B.opara_persistent_time_kernel(exe, h, 5)
        assert 20.0 < us < 5000.0
        assert s.persistent_status(exe) == 0
        assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(before, s.out_dev))
        s.replay(exe)                                       # the graph still replays after the ordinary launches
        assert s.persistent_status(exe) == 0
        assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(before, s.out_dev))
    finally:
        s.close()


def test_persistent_rejects_bad_arguments():
    wl = inception_block()
    s = Session(wl)
    try:
        B.opara_order_launch_policy(s.dag, B.ORDER_ALG2)
        need = B.opara_persistent_workspace_bytes(s.dag)
        ws = torch.zeros(need + 256, dtype=torch.uint8, device="cuda")
        ptr = (ws.data_ptr() + 255) // 256 * 256
        with pytest.raises(B.OparaError):
            B.opara_capture_persistent(s.dag, ptr, need - 1)
        with pytest.raises(B.OparaError):
            B.opara_capture_persistent(s.dag, ptr + 4, need)
        seq = s.capture(B.SEQUENTIAL)
        with pytest.raises(B.OparaError):
            B.opara_persistent_status(seq, s.make_streams(1).handles[0])
    finally:
        s.close()
