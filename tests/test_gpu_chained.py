"""GPU parity of the chained executor (the whole DAG as one loop-free launch: one tile per
workgroup, blocks in launch-queue order, dependencies through completion flags) against the
CPU oracle, through the C ABI; its failure handling and its timeline."""
import numpy as np
import pytest
import torch
from oracle import executor
from paper_2312_10351_amd import binding as B
from paper_2312_10351_amd.runtime import Session
from workloads import (inception_block, googlenet_like, inception_v3_like, bert_base_like, random_wide_dag,
                       random_small_dag)
from util import compare_all
from test_gpu_parity import run_modes

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("builder,kw", [
    (inception_block, dict(random_bias=True)), (inception_block, dict(dtype="f16", batch=3)),
    (googlenet_like, dict(he_init=True)), (inception_v3_like, dict(he_init=True)), (bert_base_like, {}),
    (googlenet_like, dict(he_init=True, batch=2))])
def test_model_configs_chained(builder, kw):
    run_modes(builder(**kw), modes=("chain",), outlier_frac=1e-3)


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_random_small_dags_chained(seed, dtype):
    run_modes(random_small_dag(seed, dtype), modes=("chain",), outlier_frac=1e-3)


def test_random_wide_dag_chained():
    """313,200 workgroups in one launch, far more than the device holds at once: the launch
    drains because blocks are dispatched in order and predecessors come first."""
    run_modes(random_wide_dag(), modes=("chain",), outlier_frac=1e-3)


def test_replays_are_identical_under_every_launch_order_and_beside_other_work():
    wl = googlenet_like(he_init=True)
    ref = executor.run_dag(wl)
    s = Session(wl, zero_copy_concat=True)
    try:
        side = torch.cuda.Stream()
        a = torch.randn(4096, 4096, device="cuda", dtype=torch.float16)
        first = None
        for pol in range(len(B.ORDER_POLICY_NAMES)):
            exe = s.capture_chained(policy=pol)
            prefix = B.opara_persistent_prefix(exe)
            assert B.opara_exec_info(exe) == (prefix + 1, prefix) and prefix == 5
            items, wgs = B.opara_persistent_info(exe)
            assert items == wgs and items % 8 == 0
            for rep in range(3):
                for t in s.out_dev:
                    t.fill_(float("nan"))        # a skipped tile or a read before its producer shows up as NaN
                torch.cuda.synchronize()
                if rep == 2:                     # other kernels hold compute units meanwhile: no residency assumption
                    with torch.cuda.stream(side):
                        for _ in range(4):
                            a @ a
                s.replay(exe)
                torch.cuda.synchronize()
                assert s.persistent_status(exe) == 0
                assert not compare_all(s, ref, outlier_frac=1e-3)
                bits = [s.output(v).tobytes() for v in range(len(wl.ops))]
                assert first is None or bits == first, B.ORDER_POLICY_NAMES[pol]
                first = bits
        for _ in range(20):                      # back to back, no host synchronisation in between
            s.replay(exe, sync=False)
        torch.cuda.synchronize()
        assert s.persistent_status(exe) == 0
        assert [s.output(v).tobytes() for v in range(len(wl.ops))] == first
        us = B.opara_persistent_time_kernel(exe, s.make_streams(1).handles[0], 5)
        assert 20.0 < us < 5000.0 and s.persistent_status(exe) == 0
    finally:
        s.close()


def test_bounded_wait_reports_and_recovers_chained():
    """With a spin limit of one poll the waits run out: every workgroup leaves, the error word
    names a queue position, and after a reset the executor works again.  The kernel exits
    normally in both cases."""
    wl = googlenet_like(he_init=True)
    ref = executor.run_dag(wl)
    s = Session(wl)
    try:
        exe = s.capture_chained()
        s.persistent_reset(exe, spin_limit=1)
        s.replay(exe)
        assert 1 <= s.persistent_status(exe) <= len(wl.ops)
        s.replay(exe)                                  # sticky
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


def test_timeline_of_the_chained_executor_is_consistent_with_the_dag():
    """One stamp record per block; no tile became ready before every tile of each predecessor
    had started and (up to the delay between a publication and its time stamp) finished."""
    wl = inception_v3_like()
    s = Session(wl)
    try:
        exe = s.capture_chained()
        s.replay(exe)
        tr = s.persistent_trace(exe)
        assert s.persistent_status(exe) == 0
        order = B.opara_order_launch_policy(s.dag, B.ORDER_ALG2)
        pos_of = {v: i for i, v in enumerate(order)}
        prefix = B.opara_persistent_prefix(exe)
        assert np.all(tr[:, 0] <= tr[:, 1]) and np.all(tr[:, 1] <= tr[:, 2]) and not np.any(tr[:, 3] < prefix)
        first_ready, last_start, last_end = {}, {}, {}
        for p in range(prefix, len(order)):
            m = tr[:, 3] == p
            assert m.sum() >= 1
            first_ready[p], last_start[p], last_end[p] = tr[m, 1].min(), tr[m, 1].max(), tr[m, 2].max()
        for u, v in wl.edges():
            if pos_of[u] < prefix:
                continue
            assert first_ready[pos_of[v]] >= last_start[pos_of[u]]
            assert first_ready[pos_of[v]] + 3000 >= last_end[pos_of[u]]
    finally:
        s.close()


def test_chained_rejects_bad_arguments():
    s = Session(inception_block())
    try:
        B.opara_order_launch_policy(s.dag, B.ORDER_ALG2)
        need = B.opara_chained_workspace_bytes(s.dag)
        ws = torch.zeros(need + 256, dtype=torch.uint8, device="cuda")
        ptr = (ws.data_ptr() + 255) // 256 * 256
        with pytest.raises(B.OparaError):
            B.opara_capture_chained(s.dag, ptr, need - 1)
        with pytest.raises(B.OparaError):
            B.opara_capture_chained(s.dag, ptr + 4, need)
    finally:
        s.close()
