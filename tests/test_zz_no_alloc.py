"""The entry point for callers that cannot allocate (opara_run_persistent_noalloc): its
results against the existing persistent executor (opara_capture_persistent + opara_replay)
on the same DAG, bit for bit, on two calls in a row, the second on a smaller DAG."""
import numpy as np
import pytest
import torch
from oracle import executor
from paper_2312_10351_amd import binding as B
from paper_2312_10351_amd.runtime import Session
from workloads import googlenet_like, inception_block, random_small_dag
from util import compare_all

pytestmark = pytest.mark.gpu


def outputs(session):
    return [session.output(op.id).tobytes() for op in session.wl.ops]


@pytest.mark.parametrize("first,second", [
    (lambda: googlenet_like(he_init=True), lambda: inception_block(dtype="f16", random_bias=True)),
    (lambda: random_small_dag(3, "f32", n_ops=60, max_width=8), lambda: inception_block(random_bias=True))])
def test_no_alloc_entry_point_matches_the_persistent_executor(first, second):
    big, small = Session(first()), Session(second())
    try:
        want = {}
        for s in (big, small):                      # the existing entry point, caller-owned workspace
            exe = s.capture_persistent()
            s.clear_outputs()
            s.replay(exe)
            assert s.persistent_status(exe) == 0
            want[s] = outputs(s)
            assert not compare_all(s, executor.run_dag(s.wl), outlier_frac=1e-3)
        for rep in range(2):                        # two calls in a row, the second with the smaller DAG
            for s in (big, small):
                s.clear_outputs()
                assert s.run_persistent_noalloc() == 0
                torch.cuda.synchronize()
                assert outputs(s) == want[s], (s.wl.name, rep)
    finally:
        big.close()
        small.close()


def test_no_alloc_entry_point_rejects_what_does_not_fit():
    from workloads import Builder
    b = Builder("long_chain", "f16")
    x = b.ext((4, 64))
    for _ in range(513):
        x = b.rowwise("relu", [x], 4, 64)
    s = Session(b.build(1))
    try:
        with pytest.raises(B.OparaError) as e:
            s.run_persistent_noalloc()
        assert e.value.status == B.EUNSUPPORTED and "512" in str(e.value)
    finally:
        s.close()
