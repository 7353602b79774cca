"""The C ABI from a C program (no Python, no PyTorch in the process): the demo built with the
library allocates with hipMalloc, rewrites a two-block DAG with opara_elide_concats, captures
the sequential graph, the validated multi-stream graph and the fused executor, and requires
bit-identical results from all of them."""
import os
import subprocess
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_caller_gets_identical_bits_from_every_executor():
    demo = os.path.join(ROOT, "paper_2312_10351_amd", "abi_demo")
    assert os.path.exists(demo), "run __graft_entry__.build() first"
    p = subprocess.run([demo], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert p.returncode == 0 and "abi_demo ok" in p.stdout, p.stdout
    assert "multi-stream graph" in p.stdout and "validation 2" in p.stdout, p.stdout
