"""Builds libopara.so in-tree with hipcc for gfx950.

Two steps: (1) compile the kernel translation unit and turn the compiler's
per-kernel resource report (vector registers, accumulation registers, LDS) into
csrc/_build/kernel_resources.inc; (2) compile the host-side scheduler/planner against
that table and link everything into one shared library.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libopara.so")
DEMO = os.path.join(HERE, "abi_demo")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"
COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(HERE, "..", "include"), "-I", BUILD, "-I", CSRC]
HIPFLAGS = [f"--offload-arch={ARCH}", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stdout + p.stderr)
        raise RuntimeError("command failed: " + " ".join(cmd))
    return p.stderr


def kernel_names():
    text = open(os.path.join(CSRC, "kernel_args.h")).read()
    block = text[text.index("#define OPARA_KERNEL_LIST(X)"):text.index("enum KernelId")]
    return re.findall(r"X\((\w+),", block)[0:]


def parse_resources(report):
    """Compiler remarks -> {kernel: (vgprs, agprs, lds_bytes)}."""
    out, cur = {}, None
    for line in report.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = m.group(1)
            out.setdefault(cur, {})
            continue
        for key, tag in (("VGPRs", "vgprs"), ("AGPRs", "agprs"), (r"LDS Size \[bytes/block\]", "lds")):
            m = re.search(r"remark:\s+" + key + r": (\d+)", line)
            if m and cur:
                out[cur][tag] = int(m.group(1))
    return out


def build(verbose=False):
    os.makedirs(BUILD, exist_ok=True)
    k_obj = os.path.join(BUILD, "kernels.o")
    g_obj = os.path.join(BUILD, "graph.o")
    names = kernel_names()
    with ThreadPoolExecutor(2) as ex:
        f1 = ex.submit(_run, [HIPCC, *HIPFLAGS, *COMMON, "-Rpass-analysis=kernel-resource-usage",
                              "-c", os.path.join(CSRC, "kernels.hip"), "-o", k_obj])
        f2 = ex.submit(_run, [HIPCC, *HIPFLAGS, *COMMON, "-c", os.path.join(CSRC, "graph.hip"), "-o", g_obj])
        report = f1.result()
        f2.result()
    res = parse_resources(report)
    lines = []
    for n in names:
        r = res.get("opara_k_" + n)
        if not r or not {"vgprs", "agprs", "lds"} <= set(r):
            raise RuntimeError(f"no resource report for kernel {n}")
        lines.append(f'{{"{n}", {r["vgprs"]}u, {r["agprs"]}u, {r["lds"]}u}},')
    inc = os.path.join(BUILD, "kernel_resources.inc")
    new = "\n".join(lines) + "\n"
    if not os.path.exists(inc) or open(inc).read() != new:
        open(inc, "w").write(new)
    objs = [k_obj, g_obj]
    for src in ("sched.cpp", "plan.cpp", "rewrite.cpp"):
        o = os.path.join(BUILD, src.replace(".cpp", ".o"))
        _run([HIPCC, "-x", "c++", *COMMON, "-Wall", "-c", os.path.join(CSRC, src), "-o", o])
        objs.append(o)
    _run([HIPCC, f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", LIB, *objs])
    # A plain C caller of the ABI (no Python, no PyTorch), run by the GPU tests.
    _run(["gcc", "-O1", "-std=c11", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(HERE, "..", "include"),
          "-I", "/opt/rocm/include", os.path.join(CSRC, "abi_demo.c"), "-o", DEMO, "-L", HERE, "-lopara",
          "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib"])
    if verbose:
        for n in names:
            print(n, res["opara_k_" + n])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
