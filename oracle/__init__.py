"""CPU oracle: TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct reference for what the operator-parallel DAG
executor computes: every operator by its textbook definition in fp64 (ops.py,
executor.py) and the paper's two scheduling algorithms step by step (sched.py).
It shares no code with the HIP path and must never be imported by the product
package; only tests, the smoke check and the benchmark's cpu_baseline leg use it.
"""
