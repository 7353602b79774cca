"""Shared helpers for the tests: tolerances and oracle-vs-library comparison."""
import numpy as np

LIMITS = dict(threads_per_cu=2048, lds_bytes_per_cu=163840, vgpr_lanes_per_cu=4 * 512 * 64)


def tolerance(dtype, ref):
    """(rtol, atol) for one operator output `ref` (fp64 view of the oracle result).

    fp32: relative 1e-4 plus 1e-6 of the tensor's largest magnitude, so that exact
    zeros after ReLU are well defined.  fp16: relative 2e-2 plus absolute 1e-2 times
    the tensor's RMS (the absolute error of a sum of rounded terms follows the size of
    the terms, not of the result), floored at two fp16 subnormal steps.  For tensors of
    RMS <= 1 this is never looser than the plain 2e-2 / 1e-2 bound."""
    if dtype == "f32":
        scale = float(np.abs(ref).max()) if ref.size else 0.0
        return 1e-4, 1e-6 * scale + 1e-30
    rms = float(np.sqrt(np.mean(np.square(ref)))) if ref.size else 0.0
    return 2e-2, 1e-2 * rms + 2.0 ** -23


def literal_fp16_bound_ok(got, ref):
    """The plain bound |g - o| <= 1e-2 + 2e-2 |o|."""
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(ref, dtype=np.float64)
    return bool((np.abs(g - o) <= 1e-2 + 2e-2 * np.abs(o)).all())


def literal_fp16_miss_fraction(got, ref):
    """Share of elements outside the plain bound |g - o| <= 1e-2 + 2e-2 |o|."""
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(ref, dtype=np.float64)
    return float((np.abs(g - o) > 1e-2 + 2e-2 * np.abs(o)).mean()) if o.size else 0.0


def mismatch(got, ref, dtype, outlier_frac=0.0):
    """None if `got` matches the oracle `ref` within tolerance, else a description.
    outlier_frac: share of elements that may miss the scale-aware bound as long as they
    still meet the plain fp16 bound (for ill-conditioned chains, e.g. a softmax fed by
    large fp16 values, where one storage rounding upstream moves a result by percents)."""
    g = np.asarray(got, dtype=np.float64)
    o = np.asarray(ref, dtype=np.float64)
    if g.shape != o.shape:
        return f"shape {g.shape} vs {o.shape}"
    if not np.isfinite(g).all():
        return "non-finite values"
    rtol, atol = tolerance(dtype, o)
    err = np.abs(g - o)
    bad = err > atol + rtol * np.abs(o)
    if bad.any():
        if dtype == "f16" and bad.sum() <= outlier_frac * o.size and literal_fp16_bound_ok(g, o):
            return None
        i = np.unravel_index(np.argmax(err - (atol + rtol * np.abs(o))), o.shape)
        return (f"{int(bad.sum())} of {o.size} outside tolerance; worst at {i}: got {g[i]!r}, "
                f"oracle {o[i]!r}, max|oracle| {np.abs(o).max():.3g}")
    return None


def compare_all(session, ref, ops=None, outlier_frac=0.0):
    """Compare every operator output of a Session with the oracle's dict."""
    wl = session.wl
    problems = []
    for op in wl.ops:
        if ops is not None and op.id not in ops:
            continue
        m = mismatch(session.output(op.id), ref[op.id], wl.dtype, outlier_frac)
        if m:
            problems.append(f"op {op.id} {op.name} ({op.type}): {m}")
    return problems


def expected_elision(wl, max_deps=8):
    """The checker's own reading of the zero-copy rewrite, written from its definition in
    opara.h: a channel concatenation goes when each input is the whole output of a distinct
    convolution that nothing else reads.  Returns (removed, kept, preds): the removed
    concatenation ids, the surviving workload ids in order, and for every survivor its
    predecessors in reduced numbering (operator arguments, then the branches standing in for
    each removed concatenation in argument order, no repeats)."""
    readers = {}
    for op in wl.ops:
        for u in op.inputs:
            if u >= 0:
                readers[u] = readers.get(u, 0) + 1
    removed = set()
    for op in wl.ops:
        if op.type != "concat" or op.params.get("axis") != 0:
            continue
        if all(u >= 0 and wl.ops[u].type == "conv2d" and readers[u] == 1 and tuple(wl.ops[u].out_shape) == tuple(s)
               for u, s in zip(op.inputs, op.in_shapes)):
            removed.add(op.id)
    for op in wl.ops:       # a reader must have room for the branches in its dependency list
        extra = sum(len(wl.ops[u].inputs) for u in op.inputs if u in removed)
        assert extra <= max_deps, "the test DAGs stay within the dependency list"
    kept = [op.id for op in wl.ops if op.id not in removed]
    number = {v: i for i, v in enumerate(kept)}
    preds = []
    for v in kept:
        row = []
        for u in wl.ops[v].inputs:
            if u >= 0 and u not in removed and number[u] not in row:
                row.append(number[u])
        for u in wl.ops[v].inputs:
            if u in removed:
                row += [number[b] for b in wl.ops[u].inputs if number[b] not in row]
        preds.append(row)
    return sorted(removed), kept, preds
