"""ctypes binding of include/opara.h: same names, argument marshalling only."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libopara.so")
MAX_INPUTS = 8

OK, EINVAL, ECYCLE, ENOMEM, ESTATE, EHIP, EUNSUPPORTED, EGRAPH = 0, -1, -2, -3, -4, -5, -6, -7
NOT_VALIDATED, SCREENED_ON_TWIN, VALIDATED_IN_PLACE = 0, 1, 2
(CONV2D, GEMM, BGEMM, MAXPOOL, AVGPOOL, GAVGPOOL, CONCAT, LAYERNORM, SOFTMAX, GELU, RELU,
 ADD) = range(12)
OP_TYPE_IDS = dict(conv2d=CONV2D, gemm=GEMM, bgemm=BGEMM, maxpool=MAXPOOL, avgpool=AVGPOOL,
                   gavgpool=GAVGPOOL, concat=CONCAT, layernorm=LAYERNORM, softmax=SOFTMAX,
                   gelu=GELU, relu=RELU, add=ADD)
CLASS_DEFAULT, MEM, COMP = -1, 0, 1
F32, F16 = 0, 1
PARALLEL, SEQUENTIAL, PARALLEL_CAPTURE, PARALLEL_PRUNED, FUSED = 0, 1, 2, 3, 4
STREAMS_ALG1, STREAMS_MIN = 0, 1
FLAG_RELU, FLAG_B_KMAJOR = 1, 2
(ORDER_ALG2, ORDER_ALG2_COMP_FIRST, ORDER_LEAST_DEMAND, ORDER_MOST_DEMAND, ORDER_TOPO,
 ORDER_LEVEL) = range(6)
ORDER_POLICY_NAMES = ("alg2", "alg2_comp_first", "least_demand", "most_demand", "topo", "level")


class OparaError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"opara status {status}: {text}")
        self.status = status


class Limits(C.Structure):
    _fields_ = [("num_cus", C.c_uint32), ("threads_per_cu", C.c_uint32),
                ("lds_bytes_per_cu", C.c_uint32), ("vgpr_lanes_per_cu", C.c_uint32)]


class OpParams(C.Structure):
    _fields_ = [("h_in", C.c_int32), ("w_in", C.c_int32), ("c_in", C.c_int32),
                ("h_out", C.c_int32), ("w_out", C.c_int32), ("c_out", C.c_int32),
                ("kh", C.c_int32), ("kw", C.c_int32), ("sh", C.c_int32), ("sw", C.c_int32),
                ("ph", C.c_int32), ("pw", C.c_int32),
                ("m", C.c_int32), ("n", C.c_int32), ("k", C.c_int32), ("batch", C.c_int32),
                ("a_batch_stride", C.c_int64), ("a_row_stride", C.c_int64),
                ("b_batch_stride", C.c_int64), ("b_row_stride", C.c_int64),
                ("c_batch_stride", C.c_int64), ("c_row_stride", C.c_int64),
                ("in_cols", C.c_int32 * MAX_INPUTS),
                ("alpha", C.c_float), ("eps", C.c_float), ("flags", C.c_uint32)]


class OpDesc(C.Structure):
    _fields_ = [("op_type", C.c_int32), ("op_class", C.c_int32), ("dtype", C.c_int32),
                ("n_inputs", C.c_int32), ("inputs", C.c_int32 * MAX_INPUTS),
                ("grid_blocks", C.c_uint32), ("block_threads", C.c_uint32),
                ("lds_bytes", C.c_uint32), ("vgprs", C.c_uint32),
                ("params", OpParams),
                ("weight", C.c_void_p), ("bias", C.c_void_p), ("out", C.c_void_p),
                ("n_deps", C.c_int32), ("deps", C.c_int32 * MAX_INPUTS)]


class Demand(C.Structure):
    _fields_ = [("grid_blocks", C.c_uint32), ("block_threads", C.c_uint32),
                ("lds_bytes", C.c_uint32), ("vgprs", C.c_uint32),
                ("op_class", C.c_int32), ("kernel_id", C.c_int32), ("demand", C.c_uint64)]


EXPORTS = ["opara_build_dag", "opara_elide_concats", "opara_assign_streams", "opara_assign_streams_policy", "opara_order_launch",
           "opara_order_launch_policy", "opara_sync_edges", "opara_sync_edges_pruned",
           "opara_get_demands", "opara_wave_of", "opara_topo_order", "opara_num_ops", "opara_capture",
           "opara_persistent_workspace_bytes", "opara_capture_persistent", "opara_persistent_status",
           "opara_persistent_reset", "opara_persistent_info", "opara_persistent_plan", "opara_persistent_prefix", "opara_persistent_time_kernel",
           "opara_persistent_set_trace",
           "opara_run_persistent_noalloc", "opara_chained_workspace_bytes", "opara_capture_chained",
           "opara_replay", "opara_verify_dependencies", "opara_exec_info", "opara_exec_validation", "opara_set_operator_trace", "opara_fused_plan", "opara_fused_time_nodes", "opara_launch_op", "opara_run_eager",
           "opara_kernel_count", "opara_kernel_info", "opara_kernel_device_attrs",
           "opara_exec_destroy", "opara_dag_destroy", "opara_last_error"]

_lib = None


def load():
    """Load libopara.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.opara_build_dag.argtypes = [C.POINTER(OpDesc), C.c_int32, C.POINTER(C.c_void_p), C.c_int32,
                                    C.POINTER(Limits), C.POINTER(vp)]
    lib.opara_elide_concats.argtypes = [C.POINTER(OpDesc), C.c_int32, C.POINTER(C.c_void_p), C.c_int32,
                                        C.POINTER(OpDesc), i32p, i32p, C.POINTER(C.c_void_p), i32p]
    lib.opara_assign_streams.argtypes = [vp, i32p, i32p]
    lib.opara_assign_streams_policy.argtypes = [vp, C.c_int32, i32p, i32p]
    lib.opara_sync_edges_pruned.argtypes = [vp, i32p, C.c_int32, i32p]
    lib.opara_order_launch.argtypes = [vp, i32p]
    lib.opara_order_launch_policy.argtypes = [vp, C.c_int32, i32p]
    lib.opara_sync_edges.argtypes = [vp, i32p, C.c_int32, i32p]
    lib.opara_get_demands.argtypes = [vp, C.POINTER(Demand)]
    lib.opara_wave_of.argtypes = [vp, i32p, i32p]
    lib.opara_topo_order.argtypes = [vp, i32p]
    lib.opara_num_ops.argtypes = [vp]
    lib.opara_capture.argtypes = [vp, C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.POINTER(vp)]
    lib.opara_replay.argtypes = [vp, vp]
    lib.opara_persistent_workspace_bytes.argtypes = [vp, C.POINTER(C.c_uint64)]
    lib.opara_capture_persistent.argtypes = [vp, vp, C.c_uint64, C.c_int32, C.POINTER(vp)]
    lib.opara_persistent_status.argtypes = [vp, vp, C.POINTER(C.c_uint32)]
    lib.opara_chained_workspace_bytes.argtypes = [vp, C.POINTER(C.c_uint64)]
    lib.opara_capture_chained.argtypes = [vp, vp, C.c_uint64, C.POINTER(vp)]
    lib.opara_persistent_reset.argtypes = [vp, vp, C.c_uint32]
    lib.opara_persistent_info.argtypes = [vp, i32p, i32p]
    lib.opara_persistent_plan.argtypes = [vp, i32p, i32p]
    lib.opara_persistent_prefix.argtypes = [vp, i32p]
    lib.opara_persistent_time_kernel.argtypes = [vp, vp, C.c_int32, C.POINTER(C.c_float)]
    lib.opara_persistent_set_trace.argtypes = [vp, vp, vp, C.c_uint64]
    lib.opara_verify_dependencies.argtypes = [vp, vp, i32p]
    lib.opara_exec_info.argtypes = [vp, i32p, i32p]
    lib.opara_exec_validation.argtypes = [vp, i32p, i32p]
    lib.opara_set_operator_trace.argtypes = [vp]
    lib.opara_fused_plan.argtypes = [vp, i32p, i32p, i32p]
    lib.opara_fused_time_nodes.argtypes = [vp, vp, C.c_int32, C.POINTER(C.c_float)]
    lib.opara_run_persistent_noalloc.argtypes = [vp, vp, C.POINTER(C.c_uint32)]
    lib.opara_launch_op.argtypes = [vp, C.c_int32, vp]
    lib.opara_run_eager.argtypes = [vp, vp]
    lib.opara_kernel_count.argtypes = []
    lib.opara_kernel_info.argtypes = [C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.opara_kernel_device_attrs.argtypes = [C.c_int32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.opara_exec_destroy.argtypes = [vp]
    lib.opara_exec_destroy.restype = None
    lib.opara_dag_destroy.argtypes = [vp]
    lib.opara_dag_destroy.restype = None
    lib.opara_last_error.argtypes = []
    lib.opara_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc):
    if rc != OK:
        raise OparaError(rc, load().opara_last_error().decode())


def opara_last_error():
    return load().opara_last_error().decode()


def opara_build_dag(descs, ext_ptrs, limits=None):
    """descs: list[OpDesc]; ext_ptrs: list[int] device addresses.  Returns the dag handle."""
    arr = (OpDesc * max(len(descs), 1))(*descs)
    ext = (C.c_void_p * max(len(ext_ptrs), 1))(*ext_ptrs)
    out = C.c_void_p()
    lim = C.byref(limits) if limits is not None else None
    _check(load().opara_build_dag(arr, len(descs), ext, len(ext_ptrs), lim, C.byref(out)))
    return out


def opara_elide_concats(descs, ext_ptrs):
    """Zero-copy concatenation rewrite.  Returns (reduced descs, new_id per operator (-1 = removed),
    external pointers of the reduced list)."""
    n = len(descs)
    arr = (OpDesc * max(n, 1))(*descs)
    ext = (C.c_void_p * max(len(ext_ptrs), 1))(*ext_ptrs)
    out = (OpDesc * max(n, 1))()
    new_id = (C.c_int32 * max(n, 1))()
    ext_out = (C.c_void_p * (len(ext_ptrs) + max(n, 1)))()
    n_out, n_ext_out = C.c_int32(), C.c_int32()
    _check(load().opara_elide_concats(arr, n, ext, len(ext_ptrs), out, C.byref(n_out), new_id, ext_out,
                                      C.byref(n_ext_out)))
    reduced = []
    for i in range(n_out.value):
        d = OpDesc()
        C.memmove(C.byref(d), C.byref(out[i]), C.sizeof(OpDesc))
        reduced.append(d)
    return reduced, list(new_id)[:n], [ext_out[i] or 0 for i in range(n_ext_out.value)]


def opara_num_ops(dag):
    return load().opara_num_ops(dag)


def opara_assign_streams(dag):
    n = opara_num_ops(dag)
    so = (C.c_int32 * n)()
    ns = C.c_int32()
    _check(load().opara_assign_streams(dag, so, C.byref(ns)))
    return list(so), ns.value


def opara_assign_streams_policy(dag, policy):
    n = opara_num_ops(dag)
    so = (C.c_int32 * n)()
    ns = C.c_int32()
    _check(load().opara_assign_streams_policy(dag, policy, so, C.byref(ns)))
    return list(so), ns.value


def opara_order_launch(dag):
    n = opara_num_ops(dag)
    q = (C.c_int32 * n)()
    _check(load().opara_order_launch(dag, q))
    return list(q)


def opara_order_launch_policy(dag, policy):
    n = opara_num_ops(dag)
    q = (C.c_int32 * n)()
    _check(load().opara_order_launch_policy(dag, policy, q))
    return list(q)


def opara_sync_edges(dag):
    ne = C.c_int32()
    _check(load().opara_sync_edges(dag, None, 0, C.byref(ne)))
    uv = (C.c_int32 * max(2 * ne.value, 1))()
    _check(load().opara_sync_edges(dag, uv, ne.value, C.byref(ne)))
    return [(uv[2 * i], uv[2 * i + 1]) for i in range(ne.value)]


def opara_sync_edges_pruned(dag):
    ne = C.c_int32()
    _check(load().opara_sync_edges_pruned(dag, None, 0, C.byref(ne)))
    uv = (C.c_int32 * max(2 * ne.value, 1))()
    _check(load().opara_sync_edges_pruned(dag, uv, ne.value, C.byref(ne)))
    return [(uv[2 * i], uv[2 * i + 1]) for i in range(ne.value)]


def opara_get_demands(dag):
    n = opara_num_ops(dag)
    d = (Demand * n)()
    _check(load().opara_get_demands(dag, d))
    return list(d)


def opara_wave_of(dag):
    """(wave of every operator, number of waves)."""
    n = opara_num_ops(dag)
    w, nw = (C.c_int32 * n)(), C.c_int32()
    _check(load().opara_wave_of(dag, w, C.byref(nw)))
    return list(w), nw.value


def opara_topo_order(dag):
    n = opara_num_ops(dag)
    q = (C.c_int32 * n)()
    _check(load().opara_topo_order(dag, q))
    return list(q)


def opara_capture(dag, stream_handles, mode):
    arr = (C.c_void_p * len(stream_handles))(*stream_handles)
    out = C.c_void_p()
    _check(load().opara_capture(dag, arr, len(stream_handles), mode, C.byref(out)))
    return out


def opara_persistent_workspace_bytes(dag):
    n = C.c_uint64()
    _check(load().opara_persistent_workspace_bytes(dag, C.byref(n)))
    return n.value


def opara_capture_persistent(dag, workspace_ptr, workspace_bytes, n_workgroups=0):
    out = C.c_void_p()
    _check(load().opara_capture_persistent(dag, C.c_void_p(workspace_ptr), workspace_bytes, n_workgroups,
                                           C.byref(out)))
    return out


def opara_chained_workspace_bytes(dag):
    n = C.c_uint64()
    _check(load().opara_chained_workspace_bytes(dag, C.byref(n)))
    return n.value


def opara_capture_chained(dag, workspace_ptr, workspace_bytes):
    out = C.c_void_p()
    _check(load().opara_capture_chained(dag, C.c_void_p(workspace_ptr), workspace_bytes, C.byref(out)))
    return out


def opara_persistent_status(exe, stream_handle):
    w = C.c_uint32()
    _check(load().opara_persistent_status(exe, C.c_void_p(stream_handle), C.byref(w)))
    return w.value


def opara_persistent_info(exe):
    a, b = C.c_int32(), C.c_int32()
    _check(load().opara_persistent_info(exe, C.byref(a), C.byref(b)))
    return a.value, b.value


def opara_persistent_prefix(exe):
    """Leading queue operators launched as ordinary kernels ahead of the persistent kernel."""
    a = C.c_int32()
    _check(load().opara_persistent_prefix(exe, C.byref(a)))
    return a.value


def opara_persistent_time_kernel(exe, stream_handle, launches):
    """Mean duration (us) of the persistent kernel launched alone, between HIP events on the stream."""
    a = C.c_float()
    _check(load().opara_persistent_time_kernel(exe, C.c_void_p(stream_handle), launches, C.byref(a)))
    return a.value


def opara_persistent_plan(dag):
    """(tiles, kernel ids) per operator as the persistent executor runs them."""
    n = opara_num_ops(dag)
    t, k = (C.c_int32 * n)(), (C.c_int32 * n)()
    _check(load().opara_persistent_plan(dag, t, k))
    return list(t), list(k)


def opara_persistent_set_trace(exe, stream_handle, trace_ptr, trace_bytes):
    _check(load().opara_persistent_set_trace(exe, C.c_void_p(stream_handle), C.c_void_p(trace_ptr), trace_bytes))


def opara_persistent_reset(exe, stream_handle, spin_limit=0):
    _check(load().opara_persistent_reset(exe, C.c_void_p(stream_handle), spin_limit))


def opara_replay(exe, stream_handle):
    _check(load().opara_replay(exe, C.c_void_p(stream_handle)))


def opara_verify_dependencies(dag, stream_handle):
    n = C.c_int32()
    _check(load().opara_verify_dependencies(dag, C.c_void_p(stream_handle), C.byref(n)))
    return n.value


def opara_exec_info(exe):
    a, b = C.c_int32(), C.c_int32()
    _check(load().opara_exec_info(exe, C.byref(a), C.byref(b)))
    return a.value, b.value


GROUP_KERNEL_LIGHT, GROUP_KERNEL_HEAVY, GROUP_KERNEL_STREAM = -1, -2, -3


def opara_fused_plan(exe, n_ops):
    """(node of every operator, number of nodes) of a fused executor."""
    node_of, n = (C.c_int32 * n_ops)(), C.c_int32()
    _check(load().opara_fused_plan(exe, node_of, C.byref(n), None))
    return list(node_of), n.value


def opara_fused_node_kernels(exe, dtype):
    """Kernel name of every node of a fused executor ("group_<dtype>_light/heavy" for group nodes)."""
    n = C.c_int32()
    _check(load().opara_fused_plan(exe, None, C.byref(n), None))
    k = (C.c_int32 * n.value)()
    _check(load().opara_fused_plan(exe, None, None, k))
    group = {GROUP_KERNEL_LIGHT: "light", GROUP_KERNEL_HEAVY: "heavy", GROUP_KERNEL_STREAM: "stream"}
    return [f"group_{dtype}_{group[i]}" if i in group else opara_kernel_info(i)[0] for i in k]


def opara_fused_time_nodes(exe, stream_handle, launches):
    """Microseconds per launch of every node of a fused executor, launched by itself."""
    n = C.c_int32()
    _check(load().opara_fused_plan(exe, None, C.byref(n), None))
    us = (C.c_float * n.value)()
    _check(load().opara_fused_time_nodes(exe, C.c_void_p(stream_handle), launches, us))
    return list(us)


def opara_set_operator_trace(device_ptr):
    _check(load().opara_set_operator_trace(C.c_void_p(device_ptr)))


def opara_exec_validation(exe):
    """(kind, attempts): how opara_capture checked the executable graph it returned."""
    a, b = C.c_int32(), C.c_int32()
    _check(load().opara_exec_validation(exe, C.byref(a), C.byref(b)))
    return a.value, b.value


def opara_run_persistent_noalloc(dag, stream_handle, want_error_word=True):
    """One pass through the persistent executor on the library's static workspace.  Returns the
    kernel's error word (after synchronising the stream), or None when not asked for."""
    w = C.c_uint32()
    _check(load().opara_run_persistent_noalloc(dag, C.c_void_p(stream_handle), C.byref(w) if want_error_word else None))
    return w.value if want_error_word else None


def opara_launch_op(dag, op, stream_handle):
    _check(load().opara_launch_op(dag, op, C.c_void_p(stream_handle)))


def opara_run_eager(dag, stream_handle):
    _check(load().opara_run_eager(dag, C.c_void_p(stream_handle)))


def opara_kernel_count():
    return load().opara_kernel_count()


def opara_kernel_info(kernel_id):
    name, v, l = C.c_char_p(), C.c_uint32(), C.c_uint32()
    _check(load().opara_kernel_info(kernel_id, C.byref(name), C.byref(v), C.byref(l)))
    return name.value.decode(), v.value, l.value


def opara_kernel_device_attrs(kernel_id):
    v, l = C.c_uint32(), C.c_uint32()
    _check(load().opara_kernel_device_attrs(kernel_id, C.byref(v), C.byref(l)))
    return v.value, l.value


def opara_exec_destroy(exe):
    load().opara_exec_destroy(exe)


def opara_dag_destroy(dag):
    load().opara_dag_destroy(dag)
