"""Marshalling between a workload description and the C ABI.

Allocates device buffers through PyTorch (memory and streams are the only things
PyTorch provides), converts logical tensors to the library's physical layouts
([H][W][C] images, [N][K] GEMM weights, [C_out][kh][kw][C_in] convolution weights),
fills opara_op_desc records and drives the library.  No operator arithmetic and no
scheduling decision happens here.
"""
import ctypes as C
import numpy as np
from . import binding as B

_IMAGE_TYPES = ("conv2d", "maxpool", "avgpool", "gavgpool")


def _is_image(op):
    return op.type in _IMAGE_TYPES or (op.type == "concat" and op.params.get("axis") == 0) \
        or (op.type in ("add", "relu", "gelu") and len(op.out_shape) == 3)


def _hip():
    import torch  # noqa: F401  (makes sure the HIP runtime PyTorch uses is the one loaded)
    return C.CDLL("libamdhip64.so.7") if not hasattr(_hip, "lib") else _hip.lib


class StreamSet:
    """n distinct non-blocking HIP streams (PyTorch's own pool holds only 32 handles,
    fewer than Alg. 1 may open), wrapped as torch ExternalStream objects."""

    def __init__(self, n, device):
        import torch
        self.lib = C.CDLL("libamdhip64.so.7")
        self.lib.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        self.lib.hipStreamDestroy.argtypes = [C.c_void_p]
        self.handles = []
        torch.cuda.set_device(device)
        for _ in range(n):
            h = C.c_void_p()
            rc = self.lib.hipStreamCreateWithFlags(C.byref(h), 1)  # hipStreamNonBlocking
            if rc != 0:
                raise RuntimeError(f"hipStreamCreateWithFlags failed with {rc}")
            self.handles.append(h.value)
        self.torch_streams = [torch.cuda.ExternalStream(h, device=device) for h in self.handles]

    def close(self):
        for h in self.handles:
            self.lib.hipStreamDestroy(C.c_void_p(h))
        self.handles = []


class Session:
    """One workload bound to device buffers and a built DAG handle."""

    def __init__(self, wl, device="cuda:0", demand_override=None, class_override=None, pad_channels=True,
                 zero_copy_concat=False):
        """pad_channels: an external image whose channel count is not a multiple of the
        16-byte vector width and that feeds convolutions only is stored with zero
        channels appended (and the weights with matching zero taps) - a storage layout,
        the results are unchanged.
        zero_copy_concat: the operator list goes through opara_elide_concats before the DAG is
        built: concatenations of convolution branches are removed, each branch writes its
        channel slice of the concatenated buffer and the readers depend on the branches.
        `self.lib_ops[i]` is the workload id of library operator i, `self.lib_id[v]` the
        library id of workload operator v (absent if removed), `self.elided` the removed
        concatenations.  Outputs are still addressed by workload id."""
        self.wl = wl
        self.device = device
        self.dag = None
        self.execs = []
        self._workspaces = []
        self.streams = None
        self.capture_log = []
        self._fake = 0x10000
        self._keep = []
        self.dtype_id = B.F32 if wl.dtype == "f32" else B.F16
        ve = 4 if wl.dtype == "f32" else 8
        self.ext_pad = {}
        if pad_channels:
            users = {}
            for op in wl.ops:
                for u in op.inputs:
                    if u < 0:
                        users.setdefault(-u - 1, []).append(op)
            for slot, a in enumerate(wl.ext_inputs):
                chans = a.shape[-3] if a.ndim >= 3 else 0
                if a.ndim >= 3 and chans % ve and all(o.type == "conv2d" for o in users.get(slot, [])):
                    self.ext_pad[slot] = (chans + ve - 1) // ve * ve
        self.ext_dev = [self._upload(self._to_physical_input(a, self.ext_pad.get(i))) for i, a in enumerate(wl.ext_inputs)]
        self.out_dev = [None] * len(wl.ops)
        self.w_dev, self.b_dev = {}, {}
        descs = []
        for op in wl.ops:
            d = B.OpDesc()
            d.op_type = B.OP_TYPE_IDS[op.type]
            d.op_class = B.CLASS_DEFAULT if class_override is None else class_override[op.id]
            d.dtype = self.dtype_id
            d.n_inputs = len(op.inputs)
            for i, u in enumerate(op.inputs):
                d.inputs[i] = u
            if demand_override is not None:
                d.grid_blocks, d.block_threads, d.lds_bytes, d.vgprs = demand_override[op.id]
            self._fill_params(op, d.params)
            if op.type == "conv2d" and op.inputs[0] < 0 and (-op.inputs[0] - 1) in self.ext_pad:
                d.params.c_in = self.ext_pad[-op.inputs[0] - 1]
            if op.id in wl.weights:
                w, b = wl.weights[op.id]["w"], wl.weights[op.id]["b"]
                if op.type == "conv2d":
                    wp = np.transpose(w, (0, 2, 3, 1))
                    cpad = self.ext_pad.get(-op.inputs[0] - 1) if op.inputs[0] < 0 else None
                    if cpad:
                        wp = np.concatenate([wp, np.zeros(wp.shape[:3] + (cpad - wp.shape[3],), dtype=w.dtype)], axis=3)
                    wp = np.ascontiguousarray(wp)
                else:
                    wp = np.ascontiguousarray(w.T)
                self.w_dev[op.id] = self._upload(wp)
                self.b_dev[op.id] = self._upload(b.astype(np.float32))
                d.weight = self._ptr(self.w_dev[op.id])
                d.bias = self._ptr(self.b_dev[op.id])
            self.out_dev[op.id] = self._alloc(int(np.prod(op.out_shape)) * (wl.batch if _is_image(op) else 1))
            d.out = self._ptr(self.out_dev[op.id])
            descs.append(d)
        ext_ptrs = [self._ptr(t) for t in self.ext_dev]
        self.elided = []                    # workload ids of the concatenations the library removed
        self.lib_ops = list(range(len(wl.ops)))
        if zero_copy_concat:
            # The library decides which concatenations go and where their branches write; here
            # only the buffers follow: a branch's output becomes a view into the concatenation's.
            full = descs
            descs, new_id, ext_ptrs = B.opara_elide_concats(full, ext_ptrs)
            self.lib_ops = [v for v in range(len(wl.ops)) if new_id[v] >= 0]
            self.elided = [v for v in range(len(wl.ops)) if new_id[v] < 0]
            owner = {self._ptr(self.out_dev[c]): c for c in self.elided}
            es = self._elsize()
            for v in self.lib_ops:
                d, before = descs[new_id[v]], full[v]
                if d.out == before.out:
                    continue
                total = d.params.c_row_stride
                c = next(c for base, c in owner.items() if base <= d.out < base + self._numel(c) * es)
                off = (d.out - self._ptr(self.out_dev[c])) // es
                if self.device is None:
                    self.out_dev[v] = d.out
                else:
                    self.out_dev[v] = self.out_dev[c].view(-1, total)[:, off:off + d.params.c_out]
        self.lib_id = {v: i for i, v in enumerate(self.lib_ops)}
        self.descs = descs
        self.dag = B.opara_build_dag(descs, ext_ptrs)

    def _numel(self, op_id):
        op = self.wl.ops[op_id]
        return int(np.prod(op.out_shape)) * (self.wl.batch if _is_image(op) else 1)

    # ---- device memory (PyTorch) or fake addresses when there is no device
    def _upload(self, arr):
        if self.device is None:
            return self._fake_ptr(arr.nbytes)
        import torch
        return torch.from_numpy(np.ascontiguousarray(arr)).to(self.device)

    def _alloc(self, numel):
        if self.device is None:
            return self._fake_ptr(numel * (4 if self.wl.dtype == "f32" else 2))
        import torch
        return torch.zeros(numel, dtype=torch.float32 if self.wl.dtype == "f32" else torch.float16,
                           device=self.device)

    def _elsize(self):
        return 4 if self.wl.dtype == "f32" else 2

    def _fake_ptr(self, nbytes):
        p = self._fake
        self._fake += (nbytes + 255) // 256 * 256
        return p

    def _ptr(self, t):
        return t if isinstance(t, int) else t.data_ptr()

    @staticmethod
    def _to_physical_input(a, pad_to=None):
        if a.ndim < 3:
            return a
        hwc = np.moveaxis(a, -3, -1)                  # [..., C, H, W] -> [..., H, W, C]
        if pad_to:
            hwc = np.concatenate([hwc, np.zeros(hwc.shape[:-1] + (pad_to - hwc.shape[-1],), dtype=a.dtype)], axis=-1)
        return np.ascontiguousarray(hwc)

    def _fill_params(self, op, p):
        q, t = op.params, op.type
        if t in ("conv2d", "maxpool", "avgpool", "gavgpool"):
            p.c_in, p.h_in, p.w_in = op.in_shapes[0]
            p.c_out, p.h_out, p.w_out = op.out_shape
            p.batch = self.wl.batch
            for k in ("kh", "kw", "sh", "sw", "ph", "pw"):
                if k in q:
                    setattr(p, k, q[k])
            if q.get("relu"):
                p.flags |= B.FLAG_RELU
        elif t == "gemm":
            p.m, p.n, p.k = q["m"], q["n"], q["k"]
            if q.get("relu"):
                p.flags |= B.FLAG_RELU
        elif t == "bgemm":
            h, s, d = q["heads"], q["seq"], q["dhead"]
            p.batch, p.alpha = h, q["alpha"]
            if q["mode"] == "qk":      # scores_h = alpha * Q_h . K_h^T
                p.m, p.n, p.k = s, s, d
                p.a_batch_stride, p.a_row_stride = d, h * d
                p.b_batch_stride, p.b_row_stride = d, h * d
                p.c_batch_stride, p.c_row_stride = s * s, s
            else:                      # context_h = P_h . V_h, V read in place ([K][N])
                p.m, p.n, p.k = s, d, s
                p.a_batch_stride, p.a_row_stride = s * s, s
                p.b_batch_stride, p.b_row_stride = d, h * d
                p.c_batch_stride, p.c_row_stride = d, h * d
                p.flags |= B.FLAG_B_KMAJOR
        elif t == "concat":
            if q["axis"] == 0:
                p.m = op.out_shape[1] * op.out_shape[2] * self.wl.batch
                cols = [s[0] for s in op.in_shapes]
            else:
                p.m = op.out_shape[0]
                cols = [s[1] for s in op.in_shapes]
            for i, c in enumerate(cols):
                p.in_cols[i] = c
            p.n = sum(cols)
        elif len(op.out_shape) == 3:   # gelu, relu, add on images: element-wise over [B][H][W][C]
            c, h, w = op.out_shape
            p.m, p.n = h * w * self.wl.batch, c
        else:                          # layernorm, softmax, gelu, relu, add
            p.m, p.n = op.in_shapes[0]
            p.eps = q.get("eps", 0.0)

    # ---- the path
    def schedule(self, policy=B.ORDER_ALG2, stream_policy=B.STREAMS_ALG1):
        so, ns = B.opara_assign_streams_policy(self.dag, stream_policy)
        order = B.opara_order_launch_policy(self.dag, policy)
        return so, ns, order, B.opara_sync_edges(self.dag)

    def make_streams(self, n):
        if self.streams is None or len(self.streams.handles) < n:
            if self.streams is not None:
                self.streams.close()
            self.streams = StreamSet(n, self.device)
        return self.streams

    def capture(self, mode, policy=B.ORDER_ALG2, stream_policy=B.STREAMS_ALG1):
        """Schedule (parallel modes) and capture a graph.  The library validates a multi-stream
        graph before it returns it; `self.capture_log` records how (kind, instances built)."""
        if mode in (B.SEQUENTIAL, B.FUSED):
            if mode == B.FUSED:
                B.opara_order_launch_policy(self.dag, policy)
            st = self.make_streams(1)
            exe = B.opara_capture(self.dag, st.handles[:1], mode)
            self.execs.append(exe)
            return exe
        _, ns, _, _ = self.schedule(policy, stream_policy)
        st = self.make_streams(max(ns, 1))
        exe = B.opara_capture(self.dag, st.handles[:ns], mode)
        kind, attempts = B.opara_exec_validation(exe)
        self.capture_log.append(dict(mode=mode, policy=policy, validation=kind, attempts=attempts))
        self.execs.append(exe)
        return exe

    def capture_persistent(self, policy=B.ORDER_ALG2, n_workgroups=0):
        """Capture the whole DAG as one persistent kernel (work items in launch-queue order,
        dependencies through completion counters).  The workspace is a torch allocation
        kept alive by the session."""
        import torch
        B.opara_order_launch_policy(self.dag, policy)
        nbytes = B.opara_persistent_workspace_bytes(self.dag)
        ws = torch.zeros(nbytes + 256, dtype=torch.uint8, device=self.device)
        ptr = (ws.data_ptr() + 255) // 256 * 256
        torch.cuda.synchronize()
        exe = B.opara_capture_persistent(self.dag, ptr, nbytes, n_workgroups)
        self._workspaces.append(ws)
        self.execs.append(exe)
        return exe

    def capture_chained(self, policy=B.ORDER_ALG2):
        """Capture the DAG as one loop-free kernel (one tile per workgroup, blocks in launch-queue
        order, dependencies through completion flags).  The workspace is a torch allocation kept
        alive by the session."""
        import torch
        B.opara_order_launch_policy(self.dag, policy)
        nbytes = B.opara_chained_workspace_bytes(self.dag)
        ws = torch.zeros(nbytes + 256, dtype=torch.uint8, device=self.device)
        ptr = (ws.data_ptr() + 255) // 256 * 256
        torch.cuda.synchronize()
        exe = B.opara_capture_chained(self.dag, ptr, nbytes)
        self._workspaces.append(ws)
        self.execs.append(exe)
        return exe

    def run_persistent_noalloc(self, policy=B.ORDER_ALG2):
        """One pass through the persistent executor on the library's static workspace (no graph,
        no allocation).  Returns the kernel's error word."""
        B.opara_order_launch_policy(self.dag, policy)
        return B.opara_run_persistent_noalloc(self.dag, self.make_streams(1).handles[0])

    def persistent_trace(self, exe):
        """Replay once with the in-kernel timeline on.  Returns an int64 array [tiles, 5]:
        lookup start, predecessors complete, body end (ns since the first event), queue
        position, workgroup.  Operators of the serial prefix (ordinary kernels ahead of the
        persistent one) have no rows."""
        import torch
        items, _ = B.opara_persistent_info(exe)
        buf = torch.zeros(items * 4, dtype=torch.int64, device=self.device)
        h = self.make_streams(1).handles[0]
        torch.cuda.synchronize()
        B.opara_persistent_set_trace(exe, h, buf.data_ptr(), buf.numel() * 8)
        self.replay(exe)
        B.opara_persistent_set_trace(exe, h, 0, 0)
        raw = buf.cpu().numpy().reshape(items, 4)
        raw = raw[raw[:, 2] != 0]                 # items that only pad an operator's range record nothing
        t = raw[:, :3] * 10                       # 100 MHz ticks -> ns
        t = t - t.min()
        # the kernel counts queue positions from the first operator it runs itself
        pos = (raw[:, 3:4] >> 32) + B.opara_persistent_prefix(exe)
        return np.concatenate([t, pos, (raw[:, 3:4] & 0xffffffff)], axis=1)

    def operator_trace(self, mode, policy=B.ORDER_ALG2, replays=3):
        """Capture the sequential / multi-stream / fused executor with the operator timeline on and
        replay it.  Returns an int64 array [library operators, 2]: earliest start and latest end of
        every operator's kernel in the last replay, ns from the first start (-1: no stamp)."""
        import torch
        n = len(self.lib_ops)
        buf = torch.empty(n, 2, dtype=torch.int64, device=self.device)
        torch.cuda.synchronize()
        B.opara_set_operator_trace(buf.data_ptr())
        try:
            exe = self.capture(mode, policy=policy)
        finally:
            B.opara_set_operator_trace(0)
        for _ in range(replays):
            buf[:, 0] = -1                              # all ones: the minimum folds into it
            buf[:, 1] = 0
            torch.cuda.synchronize()
            self.replay(exe)
        raw = buf.cpu().numpy()
        self._keep.append(buf)                          # the executor keeps the address
        ok = (raw[:, 0] != -1) & (raw[:, 1] != 0)
        t = raw.astype(np.int64) * 10                   # 100 MHz ticks -> ns
        t0 = t[ok, 0].min() if ok.any() else 0
        t = t - t0
        t[~ok] = -1
        return t

    def persistent_status(self, exe):
        return B.opara_persistent_status(exe, self.make_streams(1).handles[0])

    def persistent_reset(self, exe, spin_limit=0):
        B.opara_persistent_reset(exe, self.make_streams(1).handles[0], spin_limit)

    def replay(self, exe, sync=True):
        import torch
        st = self.make_streams(1)
        B.opara_replay(exe, st.handles[0])
        if sync:
            st.torch_streams[0].synchronize()

    def run_eager(self):
        st = self.make_streams(1)
        B.opara_run_eager(self.dag, st.handles[0])
        st.torch_streams[0].synchronize()

    def clear_outputs(self):
        for t in self.out_dev:
            t.zero_()
        import torch
        torch.cuda.synchronize()

    def output(self, op_id):
        """Operator output as a numpy array in the logical layout of the workload."""
        op = self.wl.ops[op_id]
        a = self.out_dev[op_id].cpu().numpy()
        if _is_image(op):
            c, h, w = op.out_shape
            if self.wl.batch > 1:
                return np.ascontiguousarray(np.transpose(a.reshape(self.wl.batch, h, w, c), (0, 3, 1, 2)))
            return np.ascontiguousarray(np.transpose(a.reshape(h, w, c), (2, 0, 1)))
        return a.reshape(op.out_shape)

    def close(self):
        for e in self.execs:
            B.opara_exec_destroy(e)
        self.execs = []
        if self.dag is not None:
            B.opara_dag_destroy(self.dag)
            self.dag = None
        if self.streams is not None:
            self.streams.close()
            self.streams = None
