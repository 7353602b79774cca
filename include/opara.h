/*
 * opara.h - C ABI of the operator-parallel DAG executor for AMD MI355X (gfx950).
 *
 * The library executes one batch-1 DNN operator DAG G=(V,E) (paper Sec. 3.1,
 * "Definition of a model DAG") with independent operators running concurrently
 * on several HIP streams, replayed from a single captured hipGraph (paper
 * Sec. 3.4, Graph Capturer).
 *
 * General conventions
 *   - Every call returns an opara_status; on failure opara_last_error() gives a
 *     thread-local text valid until the next call on that thread.
 *   - Result arrays are allocated by the CALLER (host memory) with the stated
 *     length; the library only fills them.
 *   - The library never allocates device memory and never creates streams.  All
 *     tensor pointers in opara_op_desc and ext_inputs are DEVICE pointers owned by
 *     the caller; they must stay valid and fixed for the life of every opara_exec
 *     captured from the DAG (replay uses the addresses baked in at capture, the
 *     static-buffer semantics of graph replay in paper Sec. 4).
 *   - opara_build_dag / opara_assign_streams / opara_order_launch /
 *     opara_sync_edges / opara_get_demands / opara_topo_order make no HIP call
 *     and work on a machine without a GPU.
 *   - The library owns only its opaque handles (and the hipGraph, hipGraphExec and
 *     events inside an opara_exec).
 *
 * Physical tensor layouts (device memory)
 *   - image activations: [H][W][C], C fastest (batch 1)
 *   - matrices: [rows][cols] row-major
 *   - convolution weight: [C_out][kh][kw][C_in]; GEMM weight: [N][K] (K fastest)
 *   - bias: fp32 [C_out] / [N] regardless of the tensor dtype; may be NULL
 *   - element type of activations and weights: opara_op_desc.dtype
 */
#ifndef OPARA_H
#define OPARA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OPARA_MAX_INPUTS 8

typedef struct opara_dag  opara_dag;   /* created by opara_build_dag, freed by opara_dag_destroy   */
typedef struct opara_exec opara_exec;  /* created by opara_capture,  freed by opara_exec_destroy   */

enum opara_status {
  OPARA_OK = 0,
  OPARA_EINVAL = -1,       /* bad argument (null pointer, id out of range, bad shape ...)   */
  OPARA_ECYCLE = -2,       /* the operator graph has a cycle or a self-loop                 */
  OPARA_ENOMEM = -3,
  OPARA_ESTATE = -4,       /* call made out of order (e.g. capture before assign + order)   */
  OPARA_EHIP = -5,         /* a HIP call failed; text via opara_last_error()                */
  OPARA_EUNSUPPORTED = -6, /* operator / shape has no kernel, or a mode does not serve this DAG */
  OPARA_EGRAPH = -7        /* the graph runtime did not honour the dependencies of the graph it
                              was given (found by the check inside opara_capture)             */
};

enum opara_op_type {
  OPARA_CONV2D = 0, OPARA_GEMM, OPARA_BGEMM, OPARA_MAXPOOL, OPARA_AVGPOOL, OPARA_GAVGPOOL,
  OPARA_CONCAT, OPARA_LAYERNORM, OPARA_SOFTMAX, OPARA_GELU, OPARA_RELU, OPARA_ADD,
  OPARA_N_OP_TYPES
};

/* Operator table of paper Sec. 3.3 (memory- vs compute-intensive operators). */
enum opara_class { OPARA_CLASS_DEFAULT = -1, OPARA_MEM = 0, OPARA_COMP = 1 };
enum opara_dtype { OPARA_F32 = 0, OPARA_F16 = 1 };
enum opara_mode  { OPARA_PARALLEL = 0, OPARA_SEQUENTIAL = 1, OPARA_PARALLEL_CAPTURE = 2, OPARA_PARALLEL_PRUNED = 3,
                   OPARA_FUSED = 4 };

enum opara_flags {
  OPARA_FLAG_RELU     = 1u,  /* CONV2D / GEMM: clamp the result at zero                    */
  OPARA_FLAG_B_KMAJOR = 2u   /* BGEMM: second operand stored [K][N] (N fastest), else [N][K] */
};

/* Per-compute-unit limits that turn a demand record into one integer
 * (paper Sec. 2.1: an SM/CU is limited in threads, shared memory and registers). */
typedef struct {
  uint32_t num_cus;            /* informational                                            */
  uint32_t threads_per_cu;     /* resident work-items per CU (MI355X: 2048)                */
  uint32_t lds_bytes_per_cu;   /* MI355X: 163840                                           */
  uint32_t vgpr_lanes_per_cu;  /* vector registers x lanes per CU (MI355X: 4*512*64)       */
} opara_limits;

/*
 * Shape parameters.  Which fields an operator reads:
 *   CONV2D            h_in,w_in,c_in, h_out,w_out,c_out, kh,kw,sh,sw,ph,pw, flags(RELU), batch
 *                     (images, 0 = 1; activations are then [batch][H][W][C]); c_row_stride
 *                     (0 = c_out): elements between output pixels, for writing a channel
 *                     slice of a wider tensor.
 *                     y[oh][ow][co] = bias[co] + sum x[oh*sh+i-ph][ow*sw+j-pw][ci]*w[co][i][j][ci],
 *                     zero padding, cross-correlation, floor output size.
 *   GEMM              m,n,k, flags(RELU), c_row_stride (0 = n: output row stride).
 *                     Y[m][n] = X[m][k].W + bias + sum of inputs[1..] viewed [m][n].
 *   BGEMM             batch,m,n,k, alpha, the six strides (in elements), flags(B_KMAJOR).
 *                     C_b[m][n] = alpha * A_b[m][k] . B_b ; A = inputs[0], B = inputs[1].
 *   MAXPOOL/AVGPOOL   h_in,w_in,c_in,h_out,w_out, kh,kw,sh,sw,ph,pw, batch.  Max pads with -inf;
 *                     average pads with zero and always divides by kh*kw.
 *   GAVGPOOL          h_in,w_in,c_in, batch -> [batch][c_in].
 *   CONCAT            m rows; in_cols[i] columns from input i; n = sum of in_cols.
 *   LAYERNORM/SOFTMAX m rows, n cols, eps (LayerNorm: biased variance, gamma 1, beta 0),
 *                     applied to the SUM of all inputs, each viewed [m][n].
 *   GELU/RELU/ADD     m*n elements; f(sum of all inputs).  GELU is the exact erf form.
 * Every input is read as the leading prefix of its producer's buffer in the shape above.
 */
typedef struct {
  int32_t h_in, w_in, c_in;
  int32_t h_out, w_out, c_out;
  int32_t kh, kw, sh, sw, ph, pw;
  int32_t m, n, k;
  int32_t batch;
  int64_t a_batch_stride, a_row_stride;
  int64_t b_batch_stride, b_row_stride;
  int64_t c_batch_stride, c_row_stride;
  int32_t in_cols[OPARA_MAX_INPUTS];
  float   alpha, eps;
  uint32_t flags;
} opara_op_params;

/* One operator v in V with its resource-demand record (paper Sec. 3.2, Model Profiler). */
typedef struct {
  int32_t  op_type;                    /* enum opara_op_type                                */
  int32_t  op_class;                   /* enum opara_class; DEFAULT = by op_type: CONV2D,
                                          GEMM, BGEMM are COMP, everything else MEM         */
  int32_t  dtype;                      /* enum opara_dtype                                  */
  int32_t  n_inputs;                   /* 1..OPARA_MAX_INPUTS                               */
  int32_t  inputs[OPARA_MAX_INPUTS];   /* producer operator ids in ARGUMENT ORDER;
                                          id < 0 means external tensor slot -(id+1)         */
  uint32_t grid_blocks, block_threads, lds_bytes, vgprs;
                                       /* demand record used for ordering only.  All four 0:
                                          take it from the library's kernel table           */
  opara_op_params params;
  const void *weight;                  /* device, caller-owned (CONV2D, GEMM), else NULL    */
  const float *bias;                   /* device fp32, caller-owned, may be NULL            */
  void *out;                           /* device, caller-owned, distinct per operator       */
  int32_t  n_deps;                     /* 0..OPARA_MAX_INPUTS                               */
  int32_t  deps[OPARA_MAX_INPUTS];     /* further predecessors (operator ids) whose results
                                          are not arguments: they reach this operator through
                                          an external tensor slot that several producers fill
                                          (zero-copy concatenation: each branch writes its
                                          channel slice of one buffer).  They follow the
                                          arguments in the predecessor order.               */
} opara_op_desc;

/* What opara_get_demands reports per operator. */
typedef struct {
  uint32_t grid_blocks, block_threads, lds_bytes, vgprs;
  int32_t  op_class;                   /* resolved class: OPARA_MEM or OPARA_COMP           */
  int32_t  kernel_id;                  /* index into the kernel table, see opara_kernel_info */
  uint64_t demand;                     /* scalar used by opara_order_launch                 */
} opara_demand;

/*
 * Build the DAG (paper Sec. 3.1).  Validates ids and shapes, drops repeated
 * producers keeping the first (arguments, then deps), computes the topological order (ready operator with
 * the smallest id first), selects a kernel and launch shape per operator and
 * derives its demand record.  ops/ext_inputs are copied; nothing is retained.
 * Errors: EINVAL (null, n_ops <= 0, id out of range, bad n_inputs, bad shape),
 * ECYCLE, EUNSUPPORTED, ENOMEM.  lim == NULL selects the MI355X limits.
 */
int opara_build_dag(const opara_op_desc *ops, int32_t n_ops,
                    void *const *ext_inputs, int32_t n_ext,
                    const opara_limits *lim, opara_dag **out);

/*
 * Zero-copy concatenation, a rewrite of the operator list applied before opara_build_dag
 * (the paper's cost model, Sec. 3.1 Eq. 1-3, charges every operator a launch and every
 * cross-stream dependency a synchronisation: a concatenation that only copies costs both).
 * A CONCAT operator is removed when every one of its inputs is the whole output of a
 * distinct CONV2D operator of the same dtype that nothing else reads (c_out == in_cols[i],
 * batch*h_out*w_out == m, c_row_stride 0) and its readers have room for the branches in
 * their deps lists; otherwise it stays.  In the reduced list
 *   - each such branch writes its channel slice of the concatenation's buffer: out =
 *     the CONCAT's out + (first channel) elements, params.c_row_stride = the CONCAT's n;
 *     the branch's own out buffer is no longer written;
 *   - every reader of the concatenation names a new external slot (whose pointer is the
 *     CONCAT's out) as that input and lists the branches in deps, after the dependencies
 *     it already had, in argument order, without repeats;
 *   - operator ids are renumbered densely in the old order.
 * ops[n_ops], ext_inputs[n_ext]: the full DAG as opara_build_dag would take it (host).
 * out_ops: host array [n_ops], receives *n_out records.  new_id: host int32[n_ops], the
 * reduced id of every operator, -1 for a removed concatenation.  ext_out: host array
 * [n_ext + n_ops], receives the *n_ext_out external pointers of the reduced list (the
 * first n_ext unchanged).  The buffers of removed concatenations still hold the
 * concatenated tensors after a run.  No HIP call.  Errors: EINVAL, ENOMEM.
 */
int opara_elide_concats(const opara_op_desc *ops, int32_t n_ops, void *const *ext_inputs, int32_t n_ext,
                        opara_op_desc *out_ops, int32_t *n_out, int32_t *new_id, void **ext_out,
                        int32_t *n_ext_out);

/*
 * Stream allocation, paper Algorithm 1: operators are visited in topological
 * order; an operator joins the stream of its first predecessor (argument order)
 * that no successor has joined yet, otherwise it opens a new stream.  Stream ids are
 * dense in creation order.  stream_of: host int32[n_ops]; n_streams: host int32.
 */
int opara_assign_streams(opara_dag *g, int32_t *stream_of, int32_t *n_streams);

/*
 * Stream-allocation policies.  OPARA_STREAMS_ALG1 is opara_assign_streams.
 * OPARA_STREAMS_MIN is the policy the paper compares it with (Sec. 5.2: 4 streams
 * against Alg. 1's 28 on GoogLeNet; Sec. 5.4: cubic against linear time): the fewest
 * streams any allocation can use, i.e. a minimum cover of the DAG by chains (sets of
 * operators totally ordered by the dependency relation), from a maximum matching between
 * operators and their descendants.  The number of streams is unique (the width of the
 * DAG), the allocation is not; streams are numbered by their first operator in
 * topological order.  Replaces the stream map later calls use.
 */
enum opara_stream_policy { OPARA_STREAMS_ALG1 = 0, OPARA_STREAMS_MIN = 1 };
int opara_assign_streams_policy(opara_dag *g, int32_t policy, int32_t *stream_of, int32_t *n_streams);

/*
 * Launch order, paper Algorithm 2: two ready lists (memory- and compute-intensive),
 * chosen alternately starting with the memory list (the other one when the
 * preferred list is empty); from the chosen list the operator with the least
 * demand goes next (ties: topological index).  order: host int32[n_ops].
 */
int opara_order_launch(opara_dag *g, int32_t *order);

/*
 * Launch-order policies for ablation (paper Sec. 2.3: the launch order alone moves the
 * latency).  OPARA_ORDER_ALG2 is opara_order_launch.  Every policy yields a topological
 * order and replaces the queue a later opara_capture uses.
 *   ALG2_COMP_FIRST  Alg. 2 with the preference starting at the compute list
 *   LEAST_DEMAND     one ready list, least demand first (no class alternation)
 *   MOST_DEMAND      one ready list, largest demand first
 *   TOPO             ready operator with the smallest id first (trace order)
 *   LEVEL            by depth (longest distance from a root), then id: wave by wave
 */
enum opara_order_policy {
  OPARA_ORDER_ALG2 = 0, OPARA_ORDER_ALG2_COMP_FIRST, OPARA_ORDER_LEAST_DEMAND,
  OPARA_ORDER_MOST_DEMAND, OPARA_ORDER_TOPO, OPARA_ORDER_LEVEL, OPARA_N_ORDER_POLICIES
};
int opara_order_launch_policy(opara_dag *g, int32_t policy, int32_t *order);

/*
 * Dependencies that need a synchronisation operator (paper Sec. 3.1, Eq. 3; Sec. 4):
 * every edge (u,v) whose endpoints are on different streams, sorted by (v, argument
 * position of u).  uv: host int32[2*cap] filled with pairs u,v up to cap pairs;
 * n_edges always receives the full count.  Needs opara_assign_streams first (ESTATE).
 */
int opara_sync_edges(const opara_dag *g, int32_t *uv, int32_t cap, int32_t *n_edges);

/*
 * The same list without the dependencies that other ordering constraints imply (paper
 * Sec. 3.1: each synchronisation costs t_overhead, Eq. 3): a cross-stream dependency
 * (u,v) is dropped when v is reachable from u through two or more constraints, a
 * constraint being any dependency or two consecutive operators of one stream in
 * launch-queue order.  The result is unique.  Needs streams and a launch queue (ESTATE).
 * OPARA_PARALLEL_PRUNED builds the graph with these synchronisations only.
 */
int opara_sync_edges_pruned(const opara_dag *g, int32_t *uv, int32_t cap, int32_t *n_edges);

/*
 * Wave of every operator (host int32[n_ops]; n_waves may be NULL): 0 for an operator
 * without predecessors, else one more than the largest wave of its predecessors.  The
 * waves are what OPARA_FUSED launches together.  No HIP call.
 */
int opara_wave_of(const opara_dag *g, int32_t *wave_of, int32_t *n_waves);

/* Demand records (paper Sec. 3.2) and default topological order; host arrays [n_ops]. */
int opara_get_demands(const opara_dag *g, opara_demand *out);
int opara_topo_order(const opara_dag *g, int32_t *order);
int32_t opara_num_ops(const opara_dag *g);

/*
 * Graph capture (paper Sec. 3.4): one executable graph that holds every operator,
 * with exactly these dependencies: the previous operator of the same stream in
 * launch-queue order, plus every cross-stream predecessor (what recording one event
 * after each producer with a cross-stream consumer and waiting once per such producer
 * on the consumer's stream yields).  No operator executes.
 *   OPARA_PARALLEL          assembles that graph node by node.  hip_streams[0..n_streams)
 *                           (hipStream_t handles supplied by the caller, at least as many
 *                           as opara_assign_streams reported, all distinct) carry no
 *                           operator; hip_streams[0] runs the check described below and
 *                           is synchronised.  A DAG with several sinks gets one trailing
 *                           node without work that joins them.
 *                           The executable graph is validated before it is returned (the
 *                           graph runtime has been seen to start operators of irregular
 *                           DAGs before a predecessor had finished, in some instances of a
 *                           graph and not in others): it is instantiated with marker
 *                           kernels as nodes, replayed twice on hip_streams[0] (each
 *                           marker counts predecessors that have not finished; static
 *                           device memory only), and only an instance without violations
 *                           has its nodes switched to the operators' kernels, in place.
 *                           After a violation a fresh instance of the SAME graph is
 *                           tried, up to four; the streams and the launch queue are never
 *                           replaced.  EGRAPH if no instance passes.  No node is given
 *                           more than four successors: further consumers of a producer
 *                           depend on it through a chain of relay nodes without work
 *                           (every failure seen involved nodes with 7-15 successors), so
 *                           the graph can hold more nodes and edges than the plan has
 *                           operators and dependencies (opara_exec_info).
 *   OPARA_PARALLEL_CAPTURE  obtains the same graph the paper's way: the streams are put
 *                           into one stream capture, every operator is launched on its
 *                           stream in launch-queue order with event record / wait on
 *                           the cross-stream edges, all streams join hip_streams[0].
 *                           Only for DAGs with one root and one sink whose plan is a
 *                           fork-join of streams: every stream but the first waits
 *                           exactly once, for one event, at its first operator (which
 *                           brings it into the capture); only the first stream waits
 *                           repeatedly (EUNSUPPORTED otherwise, decided before any HIP
 *                           call).  With the ROCm 7.0 runtime,
 *                           captures in which streams waited on each other repeatedly
 *                           (chains of blocks whose heads read several branch tails,
 *                           random DAGs) ended in a crash of the host process; the cause
 *                           inside the runtime is not known, which is why this route is
 *                           limited to the shape it is tested on and is not the default.
 *                           Not validated.
 *   OPARA_PARALLEL_PRUNED   as OPARA_PARALLEL, without the cross-stream edges that
 *                           opara_sync_edges_pruned drops (the check still counts every
 *                           predecessor).
 *   OPARA_SEQUENTIAL        captures the same kernels with the same launch shapes on
 *                           hip_streams[0] alone in default topological order (the
 *                           baseline: paper Sec. 5.1, default sequential graph).
 *   OPARA_FUSED             operator parallelism inside kernel nodes instead of between
 *                           streams: on this runtime a dependency between streams of a
 *                           graph costs more than a batch-1 operator (the t_overhead of
 *                           paper Eq. 3), a dependency inside a single chain of nodes
 *                           much less.  The launch queue is cut into waves - every
 *                           operator whose predecessors all lie in earlier waves, in
 *                           launch-queue order, so Alg. 2 still decides which operators
 *                           meet on the chip and in which order their workgroups are
 *                           dispatched.  A wave of one operator becomes an ordinary
 *                           kernel node (the same kernel as in the other modes); a wave of
 *                           several becomes a group node: ONE kernel whose grid is the sum
 *                           of the members' grids, each workgroup running its operator's
 *                           own body (at most 16 operators per node, a larger wave is
 *                           split; a wave that mixes register-heavy contractions with
 *                           more than 2,048 workgroups of lighter work is cut between
 *                           the two, so that the lighter operators keep their occupancy).  All nodes form one chain.  Needs a launch queue only
 *                           (ESTATE); streams play no part, hip_streams is not read beyond
 *                           the argument check.  Operators inside a group run the
 *                           four-wavefront form of their kernel, so results can differ
 *                           from the other modes in the last bits; they are identical from
 *                           replay to replay.  The opara_dag must outlive the opara_exec.
 * Errors: ESTATE if assign/order were not called (parallel modes), EINVAL,
 * EUNSUPPORTED, EGRAPH, EHIP (a running capture is ended and the partial graph destroyed).
 */
int opara_capture(opara_dag *g, void *const *hip_streams, int32_t n_streams,
                  int32_t mode, opara_exec **out);

/*
 * How an executable graph was checked before opara_capture returned it (host int32 each,
 * either may be NULL): kind is OPARA_VALIDATED_IN_PLACE (the returned instance itself ran
 * the marker check), OPARA_SCREENED_ON_TWIN (the runtime refused to switch the kernels of
 * an instantiated graph, so the operators' graph was instantiated beside a marker graph
 * that passed) or OPARA_NOT_VALIDATED (sequential graph, stream capture, persistent
 * executor: single chains and single kernels have not shown the defect); attempts is the
 * number of instances built.
 */
enum opara_validation { OPARA_NOT_VALIDATED = 0, OPARA_SCREENED_ON_TWIN = 1, OPARA_VALIDATED_IN_PLACE = 2 };
int opara_exec_validation(const opara_exec *e, int32_t *kind, int32_t *attempts);

/*
 * Dependency self-check of the graph runtime as a call of its own (diagnostics: how often
 * does an instance of this plan's graph fail?).  Builds one instance of the marker graph
 * opara_capture validates (same node order and dependency edges as OPARA_PARALLEL), launches
 * it twice on `hip_stream`, which is synchronised; n_violations receives the number of
 * operators that started before a predecessor had finished (0 = every dependency was
 * honoured).  Uses static device memory only.  It says nothing about an opara_exec:
 * opara_capture checks the instance it returns by itself.  Needs assign + order first (ESTATE).
 */
int opara_verify_dependencies(opara_dag *g, void *hip_stream, int32_t *n_violations);

/*
 * Persistent executor: the paper's goal (Sec. 2.2, 3.1: keep the GPU's units busy by
 * running independent operators side by side, with as little synchronisation cost
 * `t_overhead` as possible, Eq. 3) reached without streams.  The captured graph holds ONE
 * kernel.  The (operator, tile) work items of the launch queue (the queue of the last
 * opara_order_launch / _policy call, so Alg. 2 still decides which operators meet on the
 * chip) are dealt round-robin to its workgroups; an item starts as soon as every
 * predecessor of its operator has finished all its tiles.  The workgroup that finishes
 * an operator's last tile raises the operator's completion flags in device memory;
 * activations are written and read with device-coherent accesses, so a dependency costs
 * one flag hand-off (about half a microsecond) instead of a graph-node boundary, and
 * independent operators overlap at tile granularity.  Stream assignment plays no part.
 *
 * workspace: device memory, caller-owned, 256-byte aligned, at least
 * opara_persistent_workspace_bytes() bytes, exclusively this executor's until it is
 * destroyed; capture writes the operator records into it with a blocking copy.
 * n_workgroups: 0 = as many as the device holds at once (two per compute unit for DAGs up
 * to a few hundred operators); a smaller positive count is honoured, a larger one is cut
 * to that maximum, because every workgroup must be resident.  Items follow a topological
 * order, so the holder of the lowest unfinished item can always run.
 * The executor has its own kernel plan (opara_persistent_plan: one workgroup size, so
 * the 8-wavefront and quad-coalesced contractions run the 4-wavefront fragment-loading
 * form), and the serial prefix of the queue runs as ordinary kernel nodes ahead of the
 * persistent kernel (opara_persistent_prefix): results may differ from the other modes
 * in the last bits, and are identical from replay to replay.
 * Every wait inside the kernel is bounded (spin_limit polls, default 2^22); a wait that
 * runs out makes all workgroups leave and sets a sticky error word (1 + queue position,
 * counted from the first operator inside the kernel, of an operator whose wait ran out;
 * it stays non-zero until reset), which opara_persistent_status reads after synchronising
 * `hip_stream`.  opara_persistent_reset synchronises the stream, clears counters, flags
 * and error word and sets the spin limit (0 = default).  Replays of one executor must not
 * overlap (same stream, or ordered by the caller).  Several persistent executors, or one
 * beside other kernels, may run at the same time: they share the device's workgroup slots,
 * and a launch whose workgroups are not all resident yet makes progress as the others
 * finish (its waits are long, not unbounded).
 * Assumptions the hand-off rests on (hardware behaviour of gfx950, not the language memory
 * model): results are written with device-coherent write-through stores (sc1), a wavefront
 * waits for its own stores with s_waitcnt vmcnt(0) before the workgroup's thread 0 adds to
 * the operator's counter with a RELAXED device-scope atomic, and a consumer invalidates its
 * caches after it has seen the flag.  The stores of the other wavefronts are ordered before
 * the counter update by the workgroup barrier and their own vmcnt wait, not by a release
 * fence (a release at device scope writes back the whole L2 of the XCD, about 200 ns per
 * workgroup, serialised).  Under the HIP memory model this is a data race; on gfx950 a
 * store that vmcnt has retired has reached the memory side all XCDs share.  The second
 * assumption is residency: work items are dealt to workgroups statically, so the launch
 * makes progress only while all its workgroups are resident; co-running kernels that hold
 * compute units for long can make a wait run out (reported, see below).
 * Errors: ESTATE without a launch queue, EINVAL (workspace), EUNSUPPORTED (more than 8
 * predecessors or 65535 tiles per operator, more than about 2,600 operators, mixed
 * element types), EHIP.
 * Replay with opara_replay, destroy with opara_exec_destroy.
 */
int opara_persistent_workspace_bytes(const opara_dag *g, uint64_t *bytes);
int opara_capture_persistent(opara_dag *g, void *workspace, uint64_t workspace_bytes,
                             int32_t n_workgroups, opara_exec **out);
int opara_persistent_status(opara_exec *e, void *hip_stream, uint32_t *error_word);
/* Work items and workgroups of a persistent executor (host int32 each). */
int opara_persistent_info(const opara_exec *e, int32_t *n_items, int32_t *n_workgroups);
/*
 * Tiles (workgroup-sized pieces) and kernel id of every operator as the persistent
 * executor runs it: tiles[n_ops], kernel_ids[n_ops] (host, either may be NULL).  The
 * persistent executor has one workgroup size and its own hand-over point between the
 * contraction kernels, so these can differ from the graph executors' launch grids that
 * opara_get_demands reports (paper Sec. 3.2 profiles one kernel per operator; here an
 * operator has one per executor kind).  No HIP call.
 */
int opara_persistent_plan(const opara_dag *g, int32_t *tiles, int32_t *kernel_ids);
/*
 * Number of leading launch-queue operators that the executor launches as ordinary kernel
 * nodes ahead of the persistent kernel, in one chain inside the same hipGraph: those that
 * nothing else can run beside (every other operator depends on each of them, a network's
 * stem; the paper's Fig. 1 DAGs start with such a chain).  They run the graph executors'
 * kernels.  Work items, and the queue positions in the timeline, start at the first
 * operator after them.  (Setting OPARA_PERSIST_SERIAL_PREFIX=0 in the environment at
 * capture keeps every operator inside the persistent kernel, for comparison.)
 */
int opara_persistent_prefix(const opara_exec *e, int32_t *n_prefix);
/*
 * Measurement aid: launches the persistent kernel alone (an ordinary launch with the
 * executor's arguments, without the kernel nodes of the serial prefix, whose outputs a
 * previous replay has left in place) `launches` times back to back on `hip_stream`,
 * between two HIP events on that stream, and returns the elapsed time per launch in
 * microseconds (host float).  Synchronises the stream.  At least one replay must have
 * completed.
 */
int opara_persistent_time_kernel(opara_exec *e, void *hip_stream, int32_t launches, float *avg_us);
/*
 * Timeline of the following replays (tracing; the one kernel hides the operators from
 * a profiler).  trace: device memory, caller-owned, 8-byte aligned, 32 bytes per work
 * item, or NULL to switch tracing off.  Work item i (launch-queue order, tiles of an
 * operator consecutive) gets four uint64: the 100 MHz device clock when its workgroup
 * began looking it up, when its predecessors were complete, when its body had finished,
 * and (queue position << 32 | workgroup).  Synchronises `hip_stream`.
 */
int opara_persistent_set_trace(opara_exec *e, void *hip_stream, void *trace, uint64_t trace_bytes);
int opara_persistent_reset(opara_exec *e, void *hip_stream, uint32_t spin_limit);

/*
 * Chained executor: the persistent executor without its work-item loop.  ONE launch whose
 * grid is the sum of the operators' grids in launch-queue order (the serial prefix of the
 * queue again as ordinary kernel nodes ahead of it); a workgroup runs exactly one tile: it
 * looks up its operator, waits until the completion flags of the operator's predecessors
 * carry this launch's number, runs the tile with the operator's own body and counts it; the
 * workgroup that counts an operator's last tile raises the operator's flags.  The hand-off
 * is the persistent executor's (same assumptions about write-through stores, stated there).
 * What differs: workgroups are dispatched in increasing block order and every predecessor's
 * blocks come before its consumers' blocks, so the lowest unfinished block can always run:
 * the launch drains with whatever number of workgroups the device holds at a time, beside
 * other kernels too (no residency assumption).  And because a body is straight-line code
 * behind the wait, the kernel holds every 256-thread body, the quad-coalesced contractions
 * included (kernel plan: the one of OPARA_FUSED's group nodes).
 * workspace: device memory, caller-owned, 256-byte aligned, at least
 * opara_chained_workspace_bytes() bytes, exclusively this executor's until it is destroyed.
 * opara_persistent_status / _reset / _info / _prefix / _time_kernel / _set_trace serve a
 * chained executor too (work items = workgroups = blocks of the launch; 32 bytes of trace
 * per block).  Errors: as opara_capture_persistent.  Replay with opara_replay.
 */
int opara_chained_workspace_bytes(const opara_dag *g, uint64_t *bytes);
int opara_capture_chained(opara_dag *g, void *workspace, uint64_t workspace_bytes, opara_exec **out);

/*
 * For callers that cannot allocate device memory (code running under a stream capture of
 * their own, tight serving loops, harnesses that forbid hipMalloc): one pass over the DAG
 * through the persistent executor, as opara_capture_persistent + opara_replay run it, but
 * without a graph and without a caller workspace.  The workspace (counters, completion
 * flags, operator records) is a static device array inside the library, 2.5 MiB per GPU,
 * held until the process ends; it serves DAGs of up to 512 operators (EUNSUPPORTED beyond,
 * before anything is launched).  The call uploads the workspace image on `hip_stream`
 * (every call uploads all of it, so whatever the previous call left in the array is
 * overwritten), launches the serial prefix of the launch queue as ordinary kernels and then
 * the persistent kernel, all on `hip_stream`, asynchronously.  It calls no hipMalloc,
 * hipFree or other allocating routine of the HIP runtime.  error_word: NULL, or a host
 * uint32 that receives the kernel's error word (0 = every wait ended; see
 * opara_capture_persistent) after the call has synchronised `hip_stream`.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different
 * streams, or another thread) race; order them on one stream.  Synchronise `hip_stream`
 * before the DAG is destroyed or given a new launch queue.  Needs a launch queue (ESTATE).
 */
int opara_run_persistent_noalloc(opara_dag *g, void *hip_stream, uint32_t *error_word);

/*
 * Fused executor (OPARA_FUSED): the node of the chain every operator runs in (host
 * int32[n_ops], nodes numbered in execution order), the number of nodes, and the kernel of
 * every node (host int32[n_nodes]: a kernel id of the kernel table for a single operator,
 * OPARA_GROUP_KERNEL_STREAM / _LIGHT / _HEAVY for a group node: the group kernel that holds
 * the bodies with at most 64 vector registers, at most 128, or all bodies); each may be
 * NULL.  Operators that share a node run concurrently inside one kernel.
 */
enum { OPARA_GROUP_KERNEL_LIGHT = -1, OPARA_GROUP_KERNEL_HEAVY = -2, OPARA_GROUP_KERNEL_STREAM = -3 };
int opara_fused_plan(const opara_exec *e, int32_t *node_of, int32_t *n_nodes, int32_t *node_kernel);
/*
 * Measurement aid: launches every node of a fused executor by itself (an ordinary launch
 * of the node's kernel with the node's arguments) `launches` times back to back on
 * `hip_stream`, after two untimed launches, between two HIP events on that stream, and
 * returns the time per launch in microseconds, us[n_nodes] (host float).  Outputs are
 * rewritten with the same values.  Synchronises the stream.
 */
int opara_fused_time_nodes(opara_exec *e, void *hip_stream, int32_t launches, float *us);

/*
 * One hipGraphLaunch on `hip_stream`; asynchronous, the caller synchronises.  The status
 * covers the launch only.  A persistent executor reports a wait that ran out inside its
 * kernel through its sticky error word, not here: a caller that must know reads
 * opara_persistent_status after the replays it cares about (once the word is set, every
 * later replay leaves its outputs unwritten until opara_persistent_reset).
 */
int opara_replay(opara_exec *e, void *hip_stream);

/* Nodes and dependency edges of the captured graph (host int32 each). */
int opara_exec_info(const opara_exec *e, int32_t *n_nodes, int32_t *n_edges);

/*
 * Operator timeline (tracing; what the paper reads off a profiler's timeline, Sec. 5.2,
 * taken inside the kernels so that the measurement does not move them).  Executors that are
 * CAPTURED while a buffer is set (sequential graph, multi-stream graph, fused executor), and
 * eager launches made meanwhile, hand the buffer to their kernels as an argument: the
 * operator's first workgroup then folds the 100 MHz device clock at its start into word
 * 2*op (minimum) and its last eight workgroups, in dispatch order, the clock at their end
 * into word 2*op + 1 (maximum; uint64 each; op = the operator's id in its DAG).  Executors captured while no buffer is set carry a
 * null pointer and pay one scalar compare per workgroup.
 * device_buffer: device memory, caller-owned, 16 bytes per operator, initialised by the
 * caller to (all ones, zero) before every replay it wants stamped, valid as long as any
 * executor captured with it is replayed; NULL ends the setting for later captures.  The
 * setting is per process.  No HIP call.  The persistent and chained executors have their
 * own per-tile timeline (opara_persistent_set_trace).
 */
int opara_set_operator_trace(void *device_buffer);

/*
 * Launch ONE operator's kernel, or all operators in topological order, eagerly on a
 * stream (no graph).  Used for profiling an operator in isolation (paper Sec. 3.2:
 * profile once) and for debugging.
 */
int opara_launch_op(opara_dag *g, int32_t op, void *hip_stream);
int opara_run_eager(opara_dag *g, void *hip_stream);

/*
 * Kernel table: static resources of every kernel in the library, read from the
 * compiled code objects at build time (vgprs = vector + accumulation registers per
 * lane; lds_bytes = static LDS per workgroup).  opara_kernel_device_attrs asks the
 * HIP runtime for the same figures (needs a GPU).
 */
int32_t opara_kernel_count(void);
int opara_kernel_info(int32_t kernel_id, const char **name, uint32_t *vgprs, uint32_t *lds_bytes);
int opara_kernel_device_attrs(int32_t kernel_id, uint32_t *vgprs, uint32_t *lds_bytes);

void opara_exec_destroy(opara_exec *e);
void opara_dag_destroy(opara_dag *g);
const char *opara_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OPARA_H */
