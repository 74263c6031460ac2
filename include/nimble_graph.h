/*
 * nimble_graph.h - C ABI of the ahead-of-time multi-stream DAG executor for MI355X.
 *
 * The calls follow the problem statement of the Nimble paper (arXiv 2012.02732):
 *   1. register a static operator DAG with a fixed input shape (Section 4, "System
 *      Design": the system takes a computation graph as input);
 *   2. run the ahead-of-time pass once (Section 4.1 "Ahead-of-time (AoT) Scheduling",
 *      Section 4.2 "Stream Assignment Algorithm", Algorithm 1, Appendix A);
 *   3. replay the recorded task schedule for every new input (Section 4.1, last
 *      paragraph: replay through a graph launch).
 *
 * General conventions
 *   - Every function returns NG_OK (0) or a negative NG_E* code. Nothing throws or
 *     aborts across this boundary. ng_last_error() gives a readable message for the
 *     last failure on that graph.
 *   - A graph is not thread-safe; use one graph from one thread at a time.
 *   - Tensors are fp32, NCHW, dense.
 *   - Ownership: the library owns the graph object, its schedule, task table, events
 *     and HIP graph objects. The CALLER owns the arena, all weight buffers and all
 *     streams, and must keep them alive and unchanged in address until ng_destroy().
 *     Weight, arena and stream arguments are DEVICE-side handles (device pointers /
 *     hipStream_t values passed as void*); every other pointer is a HOST pointer.
 *   - Call order: ng_create -> ng_add_input / ng_add_node ... -> ng_mark_output ...
 *     -> ng_schedule -> ng_plan_memory -> ng_bind -> ng_capture -> ng_replay / ng_sync.
 *     A call made too early returns NG_ESTATE. Everything up to and including
 *     ng_plan_memory is host-only and works on a machine without a GPU.
 */
#ifndef NIMBLE_GRAPH_H
#define NIMBLE_GRAPH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NG_MAX_PREDS 8

enum {
    NG_OK = 0,
    NG_EINVAL = -1, /* bad argument (null pointer, unknown id, unknown op, bad parameter) */
    NG_ESHAPE = -2, /* operand shapes do not fit the operator */
    NG_ESTATE = -3, /* call made in the wrong phase */
    NG_ENOMEM = -4, /* arena too small or too few streams */
    NG_EHIP = -5    /* a HIP runtime call failed; text in ng_last_error() */
};

/* Operator vocabulary: one node = one GPU task (the paper's operators may be several
 * tasks, Section 1; here the DAG is registered at task granularity). */
enum {
    NG_OP_INPUT = 0,          /* network input, no kernel; the caller writes it into the arena */
    NG_OP_CONV1X1 = 1,        /* pointwise conv, weights {W[cout][cin]} */
    NG_OP_DWCONV = 2,         /* depthwise k x k, k in {3,5}, stride in {1,2}, pad = k/2, weights {W[c][k][k]} */
    NG_OP_CONV3X3 = 3,        /* dense 3x3, stride in {1,2}, pad in {0,1}, weights {W[cout][cin][3][3]} */
    NG_OP_BN_ACT = 4,         /* inference batch norm (+ReLU if relu != 0), weights {gamma, beta, mean, var}, each [c] */
    NG_OP_RELU = 5,           /* max(x, 0) */
    NG_OP_ADD_N = 6,          /* elementwise sum of 2..NG_MAX_PREDS tensors of equal shape */
    NG_OP_CONCAT = 7,         /* channel slices [slice_lo[j], slice_hi[j]) of pred j stacked along C */
    NG_OP_POOL = 8,           /* 3x3 window, pool_mode 0 = max, 1 = avg (divisor = in-bounds taps), stride {1,2}, pad {0,1} */
    NG_OP_GLOBAL_AVGPOOL = 9, /* mean over H x W -> [n][c][1][1] */
    NG_OP_FC = 10,            /* y = W x + b on [n][cin][1][1], weights {W[cout][cin], b[cout]} */
    /* Training (Section 5, the training results: one whole iteration - forward pass, backward pass and
     * weight update - is recorded and replayed like an inference). The backward operators are tasks
     * of the same DAG; "dy" is the gradient of the loss with respect to the forward operator's
     * result, "x" the forward operator's input (listed where its values or only its shape are
     * needed). Weight arguments are the FORWARD operator's own buffers. Batch norm keeps its
     * statistics (mean, var) fixed. A graph with an NG_OP_SGD_UPDATE node is a graph that trains:
     * its convolutions, fc and batch-norms read their parameters where the caller keeps them on
     * every replay (nothing is repacked or folded at ng_bind). */
    NG_OP_CONV1X1_DGRAD = 11, /* preds {dy}, weights {W[cout][cin]}, cout = channels of the result (the forward cin):
                                 dx[n][ci] = sum_co W[co][ci] dy[n][co]; with h = w = 1 the fc's input gradient */
    NG_OP_CONV1X1_WGRAD = 12, /* preds {dy, x} -> dW as [cout][cin][1][1]; with h = w = 1 the fc's */
    NG_OP_CONV3X3_DGRAD = 13, /* preds {dy, x}, weights {W}, stride, pad of the forward conv -> dx, shape of x */
    NG_OP_CONV3X3_WGRAD = 14, /* preds {dy, x}, stride, pad -> dW [cout][cin][3][3] */
    NG_OP_DWCONV_DGRAD = 15,  /* preds {dy, x}, weights {W[c][k][k]}, k, stride -> dx */
    NG_OP_DWCONV_WGRAD = 16,  /* preds {dy, x}, k, stride -> dW as [1][c][k][k] */
    NG_OP_BN_ACT_DGRAD = 17,  /* preds {dy, x}, weights {gamma, beta, mean, var}, eps, relu -> dx */
    NG_OP_BN_ACT_WGRAD = 18,  /* preds {dy, x}, same weights -> [2][c][1][1]: dgamma, then dbeta */
    NG_OP_RELU_DGRAD = 19,    /* preds {dy, x} -> dy where x > 0, else 0 */
    NG_OP_POOL_DGRAD = 20,    /* preds {dy, x}, pool_mode, stride, pad -> dx; max: to the first tap (row-major in the
                                 window) that attains the maximum; avg: dy / in-bounds taps of the window */
    NG_OP_GAP_DGRAD = 21,     /* preds {dy, x} -> dy[n][c] / (h w) at every pixel */
    NG_OP_CHANNEL_SUM = 22,   /* preds {dy} -> [1][c][1][1], sum over n, h, w (the fc's bias gradient) */
    NG_OP_SLICE_PAD = 23,     /* preds {dy}: gradient of one concat input. Result has cout channels; its channels
                                 [slice_lo[1], slice_lo[1] + cnt) are dy's channels [slice_lo[0], slice_hi[0]),
                                 cnt = slice_hi[0] - slice_lo[0]; every other channel is 0 */
    NG_OP_SGD_UPDATE = 24     /* preds {grad, then any nodes that must have run first (readers of W)}, weights {W}:
                                 W[i] -= lr * grad[slice_lo[0] + i] for i < cout, IN PLACE in the caller's buffer;
                                 the node's own result is [1][1][1][1] */
};

typedef struct ng_op_params {
    int32_t cout;      /* CONV1X1, CONV3X3, FC; CONV1X1_DGRAD, SLICE_PAD: channels of the result; SGD_UPDATE: elements of W */
    int32_t k;         /* DWCONV: 3 or 5 */
    int32_t stride;    /* DWCONV, CONV3X3, POOL: 1 or 2 */
    int32_t pad;       /* CONV3X3, POOL: 0 or 1 */
    int32_t relu;      /* BN_ACT */
    int32_t pool_mode; /* POOL: 0 max, 1 avg */
    float eps;         /* BN_ACT */
    int32_t slice_lo[NG_MAX_PREDS]; /* CONCAT; slice_hi[j] == 0 means "all channels of pred j" */
    int32_t slice_hi[NG_MAX_PREDS];
    float lr;          /* SGD_UPDATE */
} ng_op_params;

typedef struct ng_graph ng_graph; /* opaque */

/* ---- 1. registration (Section 4: a DAG G = (V, E) of operators, fixed input shape) ---- */

/* Create an empty graph. *out receives the handle (host pointer, library-owned). */
int ng_create(ng_graph** out);
/* Release everything the library owns (schedule, events, HIP graphs). NULL is allowed. */
void ng_destroy(ng_graph* g);

/* Add an input node of shape nchw[4] (host array). *id receives the node id. Node ids
 * are 0, 1, 2, ... in registration order. */
int ng_add_input(ng_graph* g, const int64_t nchw[4], int* id);

/* Add an operator node. preds (host array of n_preds ids) must name existing nodes, so
 * ids are a topological order of the DAG. dev_weights (host array of n_weights DEVICE
 * pointers, caller-owned) are the operator's parameters in the order listed at the op
 * enum; they may be NULL pointers until ng_capture (host-only use). The output shape is
 * inferred here; a mismatch returns NG_ESHAPE and leaves the graph unchanged. */
int ng_add_node(ng_graph* g, int op_kind, const ng_op_params* p,
                const int* preds, int n_preds,
                const void* const* dev_weights, int n_weights, int* id);

/* Mark a node whose tensor the caller will read after a replay. */
int ng_mark_output(ng_graph* g, int id);

int ng_num_nodes(const ng_graph* g);
/* Inferred output shape of a node into nchw[4] (host). */
int ng_node_shape(const ng_graph* g, int id, int64_t nchw[4]);

/* ---- 2a. ahead-of-time pass, host part (Section 4.2, Algorithm 1, Appendix A) ---- */

/* Stream assignment and synchronisation plan. Closes registration.
 *   Step 1   minimum equivalent graph G' = (V, E');
 *   Step 2-3 maximum matching M of the bipartite graph of E' (augmenting paths, left and
 *            right nodes in ascending id);
 *   Step 4-5 chains = sets merged along M ("chain_of", Algorithm 1 verbatim);
 *   then chains are joined tail-to-head along closure edges, and a final augmenting pass
 *   over the closure makes the stream count equal the widest antichain ("stream_of");
 *   Lambda = E' edges whose ends are on different streams (Appendix A: each must be
 *   synchronised itself, Lemma 1); one event per distinct producer in Lambda.
 * Submission order is ascending node id; node 0 is on stream 0, the capture origin. */
int ng_schedule(ng_graph* g);

/* How ng_schedule forms the streams out of the chains (call before ng_schedule; NG_ESTATE after).
 *   NG_ASSIGN_ALGORITHM1 (default): as described above - Algorithm 1, chains joined, then the
 *     augmenting pass. Stream count = widest antichain always; |Lambda| = the minimum of
 *     Theorem 3, |E'| - |M|, whenever the last pass finds nothing to do.
 *   NG_ASSIGN_EXACT: the partition into the fewest chains of the closure that, among those,
 *     keeps the most E' edges inside a stream - a maximum matching of the closure's bipartite
 *     graph with as many E' edges as possible, found as a minimum-cost assignment (O(V^3)).
 *     Stream count = widest antichain and |Lambda| = the least any such partition allows, always.
 *     chain_of (Algorithm 1 verbatim) is the same in both. Which of several optimal partitions
 *     comes out is unspecified. */
enum { NG_ASSIGN_ALGORITHM1 = 0, NG_ASSIGN_EXACT = 1 };
int ng_set_assignment(ng_graph* g, int assignment);

/* Sizes of the arrays ng_get_schedule fills (any pointer may be NULL). */
int ng_schedule_sizes(const ng_graph* g, int* n_nodes, int* n_streams, int* n_chains,
                      int* n_meg_edges, int* n_matching, int* n_sync, int* n_events);

/* Copy the schedule into caller-allocated HOST arrays (any may be NULL):
 *   order[n_nodes], stream_of[n_nodes], chain_of[n_nodes], event_of[n_nodes] (-1 = none),
 *   meg_src/meg_dst[n_meg_edges] sorted by (src, dst),
 *   sync_src/sync_dst[n_sync] sorted by (src, dst). */
int ng_get_schedule(const ng_graph* g, int* order, int* stream_of, int* chain_of, int* event_of,
                    int* meg_src, int* meg_dst, int* sync_src, int* sync_dst);

/* Capture scaffolding, not part of Lambda: fork[] = non-origin streams whose first task
 * waits for nothing (they join the capture through an event recorded on the origin
 * before its first task); join[] = non-origin streams the origin waits for after its
 * last task. Arrays are caller-allocated with room for n_streams entries. */
int ng_get_scaffold(const ng_graph* g, int* fork, int* n_fork, int* join, int* n_join);

/* Static memory plan (Section 4.1: memory requests are identical on every run, so the
 * exact amount is reserved once). One buffer per node output, 256-byte aligned, no reuse over
 * time. One exception to "one buffer each": at batch 1 a tensor that a concat takes whole is
 * placed inside the concat's buffer, at its channel block (16-byte aligned), so it is produced
 * in place and the concat copies nothing for it. *arena_bytes receives the total. */
int ng_plan_memory(ng_graph* g, size_t* arena_bytes);
/* Reuse over time, off by default (call before ng_plan_memory). When on, a tensor's buffer may be
 * handed to a later node v once the tensor is dead FOR v: its producer and every one of its
 * readers are ancestors of v in the DAG, so that any execution that respects the DAG - on any
 * number of streams - is through with it before v writes. Best fit among such buffers, else new
 * memory. Network inputs, outputs and the tensors of in-place concats keep private buffers.
 * The device-resident replay normally keeps a stream's tensors in the L2 of one XCD; on such a plan
 * an address holds several tensors in the course of a replay, so there every load and store of it
 * goes through device scope instead (as with device_scope_everywhere of ng_resident_config) and no
 * task runs inside another task's tiles: slower than on a plan without reuse, same results. */
int ng_set_memory_reuse(ng_graph* g, int on);
/* Modes 0-3 launch one kernel per task, except that (on by default) a batch-norm / ReLU whose only
 * input is a convolution result is applied by that convolution's kernel, a concat whose inputs
 * were all produced in place is not launched, and weight updates (NG_OP_SGD_UPDATE) whose output no
 * node reads are carried out together by the launch of the last of them on their stream (modes 1 and
 * 2: of the last of them in the submission order; same arithmetic per element), and the input gradient
 * and the parameter gradients of a batch-norm (NG_OP_BN_ACT_DGRAD, NG_OP_BN_ACT_WGRAD with the same dy
 * and x) are computed in one walk over dy and x by the launch of whichever of the two comes first, if
 * both are on one stream (always, in modes 1 and 2); likewise the input gradient and the weight gradient
 * of a depthwise or 1 x 1 convolution (same dy) share one launch, their workgroups interleaved, if
 * everything the later one reads is complete when the earlier one starts. on = 0 switches the
 * exceptions off: one kernel per task. Call before ng_bind (NG_ESTATE after). */
int ng_set_launch_fusion(ng_graph* g, int on);
/* offset[n_nodes], bytes[n_nodes] of each node's output inside the arena (host arrays). */
int ng_get_offsets(const ng_graph* g, size_t* offset, size_t* bytes);

/* Longest path of G under per-node weights t[n_nodes] (e.g. isolated kernel times):
 * the critical-path time of Section 3. path[] (room for n_nodes) receives the node ids. */
int ng_critical_path(const ng_graph* g, const float* t, float* total, int* path, int* n_path);

/* The dependency edges of the multi-stream HIP graph (NG_MODE_GRAPH_MULTI) exactly as ng_capture
 * writes them, computed on the host (needs ng_plan_memory, no GPU): Section 4.1 replays the
 * recorded tasks through one graph launch, and by Appendix A that record is only safe if every
 * edge of E is ordered by the FIFO order of a stream or by a synchronised edge. fuse != 0: the
 * graph as launched by default; 0: one kernel node per task (see ng_set_launch_fusion); 2: what the
 * single-stream modes launch instead (the launches in submission order, each behind the one before).
 *   launched_by[n_nodes] (may be NULL): the task whose kernel node writes node v's tensor - v
 *     itself, the convolution that also applies a fused batch-norm / ReLU, the later weight update
 *     of the same stream whose launch also carries out this one, the other half of a batch-norm's
 *     backward pass that comes earlier on the stream, -1 for a network input, -2 for a
 *     concat that is not launched because its inputs are produced in place;
 *   src/dst[max_edges]: one entry per graph edge, as task ids (both ends have kernel nodes);
 *   *n_edges: the number of edges; with max_edges = 0 only the count is returned, a positive
 *     max_edges that is too small gives NG_ENOMEM. All arrays are caller-owned host memory. */
int ng_get_graph_edges(ng_graph* g, int fuse, int* launched_by, int* n_edges, int* src, int* dst, int max_edges);
/* Name of the kernel node `id` will be bound to, worked out on the host from the shapes alone (needs
 * ng_plan_memory, no GPU; after ng_bind the same as ng_task_kernel): which of the hand-written kernels a
 * task runs is decided by the library, per node, from its operator, shapes and the graph's being a
 * training graph or not (Section 4.1: the pre-run records the kernel of every task once). "" for an input
 * node, NULL on an error (ng_last_error). The string is a constant of the library. */
const char* ng_planned_task_kernel(ng_graph* g, int id);

/* ---- 2b. ahead-of-time pass, GPU part (Section 4.1: pre-run once, record the tasks) ---- */

/* Attach caller-owned device memory and streams. arena: DEVICE pointer, 256-byte aligned,
 * at least the planned size. hip_streams: HOST array of n_streams DISTINCT hipStream_t values, all
 * on the current device, n_streams >= the scheduled stream count (NG_ENOMEM otherwise).
 * Builds the task table: kernel, launch geometry and argument block with resolved device
 * addresses for every node. Also allocates a library-owned constants buffer (freed by
 * ng_destroy) and fills it from the conv1x1 weights, repacked into matrix-core operand
 * order: weight VALUES are read here, so a caller that changes them binds again. */
int ng_bind(ng_graph* g, void* arena, size_t arena_bytes, void* const* hip_streams, int n_streams);

/* Pre-run the network once and make the recorded schedule executable in every replay
 * mode: a HIP graph of the multi-stream schedule (one kernel node per task in submission
 * order, an edge from the previous task of the same stream and one per planned event
 * wait), a HIP graph with every task on the origin stream (recorded by stream capture of
 * the pre-run), and the device-resident plan (per-workgroup task lists, completion
 * counters; NG_ENOMEM if the persistent workgroups cannot all be co-resident). The arena
 * contents are overwritten with whatever the pre-run computes from its current input. */
int ng_capture(ng_graph* g);

/* Fixed DEVICE address of a node's output inside the bound arena (NULL on error). The
 * caller writes the input tensor to ng_tensor_ptr(g, input_id) before ng_replay and reads
 * outputs after ng_sync. */
void* ng_tensor_ptr(const ng_graph* g, int id);

/* ---- 3. replay (Section 4.1: raw submission of the recorded tasks) ---- */

enum {
    /* Modes 0-3 run one stand-alone kernel per task, except that a batch-norm / ReLU whose only input is a
     * convolution result is applied by the convolution's kernel (both tensors are stored) and a concat whose
     * inputs were all produced in place is not launched; such a task keeps its place in the schedule (its
     * waits and its event), and every tensor equals the one-kernel-per-task result bit for bit. */
    NG_MODE_GRAPH_MULTI = 0,  /* multi-stream graph, one hipGraphLaunch. LIMITATION: on one synthetic DAG (80 nodes,
                                 33 streams) this HIP runtime let a kernel node start before its only dependency had
                                 finished in 4-16 % of the launches, although the edge was in the graph. ng_capture
                                 therefore replays this graph 8-64 times on a poisoned arena and compares every byte
                                 with the single-stream graph's result (ng_graph_multi_check); if they ever differ
                                 the mode is not a candidate of NG_MODE_AUTO and ng_replay refuses it (NG_ESTATE).
                                 The check is a screen, not a proof: rare misorderings can pass it. */
    NG_MODE_GRAPH_SINGLE = 1, /* captured single-stream graph */
    NG_MODE_EAGER_SINGLE = 2, /* task table launched kernel by kernel on the origin stream */
    NG_MODE_EAGER_MULTI = 3,  /* task table launched on the assigned streams with real events */
    NG_MODE_DEVICE_RESIDENT = 4, /* one launch; persistent workgroups walk the recorded schedule themselves:
                                   a stream = a gang of workgroups serving its tasks in FIFO order, an event =
                                   a completion counter in device memory (record = release add, wait = poll +
                                   acquire). Raw submission of the task schedule (Section 4.1) without the
                                   command processor between dependent tasks. A batch-norm / ReLU or add_n may run
                                   inside the tiles of the task that produces its operand, and a concat whose
                                   inputs were produced in place runs nothing (ng_resident_fusion reports which);
                                   every node's tensor is written all the same and equals the other modes' bit
                                   for bit. The plan passes a self-check at ng_capture or the capture fails. */
    NG_MODE_AUTO = 5          /* the default: whichever of modes 0, 1 and 4 was fastest in a short trial at ng_capture (an
                                   ahead-of-time choice like the rest of the schedule: DAGs of many tiny tasks
                                   gain most from mode 4, plain chains and large tasks from a HIP graph) */
};
int ng_replay_mode(ng_graph* g, int mode);
/* The mode NG_MODE_AUTO stands for (0, 1 or 4) and the median replay + wait times, in
 * microseconds, the trial at ng_capture measured for modes 0, 1 and 4 (HOST array of 3;
 * either pointer may be NULL). 0 for a mode that was not a candidate: mode 0 when its check
 * failed. */
int ng_auto_mode(const ng_graph* g, int* mode, float* trial_us);
/* Result of the check of the multi-stream graph at ng_capture (see NG_MODE_GRAPH_MULTI):
 * *state = 1 every compared replay reproduced the single-stream result byte for byte, -1 some
 * replay did not (or the caller distrusts it), 0 not checked; *replays_compared = how many. */
int ng_graph_multi_check(const ng_graph* g, int* state, int* replays_compared);
/* Run the same check again with `replays` (1..100000) replays, e.g. for more confidence than the
 * 8-64 replays of ng_capture give; may turn state 1 into -1, never back. Overwrites the arena
 * (network inputs are kept); waits for the origin stream. NG_MODE_AUTO is re-decided. */
int ng_graph_multi_recheck(ng_graph* g, int replays);
/* For a caller whose own validation caught the multi-stream graph with a wrong result: marks it
 * as failed (state -1): NG_MODE_AUTO no longer picks it and ng_replay refuses it. */
int ng_graph_multi_distrust(ng_graph* g);
/* Asynchronous: enqueue one inference on the origin stream (hip_streams[0]). */
int ng_replay(ng_graph* g);
/* Wait until the origin stream is idle. */
int ng_sync(ng_graph* g);
/* The device-resident replay (NG_MODE_DEVICE_RESIDENT, whatever mode is selected) for callers that
 * cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc. Same kernel, same recorded plan and same results as ng_replay in that mode, but the
 * completion counters, the per-launch XCD records and the error flag live in a file-scope device
 * array of the library (2.5 MiB, held by every GPU the library runs on until the process ends)
 * instead of memory from hipMalloc. The call allocates and frees nothing and records no memset: it
 * enqueues a fill kernel that clears the part of the array it uses and then the replay kernel, both
 * on the origin stream. Limits: graphs of at most 1024 nodes (NG_ENOMEM with the sizes otherwise);
 * needs ng_capture (NG_ESTATE before); the
 * device the graph was bound on must be current (NG_EINVAL). All calls on one GPU - of this graph
 * or of any other - share the array: calls that overlap on one GPU race; wait (ng_sync) for one
 * before the next is enqueued. The per-task timeline (ng_resident_trace) is not recorded. */
int ng_replay_static(ng_graph* g);

/* Device-resident replay settings. workgroups_per_cu: resident workgroups per compute unit
 * (0 = automatic; only before ng_capture). xcds: number of XCDs (1..8; 0 = automatic;
 * only before ng_capture) the streams are spread over; with 1 the whole DAG runs out of one
 * XCD's L2 and no completion needs a device-scope fence. spin_limit: polls after which a waiting workgroup
 * gives up (0 = default, a few seconds); every wait in the resident kernel is bounded by it.
 * When a wait gives up, all workgroups leave, ng_sync returns NG_EHIP and the next replay
 * starts from clean counters. device_scope_everywhere != 0 (only before ng_capture) makes
 * every completion a device-scope release/acquire; by default a tensor that stays on the
 * XCD of its stream is handed over through that XCD's L2 and only the others pay for an L2
 * write-back and invalidate. */
int ng_resident_config(ng_graph* g, int workgroups_per_cu, int xcds, unsigned spin_limit, int device_scope_everywhere);
/* How many settings of the device-resident planner's cost model ng_capture tries (1..8; default 8;
 * only before ng_capture). The planner decides between plans whose expected lengths differ by
 * less than its model's error; ng_capture therefore builds the plans of `trials` settings (the
 * first is the default one), replays each distinct plan a few times and keeps the fastest -
 * the pre-run of Section 4.1 used for measuring as well as for recording. With 1 the default
 * setting's plan is taken unmeasured (capture is shorter and the plan does not depend on timing). */
int ng_resident_plan_trials(ng_graph* g, int trials);
/* *setting = which of the tried settings ng_capture kept (0 = the default one). With all 8 settings
 * tried, ng_capture also re-plans the kept setting once with every task's cost corrected by the
 * task times a traced replay of the kept plan measured, and keeps that plan instead if it replays
 * faster: *setting = 8 then. Needs ng_capture. */
int ng_resident_plan_kept(const ng_graph* g, int* setting);
/* Per-task timeline of device-resident replays. enable != 0 switches recording on and clears
 * the record (off for 0). If ticks is not NULL it first receives what was recorded since the
 * last call: four device clock readings per node (HOST array of 4 * n_nodes values, 100 MHz
 * clock; a task that did not run keeps ~0, 0, ~0, 0): the first workgroup starts to wait for
 * the producers, the last workgroup has its inputs ready, the first and the last workgroup
 * have stored their tiles. Record ONE replay between two calls for a timeline of that
 * replay. A batch-norm / ReLU node that the plan fused into the convolution feeding it has
 * no workgroups of its own: it reports the convolution's first / last store for both pairs
 * (an interval of length zero). Waits for the origin stream to go idle. */
int ng_resident_trace(ng_graph* g, int enable, unsigned long long* ticks);
/* *verified = 1 if the probe at ng_capture found that workgroups of the resident grid with equal
 * index mod 8 share an XCD, which is what the plan's use of XCD-local L2s rests on; 0 if not, in which case every hand-over
 * of the device-resident replay goes through device scope (correct on any mapping, slower). */
int ng_resident_xcd_mapping(const ng_graph* g, int* verified);
/* Which nodes the device-resident plan runs inside another node's tiles: host_of[v] (n_nodes entries,
 * caller-owned host memory) = the convolution whose tiles also apply node v (a batch-norm / ReLU
 * directly behind it, or an add_n that takes its - possibly batch-normed - result as one operand),
 * -2 for a concat that has nothing to do because the memory plan placed all its inputs inside its
 * result (its readers wait for the producers of those inputs), or -1 for a node with workgroups of
 * its own. Needs ng_capture. */
int ng_resident_fusion(const ng_graph* g, int* host_of);
/* Host-only rehearsal of the device-resident plan (needs ng_plan_memory, no GPU): plans for
 * n_workgroups persistent workgroups (a multiple of 8) over xcds XCDs (0 = let the cost
 * model choose) and reports the expected makespan in microseconds, the number of
 * (workgroup, task) entries, the number of operands that cross XCDs, and whether the plan
 * passed its self-check (every tile of every task assigned exactly once - a batch-norm / ReLU
 * node fused into its convolution counts through that convolution's tiles -, every list in one
 * common topological order, expected completion counts consistent). Any pointer may be NULL. */
int ng_resident_dry_plan(ng_graph* g, int n_workgroups, int xcds, double* expected_us, int* n_entries,
                         int* n_far_edges, int* coverage_ok);
/* The same rehearsal for the setting-th (0..7) of the planner settings that ng_capture tries
 * (ng_resident_plan_trials); setting 0 is what ng_resident_dry_plan plans with. */
int ng_resident_dry_plan_setting(ng_graph* g, int setting, int n_workgroups, int xcds, double* expected_us,
                                 int* n_entries, int* n_far_edges, int* coverage_ok);
/* Layout chosen at ng_capture: resident workgroups, total (workgroup, task) entries, XCDs in
 * use, and the makespan in microseconds that the planner's cost model expects (any pointer
 * may be NULL). */
int ng_resident_sizes(const ng_graph* g, int* n_workgroups, int* n_entries, int* xcds, double* expected_us);

/* Device time of one replay in the current mode: `reps` replays are enqueued back to back on
 * the origin stream between two events recorded on that stream; *avg_us = elapsed / reps. */
int ng_time_replay(ng_graph* g, int reps, float* avg_us);
/* Raw timing primitive: a graph that is a chain of `reps` copies of node id's kernel (id = -1:
 * an empty kernel) is launched on the origin stream and timed with events; *us_per_node
 * receives elapsed / reps (best of three launches). Includes the dependent-dispatch gap. */
int ng_time_chain(ng_graph* g, int id, int reps, float* us_per_node);
/* Cross-check of ng_time_task_device that needs no timestamps: chain time of the task's kernel minus
 * the chain time of an empty kernel (that removes the dispatch gap); a lower estimate of the kernel's
 * duration, since whatever an empty kernel itself takes is subtracted too. 0 for input nodes. */
int ng_time_task(ng_graph* g, int id, int reps, float* isolated_us);
/* Time the GPU is busy with one task's kernel when it runs alone (Section 3: the "GPU active
 * time" of an operator, which the critical-path time sums along the longest path), by the device's
 * own clock: a copy of the kernel that reads the 100 MHz clock at the first instruction of every
 * workgroup and again once the workgroup's stores are acknowledged is launched `reps` times by
 * itself; one launch's time = latest end - earliest start over its workgroups. *median_us and
 * *min_us (may be NULL) receive median and minimum. What the command processor spends around a
 * dispatch is not part of it (a kernel trace's begin-to-end time of the same kernel is 1-2 us longer).
 * as_executed = 0: the task's stand-alone kernel, one kernel per task whatever the replay mode does.
 * as_executed != 0 (needs ng_capture): the kernel the current replay mode really runs for the task -
 * in modes 0-3 a convolution together with the batch-norm / ReLU fused into its kernel, in the
 * device-resident mode the plan's kernel variant with its fused batch-norm and add_n - and 0 for a
 * task that has no kernel of its own in that mode (it runs inside another task's kernel or has
 * nothing to do) and for inputs. */
int ng_time_task_device(ng_graph* g, int id, int as_executed, int reps, float* median_us, float* min_us);
/* One launch of the same kernel (as_executed as above; id = -1: an empty kernel) on the origin
 * stream, awaited before the call returns: a solo dispatch for a kernel trace taken from outside
 * (rocprofv3 --kernel-trace), whose begin-to-end timestamps are the other definition of an isolated
 * kernel time. Nothing is launched for a task without a kernel of its own. */
int ng_launch_task_solo(ng_graph* g, int id, int as_executed);
/* Name of the kernel the current replay mode runs for the node, as timed by ng_time_task_device with
 * as_executed != 0; "" if it has none of its own. Needs ng_capture. Valid until ng_destroy. */
const char* ng_task_kernel_executed(const ng_graph* g, int id);
/* Median wall time, in microseconds, of launching one empty kernel on the origin stream and waiting
 * for it: what a replay + wait costs before any task has run. */
int ng_time_launch_floor(ng_graph* g, int reps, float* median_us);
/* Name of the kernel bound to a node ("" for input nodes); valid until ng_destroy. */
const char* ng_task_kernel(const ng_graph* g, int id);
/* Algorithmic work of a node, from its shapes: bytes moved and flops (host doubles). */
int ng_task_work(const ng_graph* g, int id, double* bytes, double* flops);

const char* ng_last_error(const ng_graph* g);
const char* ng_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_GRAPH_H */
