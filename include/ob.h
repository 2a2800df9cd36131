/*
 * ob.h - C ABI of the on-the-fly operation batching library for AMD MI355X (gfx950).
 *
 * The calls follow the paper's problem statement (Section 2, Train-Batch-Naive):
 * New-Graph, append the nodes of every instance, Forward(L), Backward(L), read
 * values and gradients.  Graph definition is lazy (Section 3.1): adding a node
 * computes nothing; ob_forward schedules every pending node on the GPU
 * (Section 3.2: signatures, depth, batches) and executes each batch as one
 * batched operation (Section 3.3).  The caller keeps seeing the unbatched node
 * ids (Section 3.3, single -> batch node conversion is internal).
 *
 * Conventions
 *  - Every function returns 0 (OB_OK) or a negative OB_E_* code; node adders
 *    return the new node id (>= 0) or a negative code.  No C++ type, exception
 *    or torch type crosses this boundary.
 *  - "host" pointers are ordinary CPU memory owned by the caller and copied (in)
 *    or filled (out) during the call.  "device" pointers are HIP device memory.
 *  - Output buffers carry a capacity in elements; a too-small buffer fails with
 *    OB_E_RANGE and writes nothing.
 *  - The device arena and the stream are owned by the caller and must outlive the
 *    context.  The library allocates no device memory of its own: parameters,
 *    graph tables, values and gradients are carved out of the arena.
 *  - A context is not thread-safe.  Work is enqueued on the context's stream;
 *    reads synchronise that stream.
 *  - Graph errors (forward reference, dimension mismatch, label or slice out of
 *    range) are detected on the host when the node is added, so the GPU never sees
 *    a malformed graph.
 *  - Matrices are row-major fp32.  A bias is a rows x 1 parameter.
 */
#ifndef OB_H
#define OB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ob_ctx ob_ctx;

/* error codes */
#define OB_OK 0
#define OB_E_BADID (-1)    /* unknown node / parameter id, or forward reference */
#define OB_E_DIM (-2)      /* operand dimensions do not fit the operation */
#define OB_E_RANGE (-3)    /* row / label / slice / capacity out of range */
#define OB_E_NOTSCALAR (-4) /* backward root is not a 1-element node */
#define OB_E_OOM (-5)      /* the caller's arena is too small */
#define OB_E_STATE (-6)    /* call not valid in the current state, or an internal check failed */
#define OB_E_HIP (-7)      /* a HIP runtime call failed; see ob_last_error */
#define OB_E_ARG (-8)      /* null pointer or otherwise invalid argument */

/* operation codes of the graph data format */
#define OB_OP_INPUT 0      /* v = payload                                   */
#define OB_OP_LOOKUP 1     /* v = E[row, :]                                 */
#define OB_OP_MATVEC 2     /* v = W x (+ b)       shared W, b (Appendix A)   */
#define OB_OP_ADD 3        /* v = x_1 + ... + x_k                           */
#define OB_OP_CMULT 4      /* v = a * b component-wise                      */
#define OB_OP_TANH 5
#define OB_OP_SIGMOID 6
#define OB_OP_CONCAT 7     /* v = [x_1; ...; x_k]                           */
#define OB_OP_SLICE 8      /* v = x[lo:hi)                                  */
#define OB_OP_PICK_NLS 9   /* v = logsumexp(x) - x[label]  (scalar)         */
#define OB_OP_SQNORM 10    /* v = sum_i x_i^2               (scalar)         */

/* batching modes (Section 4.1: NoAuto / ByDepth / ByAgenda) */
#define OB_NOBATCH 0       /* one launch per node forward and per node backward */
#define OB_BYDEPTH 1       /* depth-based batching (Section 3.2)                */
#define OB_BYAGENDA 2      /* agenda-based batching (Section 3.2): signatures ranked by the average depth of their
                            * nodes (exact), then cheap before heavy operations, then first node id; at most 1024
                            * distinct signatures per graph, else OB_E_STATE at schedule time */
#define OB_MANUAL 3        /* manual batching (Section 2): the caller names the batch of every node with
                            * ob_set_manual_batches; signatures, depths and the agenda are not computed */

/* how the per-step launches are issued */
#define OB_LAUNCH_STREAM 0     /* one kernel launch per step on the stream            */
#define OB_LAUNCH_GRAPH 1      /* the per-step launches captured in a hipGraph        */
#define OB_LAUNCH_PERSISTENT 2 /* one cooperative kernel for all steps: not built, OB_E_STATE (a grid-wide barrier
                                * measured slower than a kernel boundary on this machine) */

/* ---- context ------------------------------------------------------------------------- */

/* arena_dev: device memory, at least 256-byte aligned; hip_stream: a hipStream_t (or NULL
 * for the default stream).  Touches no GPU state until the first upload. */
int ob_ctx_create(void *arena_dev, size_t arena_bytes, void *hip_stream, ob_ctx **out);
/* A second context over its own arena and stream that SHARES the parent's parameters (same
 * device storage for values and gradients; it cannot create parameters of its own).  Lets one
 * minibatch graph be uploaded and scheduled while another one executes (Section 3: graph
 * definition and batching are separate from computation).  The parent must outlive the fork, and
 * executions that touch the shared gradients must be ordered by the caller (e.g. same stream). */
int ob_ctx_fork(ob_ctx *parent, void *arena_dev, size_t arena_bytes, void *hip_stream, ob_ctx **out);
int ob_ctx_destroy(ob_ctx *ctx);
/* Upload and scheduling go to this stream instead of the context's stream; execution waits for
 * them through an event.  Call before the first upload. */
int ob_ctx_set_schedule_stream(ob_ctx *ctx, void *hip_stream);
/* A HIP stream whose kernels run on the compute units [first_cu, first_cu + n_cus) only (the device's units
 * are numbered 0 .. count - 1 in the order of hipExtStreamCreateWithCUMask's bit mask), at the default
 * priority.  For callers that give the schedule stream and the execution stream disjoint parts of the chip:
 * scheduling kernels that share compute units with the latency-bound execution launches slow those by about a
 * tenth, on parts of their own they do not.  The stream belongs to the caller (any context may use it, as its
 * stream or its schedule stream) and is released with ob_stream_destroy once no context uses it and its work
 * is done.  OB_E_ARG: empty range or one beyond the device's units; OB_E_HIP: the runtime refused. */
int ob_stream_create_on_cus(int first_cu, int n_cus, void **hip_stream_out);
int ob_stream_destroy(void *hip_stream);
int ob_ctx_set_mode(ob_ctx *ctx, int mode);
int ob_ctx_set_launch(ob_ctx *ctx, int launch);
/* Launch fusion (default 2; every batching mode): component-wise batches whose operands are
 * row-aligned with their producer batch run inside the producer's launch (Section 3.3: inputs
 * that are already contiguous and in order are used as they are), so a chain of such batches
 * costs one launch instead of one per depth level.  Batches and their order do not change.
 * on: 0 = one launch per depth level; 1 = fused, every batch launched as early as its operands
 * allow; 2 = fused, every batch launched as late as its consumers allow (batches off the longest
 * dependency path then share the launches next to their consumers).  Other values: OB_E_ARG. */
int ob_ctx_set_fusion(ob_ctx *ctx, int on);
/* Library-owned message for the last failing call on this context (valid until the next
 * call); ctx may be NULL for errors of ob_ctx_create. */
const char *ob_last_error(ob_ctx *ctx);

/* ---- parameters (persist across graphs) ------------------------------------------------- */

/* host_init: rows*cols fp32, row-major (host).  Writes the new parameter id to *id.
 * Parameters must be created before the first graph is uploaded. */
int ob_param_create(ob_ctx *ctx, int rows, int cols, const float *host_init, int *id);
int ob_param_write(ob_ctx *ctx, int id, const float *host_data);
int ob_param_read(ob_ctx *ctx, int id, float *host_out, size_t cap);
/* Gradients accumulate over ob_backward calls until zeroed. */
int ob_param_grad_zero(ob_ctx *ctx);
int ob_param_grad_read(ob_ctx *ctx, int id, float *host_out, size_t cap);
/* The update of Section 2's training loop, plain gradient descent: every parameter becomes
 * parameter - lr * gradient, queued on the context's stream behind the backward pass (contexts
 * forked from one another share the parameters, so one call updates them for all).  zero_grad != 0
 * also clears the gradients in the same pass.  OB_E_STATE before the first upload of a graph. */
int ob_param_sgd_step(ob_ctx *ctx, float lr, int zero_grad);

/* ---- graph definition (Section 3.1; host only, nothing is computed) ---------------------- */

int ob_graph_new(ob_ctx *ctx); /* drops all nodes, keeps parameters and their gradients */
int ob_graph_size(ob_ctx *ctx, int *n_nodes, int *n_edges);

int ob_add_input(ob_ctx *ctx, int dim, const float *host_data);
int ob_add_lookup(ob_ctx *ctx, int table, int row);
int ob_add_matvec(ob_ctx *ctx, int w, int bias_or_neg1, int x);
int ob_add_unary(ob_ctx *ctx, int op, int x);                 /* OB_OP_TANH, OB_OP_SIGMOID */
int ob_add_nary(ob_ctx *ctx, int op, int k, const int *xs);   /* OB_OP_ADD, OB_OP_CMULT (k=2), OB_OP_CONCAT */
int ob_add_slice(ob_ctx *ctx, int x, int lo, int hi);
int ob_add_pick_nls(ob_ctx *ctx, int x, int label);
int ob_add_sqnorm(ob_ctx *ctx, int x);

/* Appends n nodes given as flat arrays (all host).  in_off has n+1 entries, relative to
 * this call's in_idx; in_idx holds absolute node ids (existing nodes or earlier nodes of
 * this call).  aux0: LOOKUP row, SLICE lo, PICK_NLS label, INPUT offset into `payload`;
 * aux1: SLICE hi.  out_dim is checked against the dimension the operation implies.
 * Returns the id of the first appended node.  On error no node is appended. */
int ob_add_bulk(ob_ctx *ctx, int n, const uint8_t *op, const uint32_t *out_dim,
                const uint32_t *in_off, const uint32_t *in_idx, const int32_t *param,
                const int32_t *bias, const int32_t *aux0, const int32_t *aux1,
                const float *payload, size_t payload_len);

/* Manual batching (Section 2: the programmer groups by hand the operations that run together).
 * batch_of_node (host, copied) holds one label per node of the current graph, n = its node count:
 * nodes with equal labels form one batch, batches run in ascending label order, the nodes of a
 * batch keep ascending id order.  Labels need not be dense.  Checked here, on the host: labels are
 * >= 0, every operand's label is smaller than its consumer's, and all nodes of a batch agree in
 * operation, dimensions, arity, shared parameters, slice range and operand dimensions (else
 * OB_E_ARG, naming the node).  Used by OB_MANUAL only; adding nodes afterwards or ob_graph_new
 * drops the labels, and scheduling in OB_MANUAL without labels for every scheduled node fails with
 * OB_E_STATE. */
int ob_set_manual_batches(ob_ctx *ctx, const int32_t *batch_of_node, size_t n);

/* ---- execution ------------------------------------------------------------------------------ */

/* Copies pending nodes to the device (asynchronous).  Implied by ob_forward. */
int ob_upload(ob_ctx *ctx);
/* Evaluates every node with id <= node (Section 3.1: evaluation happens when a value is
 * requested).  Schedules on the GPU (Section 3.2), then runs the batches in order
 * (Section 3.3).  Asynchronous except for one small read of the schedule header.
 * When nodes [0, k) already have values (an earlier ob_forward of a smaller id, before or after
 * more nodes were added), only the nodes [k, node] are evaluated, as a stage of their own
 * (Section 3.1): they form a graph whose leaves are the earlier nodes they read (values copied on
 * the GPU), which is scheduled in the context's mode and executed in the arena behind the earlier
 * evaluations; depths of a stage count from its own leaves.  Earlier values stay readable
 * throughout (ob_value_read, ob_all_read).  While values come from more than one stage:
 * ob_schedule_read and ob_stats_read describe the last stage; ob_debug_read fails with OB_E_STATE;
 * ob_backward runs over the stages as they are (see there).
 * If the arena has no room for another stage, or in OB_MANUAL, the whole prefix is evaluated
 * again instead.  A schedule that was never executed is dropped when nodes are added. */
int ob_forward(ob_ctx *ctx, int node);
/* Only the scheduling half of ob_forward (upload, Section 3.2's batching on the GPU, layout and
 * launch plan); a later ob_forward of the same node then only executes.  Blocks the host for one
 * small read of the schedule header. */
int ob_schedule(ob_ctx *ctx, int node);
/* Same, but only queues the scheduling work and returns; the next ob_schedule / ob_forward of
 * this context waits for it and reads the header.  Errors found on the GPU surface there. */
int ob_schedule_async(ob_ctx *ctx, int node);
/* Reverse-mode differentiation from a 1-element node that ob_forward covered: batches in
 * reverse order (Section 3.3).  Node gradients are overwritten, parameter gradients
 * accumulate.  After forwards in several stages (see ob_forward) nothing is evaluated again: the
 * stages run backward one after the other, last first, and what a stage computes for the earlier
 * nodes it read is handed down to them before their own stage runs.  This needs room in the arena
 * behind the last stage for one block of gradient size per earlier stage, and every parameter a
 * later stage uses must already occur in the first evaluation; otherwise (and never silently wrong)
 * everything evaluated so far is scheduled and evaluated once more as one graph first. */
int ob_backward(ob_ctx *ctx, int node);
int ob_sync(ob_ctx *ctx);
/* Forgets the schedule, values and gradients of the current graph but keeps its nodes (and
 * their device copy): the next ob_forward schedules and evaluates it again, e.g. after the
 * parameters changed (the update step of Section 2's training loop). */
int ob_reset(ob_ctx *ctx);

/* ---- reads (synchronise the stream) ---------------------------------------------------------- */

int ob_value_read(ob_ctx *ctx, int node, float *host_out, size_t cap);
int ob_grad_read(ob_ctx *ctx, int node, float *host_out, size_t cap);
/* All node values (which = 0) or node gradients (which = 1) concatenated in node-id order (gathered from every
 * evaluation stage; staging space comes from the free end of the arena, OB_E_OOM if there is none). */
int ob_all_read(ob_ctx *ctx, int which, float *host_out, size_t cap);

/* The schedule of the last ob_forward: batch b holds node_ids[batch_off[b] .. batch_off[b+1]).
 * batch_depth is the depth (OB_BYDEPTH), the agenda iteration (OB_BYAGENDA), the rank of the
 * batch's label (OB_MANUAL) or the step index (OB_NOBATCH); batch_sig is the 64-bit signature
 * hash (Appendix B) and is informational.  cap_batches / cap_nodes are the capacities of the
 * per-batch arrays (batch_off needs cap_batches + 1) and of node_ids.  After a forward that
 * evaluated a stage (see ob_forward) this is the stage's schedule: only its nodes, depths
 * counted from its leaves. */
int ob_schedule_read(ob_ctx *ctx, int *n_batches, int *batch_depth, uint64_t *batch_sig,
                     int *batch_off, int *node_ids, size_t cap_batches, size_t cap_nodes);

/* Counters and phase times of the last forward / backward. */
typedef struct ob_stats {
    int32_t n_nodes, n_edges, n_steps, n_batches;
    int32_t n_tiles_fwd, n_tiles_bwd_pull, n_tiles_bwd_dx, n_param_uses;
    int32_t n_launch_fwd, n_launch_bwd, n_launch_sched, n_slots;
    uint64_t value_floats, grad_floats, arena_used_bytes, upload_bytes;
    float ms_upload, ms_schedule, ms_forward, ms_backward; /* hipEvent times on the stream */
    float ms_param_grads, ms_graph_build;
    int32_t n_stages;  /* evaluations the current values come from (1: one schedule covers every evaluated node) */
    int32_t n_proxies; /* earlier nodes the last stage read (0 when n_stages is 1) */
    int32_t n_depth_retries; /* schedules of this context so far that were repeated with the single-workgroup depth pass
                              * because a range of the partitioned pass ran into the bound on its wait */
    int32_t n_launch_bwd_steps; /* launches of the backward step kernel alone (n_launch_bwd also counts the kernel that
                                 * places the root and the deferred parameter-gradient kernels) */
    int32_t n_view_batches;     /* SLICE batches: views, nothing is copied forward (Section 3.3) */
    int32_t n_uncopied_batches; /* CONCAT batches that only matrix products read: the products read the pieces where
                                 * they lie and the forward pass writes nothing for the batch (Section 3.3); their rows are
                                 * filled in when a value is read */
    uint64_t view_floats, uncopied_floats; /* elements of those batches (forward bytes saved: 8 per element) */
} ob_stats;
int ob_stats_read(ob_ctx *ctx, ob_stats *out);

/* Internal device tables of the last schedule, for stage-by-stage parity tests.
 * which: OB_DBG_*; elements are copied as 32-bit words (64-bit tables as two words each). */
#define OB_DBG_DEPTH 0     /* u32[n]  step (depth) per node        */
#define OB_DBG_SIG 1       /* u64[n]  signature hash per node      */
#define OB_DBG_SUCC_OFF 2  /* u32[n+1] successor CSR offsets       */
#define OB_DBG_SUCC_EDGE 3 /* u32[E]  edge ids sorted by producer  */
#define OB_DBG_ORDER 4     /* u32[n]  node ids in schedule order   */
#define OB_DBG_VAL_OFF 5   /* u32[n]  element offset of each node's row in the value arena */
#define OB_DBG_TILES_FWD 6 /* forward tile descriptors in launch order, 40 words each (internal layout) */
#define OB_DBG_TILES_PULL 7 /* backward pull tile descriptors in launch order, 48 words each (internal layout) */
#define OB_DBG_CHAINS 8    /* launch chains, 12 words each: first, members, slot, fused, groups, groups per block, blocks, tiles per block, forward tiles per block, 3 reserved */
#define OB_DBG_LORDER 9    /* u32 per batch: batch ids in launch order (the members of chain c are entries first .. first + members - 1) */
int ob_debug_read(ob_ctx *ctx, int which, uint32_t *host_out, size_t cap_words, size_t *n_words);
/* Internal knobs, for tests of the library's own error handling and of its alternative paths.  which: OB_DBG_SET_*;
 * unknown: OB_E_ARG. */
#define OB_DBG_SET_DEPTH_SPIN 0 /* idle polls a workgroup of the partitioned depth pass (Section 3.2) allows itself while it
                                 * waits for a lower id range, default 2^21; 0 makes every range that has to wait give up at
                                 * once, so that scheduling falls back to the single-workgroup pass (see n_depth_retries) */
#define OB_DBG_SET_CONCAT_COPY 1 /* nonzero: every CONCAT batch is copied by the forward pass from the next schedule on
                                  * (default 0: batches that only matrix products read stay uncopied, see ob_stats) */
int ob_debug_set(ob_ctx *ctx, int which, uint64_t value);

/* Stand-alone device primitives, exposed so that tests can check them directly.  All
 * pointers are host; the context's arena beyond its current use serves as scratch. */
int ob_test_sort(ob_ctx *ctx, size_t n, const uint64_t *keys, const uint32_t *vals, int lo_bit,
                 int n_bits, uint64_t *keys_out, uint32_t *vals_out);
int ob_test_scan(ob_ctx *ctx, size_t n, const uint32_t *in, uint32_t *out_exclusive,
                 uint32_t *total);
/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
 * forbid device allocation): the same stable radix sort as ob_test_sort, on the caller's DEVICE arrays,
 * in place, with every temporary (second key / value buffers, digit tables, scan sums) in a fixed
 * array inside the library's device image (about 3.5 MiB per GPU, held until the process ends).  The
 * call allocates nothing on the host or the device, needs no context, and only queues work on
 * hip_stream (a hipStream_t, NULL = default stream): the result is in keys_dev / vals_dev once the
 * stream gets there.  Sorts the n pairs stably by bits [lo_bit, lo_bit + n_bits) of the key.
 * n > OB_NOALLOC_MAX_PAIRS: OB_E_RANGE, nothing is queued.  Bad bit range or null array: OB_E_ARG.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or host threads) race and must be ordered by the caller.  Message: ob_last_error(NULL). */
#define OB_NOALLOC_MAX_PAIRS 262144
int ob_sort_pairs_noalloc(void *hip_stream, size_t n, uint64_t *keys_dev, uint32_t *vals_dev, int lo_bit, int n_bits);
/* Average duration in microseconds of n back-to-back launches of an empty kernel (touch = 0) or
 * of a kernel whose one thread does a dependent load and store (touch = 1) on the context's
 * stream: the floor of a launch boundary on this machine, reported by the benchmark. */
int ob_test_launch_cost(ob_ctx *ctx, int n, int touch, float *us_per_launch);
/* C[M x N] = A[M x K] * B[N x K]^T through the library's MFMA tile routine. */
int ob_test_gemm(ob_ctx *ctx, int M, int N, int K, const float *A, const float *B, float *C);

#ifdef __cplusplus
}
#endif
#endif /* OB_H */
