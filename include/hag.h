/*
 * libhag -- GNN neighbourhood set-aggregation over a Hierarchically Aggregated
 * computation Graph (HAG) on AMD MI355X (gfx950).  C ABI.
 *
 * Vocabulary (paper, Section 3.1): V are the nodes of the input graph, N(v) the
 * in-neighbour set of v, V_A the aggregation nodes a HAG adds, Nhat_v the
 * in-neighbours of v in the HAG (a mix of original and aggregation nodes).
 *
 * Graph layout.  CSR with rows = destinations and columns = in-neighbours
 * (Section 3.1: an edge (u,v) means computing v needs u):
 *     rowptr  int64 [n+1], col  int32 [rowptr[n]], 0 <= col < n.
 * A neighbourhood is a set: a duplicate inside one row is an error unless
 * HAG_SEARCH_DEDUP is given.  Self-loops and isolated nodes are legal.  The
 * graph need not be symmetric; the backward pass uses the true transpose.
 *
 * Unified ids.  Original nodes are 0..n-1.  Aggregation nodes are n..n+a-1.
 * Two numberings exist: "creation order" (the order Algorithm 3 created them,
 * used by hag_from_merges / hag_get_merges) and "level order" (sorted by depth,
 * stable; used by hag_get_forward and on the device).
 *
 * Feature layout.  Row-major [n, d] matrices, row stride d elements, base
 * pointer 16-byte aligned, d a positive multiple of 4 (other d: HAG_EINVAL).
 * dtype f32 or i32.  int32 sums wrap modulo 2^32.
 *
 * Semantics taken where the paper is silent:
 *   empty N(v): sum 0, mean 0, max 0 with argmax -1 (and no gradient);
 *   mean = sum / |N(v)| with the degree of the INPUT graph (not of the HAG);
 *   max ties go to the smallest original node id; argmax holds original ids.
 *
 * Ownership.  The library owns hag_t and every array returned by a getter (valid
 * until hag_free).  The caller owns all arrays it passes in; host arrays are
 * copied during the call.  Device arrays (x, y, gy, gx, argmax, workspace) are
 * caller-owned device memory and must not alias each other.
 *
 * Memory kind.  Device arrays must be ordinary device memory (hipMalloc: coarse-grained).  The
 * max backward pass accumulates with hardware floating-point atomics, which fine-grained or
 * host-mapped memory does not support.
 *
 * Environment.  The launch path never reads the environment.  Tuning and test knobs (HAG_* variables,
 * listed in the project documentation) are read once, when a handle is built.
 *
 * Execution.  Device entry points enqueue kernels on `stream` (a hipStream_t
 * passed as void*, NULL = the default stream) and return without synchronising;
 * they allocate nothing.  All functions return a status (0 = HAG_OK); the
 * message of the last failure on the calling thread is hag_last_error().
 */
#ifndef HAG_H
#define HAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hag_handle hag_t; /* opaque; immutable after construction except hag_upload and hag_set_option */

/* Table 1, set Aggregate.  HAG_GCN is the GCN row's Update up to the weight matrix, fused
 * into the aggregation: y[v] = (sum over N(v) of x[u] + x[v]) / (|N(v)| + 1); f32 only. */
typedef enum { HAG_SUM = 0, HAG_MEAN = 1, HAG_MAX = 2, HAG_GCN = 3 } hag_op_t;
typedef enum { HAG_F32 = 0, HAG_I32 = 1 } hag_dtype_t;

enum {
    HAG_OK = 0,
    HAG_EINVAL = -1,  /* bad argument (message says which) */
    HAG_ENOMEM = -2,  /* host or device allocation failed */
    HAG_EHIP = -3,    /* a HIP runtime call failed (message holds the HIP error string) */
    HAG_ESTATE = -4,  /* device entry point called before hag_upload */
    HAG_ETIMEOUT = -5 /* hag_check: a one-launch pass gave up waiting; its output is not valid */
};

enum {
    HAG_SEARCH_CANONICAL = 1, /* among pairs of maximal redundancy take the lexicographically
                                 smallest (smaller id, larger id), which makes the result unique.
                                 The search always does this; the flag is accepted and ignored. */
    HAG_SEARCH_DEDUP = 2,     /* drop duplicate neighbours instead of rejecting them */
    HAG_SEARCH_DEVICE = 4     /* hag_search only: count co-occurrences (Redundancy of Algorithm 3) on the
                                 current HIP device instead of on the host threads.  The result is the
                                 same HAG, merge for merge.  The call allocates device memory of about
                                 12 bytes per edge + 128 bytes per (node + capacity) and pinned host
                                 memory of 4 bytes per edge for its duration, uses a stream of its own and
                                 returns when the search is done; HAG_EHIP if there is no device. */
};

typedef struct hag_stats {
    int64_t n;            /* |V| */
    int64_t e;            /* |E|, directed edges of the input graph */
    int64_t a;            /* |V_A| */
    int64_t levels;       /* depth of the deepest aggregation node (0 if a == 0) */
    int64_t h;            /* sum over v in V of |Nhat_v| (edges of the final gather) */
    int64_t e_hag;        /* |E^| = h + 2a */
    int64_t aggr_naive;   /* binary aggregations on the GNN-graph: sum max(|N(v)|-1, 0)   (Section 4.1) */
    int64_t aggr_hag;     /* the same count on the HAG: sum over V and V_A of max(|Nhat|-1, 0) */
    int64_t xfer_naive;   /* neighbour-row transfers on the GNN-graph = |E|              (Section 5.4) */
    int64_t xfer_hag;     /* neighbour-row transfers on the HAG = |E^| */
    int64_t max_degree;   /* largest |N(v)| */
    int64_t max_hag_degree; /* largest |Nhat_v| */
    int64_t stages;       /* kernel launches the aggregation nodes take (runs of fused levels) */
    int64_t components;   /* number of contiguous id ranges that no edge crosses, if the graph is a batch of
                             small graphs that the one-launch component-local pass can serve; else 0 */
} hag_stats_t;

/* ---------------------------------------------------------------- host ---- */

/* Algorithm 3 for a set Aggregate: starting from the GNN-graph, repeatedly take
 * the pair (v1, v2) of HAG nodes that the largest number of original nodes
 * aggregate together (Redundancy), create an aggregation node w = v1 (+) v2 and
 * replace the pair by w in every list holding both; stop at `capacity`
 * aggregation nodes or when the best redundancy is <= 1 (such a merge saves
 * nothing; the listing's loop would not terminate there).
 * max_depth > 0 forbids aggregation nodes deeper than that (0 = no limit; the
 * paper has no such limit).  All pointers are host memory.  *out receives a new
 * handle (free with hag_free).  Errors: HAG_EINVAL for n < 0, capacity < 0,
 * non-monotone rowptr, col out of range, duplicates without HAG_SEARCH_DEDUP,
 * n + capacity >= 2^31; HAG_ENOMEM; HAG_EHIP (HAG_SEARCH_DEVICE only: no device, or a
 * HIP call failed). */
int hag_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity,
               uint32_t flags, int32_t max_depth, hag_t **out);

/* The same search run independently on each of n_graphs disjoint graphs that
 * share one block-diagonal CSR (graph g owns nodes graph_ptr[g]..graph_ptr[g+1]-1
 * and no edge crosses graphs), each with its own capacity
 * floor(capacity_fraction * nodes of the graph); the results are concatenated in
 * graph order.  Used for batches of small graphs (graph classification). */
int hag_search_batched(int64_t n, const int64_t *rowptr, const int32_t *col,
                       int64_t n_graphs, const int64_t *graph_ptr, double capacity_fraction,
                       uint32_t flags, int32_t max_depth, hag_t **out);

/* Build a handle from an explicit merge list in creation order: aggregation node
 * n+i aggregates left[i] and right[i] (unified creation-order ids < n+i), and
 * replaces that pair in every Nhat_u that holds both at that point -- the rewrite
 * loop of Algorithm 3.  HAG_EINVAL if an id is out of range, left[i] == right[i],
 * or a merge is used by no list. */
int hag_from_merges(int64_t n, const int64_t *rowptr, const int32_t *col,
                    int64_t n_merges, const int32_t *left, const int32_t *right,
                    uint32_t flags, hag_t **out);

/* New handle holding only the first n_merges merges of h (greedy with a fixed
 * tie-break is prefix-stable, so this is the HAG of a smaller capacity). */
int hag_prefix(const hag_t *h, int64_t n_merges, hag_t **out);

/* Algorithm 3 for a SEQUENTIAL Aggregate (ordered neighbour lists, e.g. an LSTM aggregator): only common
 * prefixes can be shared (Section 3.1), Redundancy(v1, v2) is the number of nodes whose current list
 * starts with (v1, v2) (the sequential branch of Redundancy in the listing), and a merge replaces that
 * leading pair by a new node w in exactly those lists, w standing for the ordered cover
 * (cover(v1), cover(v2)) of Equation 2.  Stops at `capacity` merges or when the best redundancy is <= 1;
 * ties go to the lexicographically smallest (v1, v2).  With capacity >= |E| the result has the fewest
 * aggregations any equivalent HAG can have (Theorem 3).  Host only; hag_seq_create below builds on it.
 * In: rowptr [n+1], col [rowptr[n]]: row v is the ORDERED list N(v) (a node may occur more than once).
 * Out (caller arrays): left/right/redundancy [min(capacity, rowptr[n])]: merge i created node n+i from
 * (left[i], right[i]) with that redundancy; *n_merges; hrowptr [n+1], hcol [rowptr[n]]: the final
 * ordered lists (only a list's first entry can be an aggregation node).  HAG_EINVAL on malformed input. */
int hag_seq_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity,
                   int64_t *n_merges, int32_t *left, int32_t *right, int32_t *redundancy,
                   int64_t *hrowptr, int32_t *hcol);

/* Device path for a sequential Aggregate: an LSTM aggregator over ORDERED neighbour lists (Section 3.1),
 *     (h_0, c_0) = 0,  (h_t, c_t) = cell(x[u_t], h_{t-1}, c_{t-1}) for N(v) = (u_1, ..., u_k),  a_v = h_k
 * (a_v = 0 for an empty list), cell = the standard LSTM step: gates = w_ih x + w_hh h + b split into
 * input, forget, cell and output gate, c' = sigmoid(f) c + sigmoid(i) tanh(g), h' = sigmoid(o) tanh(c').
 * hag_seq_create (host): capacity > 0 runs hag_seq_search with that capacity and plans the evaluation of
 * the resulting prefix HAG respecting the order of Algorithm 2 -- every shared prefix (an aggregation node
 * of Equation 2's ordered cover, or the one-element prefix a list or a merge starts from) is evaluated once,
 * before whatever continues from it, and every node continues from the state of its list's head; capacity = 0
 * plans the plain lists with nothing shared (the baseline).  rowptr [n+1], col [rowptr[n]] as for hag_seq_search.
 * hag_seq_cells: cell evaluations of one pass; hag_seq_ranks: the longest chain of dependent evaluations;
 * hag_seq_launches: cell-kernel launches of one forward pass under the handle's options (1 for the one-launch
 * pass, else the levels of hag_seq_get_plan); hag_seq_merges: aggregation nodes.  hag_seq_upload copies the plan
 * to the current device (once).
 * hag_seq_lstm_forward (device pointers, fp32; inference, the training pair is further down): x [n, d],
 * w_ih [4H, d], w_hh [4H, H], b [4H] with gate-major rows (input, forget, cell, output), a_out [n, H], workspace of
 * hag_seq_workspace_bytes(h, d, H) bytes (16-byte aligned; packed weights, one (h, c) state row and one flag
 * per shared prefix).  d a multiple of 4, H a multiple of 8 up to 128, d + H <= 256 (H <= 64 with d + H <= 128
 * keeps the packed weights in registers; beyond that every wavefront streams its part of them from the L2 cache
 * once per step).  Enqueues on `stream` and returns; allocates nothing.  HAG_ESTATE before hag_seq_upload,
 * HAG_EINVAL otherwise. */
typedef struct hag_seq hag_seq_t;
int hag_seq_create(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity, hag_seq_t **out);
void hag_seq_free(hag_seq_t *h);
int64_t hag_seq_cells(const hag_seq_t *h);
int64_t hag_seq_ranks(const hag_seq_t *h);
int64_t hag_seq_launches(const hag_seq_t *h);
int64_t hag_seq_merges(const hag_seq_t *h);
/* The plan as the device executes it (host arrays owned by the handle, valid until hag_seq_free; any out
 * pointer may be NULL): the shared prefixes and the nodes' remainders cut into PATHS -- a path carries its
 * running (h, c) from step to step on chip -- in groups such that a path starts only from a state that a path
 * of an EARLIER group writes.  order 0: groups are levels (level 0 starts from the zero state, level l + 1
 * from states that level l writes), the order of one launch per level; order 1: groups are the depths of the
 * start states (evaluations behind them), the order of the one-launch pass.  paths [4 * n_paths]: (state row
 * it starts from or -1 for the zero state, first step, steps, node whose a_v is its last h or -1), group by
 * group, longest first; level_ptr [n_levels + 1]: the groups, in paths; step_x / step_out [hag_seq_cells]
 * (the same for both orders): per step the input row and the state row the step's (h, c) is written to or
 * -1; final_state [n]: the state row holding a_v, -1 for an empty list, -2 where a path writes a_v itself. */
int hag_seq_get_plan(const hag_seq_t *h, int32_t order, int64_t *n_states, int64_t *n_paths, const int32_t **paths,
                     const int32_t **step_x, const int32_t **step_out, int64_t *n_levels, const int64_t **level_ptr,
                     const int32_t **final_state);
int hag_seq_upload(hag_seq_t *h);
/* With more than one level, hag_seq_lstm_forward runs all of them in ONE launch when every workgroup of it
 * can be resident at once (paths in order 1 of hag_seq_get_plan): a tile of paths waits (polling a per-state
 * flag, at most HAG_OPT_SPIN_LIMIT times, default 2^21, about half a microsecond apart) until the states it starts from are written, by tiles that come
 * before it and never wait for it.  hag_seq_set_option (host state only; later calls): HAG_OPT_SEQ_ONE_LAUNCH
 * (default 1, or the environment's HAG_SEQ_ONE_LAUNCH when the handle was built; 0 = one launch per level, no
 * waits), HAG_OPT_SPIN_LIMIT, HAG_OPT_TEST_WAIT_UNREACHABLE (tests only: no flag is ever set, so every wait
 * gives up).  hag_seq_check synchronises `stream` and returns HAG_OK, or HAG_ETIMEOUT if a wait on this handle
 * gave up since the last check (its output is not valid; the state is cleared).
 * The one-launch pass fills the device with workgroups that may wait for one another, which is safe because all of
 * them are resident; two such passes running at the same time on one device (two streams, two processes) can each
 * hold the places the other's remaining workgroups need, and then both time out.  Callers that overlap passes on
 * one device set HAG_OPT_SEQ_ONE_LAUNCH to 0. */
int hag_seq_set_option(hag_seq_t *h, int32_t option, int64_t value);
int hag_seq_check(const hag_seq_t *h, void *stream);
size_t hag_seq_workspace_bytes(const hag_seq_t *h, int64_t d, int64_t hidden);
int hag_seq_lstm_forward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih,
                         const float *w_hh, const float *b, float *a_out, void *workspace, void *stream);

/* Training with the LSTM aggregator (the sizes of hag_seq_lstm_forward).
 * hag_seq_lstm_forward_train is hag_seq_lstm_forward that also keeps, in `workspace`
 * (hag_seq_train_workspace_bytes(h, d, hidden) bytes, 16-byte aligned), what the backward pass needs of every cell: the
 * activated gates, c and h (24 H bytes per cell evaluation), besides the states of the shared prefixes.
 * hag_seq_lstm_backward, called after it with the same handle, sizes, x, w_ih, w_hh and workspace (nothing else may have
 * used the workspace in between), backpropagates through time along the plan's paths, last step first: given g_a [n, H], the
 * gradient of a loss with respect to a_out, it writes the gradients g_x [n, d], g_w_ih [4H, d], g_w_hh [4H, H], g_b [4H]
 * (the layouts of x, w_ih, w_hh, b).  A shared prefix is differentiated once, with the gradients of everything that
 * continues from it added up first (fp32 atomics: the last bits of g_x and of the weight gradients depend on the order in
 * which those arrive).  Both calls follow HAG_OPT_SEQ_ONE_LAUNCH: by default the backward pass too is one launch in
 * which a path waits, bounded, until everything that continues from a state has sent its gradients (hag_seq_check reports a
 * wait that gave up).  Device pointers, fp32; enqueues on `stream` and returns; allocates nothing. */
size_t hag_seq_train_workspace_bytes(const hag_seq_t *h, int64_t d, int64_t hidden);
int hag_seq_lstm_forward_train(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih,
                               const float *w_hh, const float *b, float *a_out, void *workspace, void *stream);
int hag_seq_lstm_backward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                          const float *g_a, float *g_x, float *g_w_ih, float *g_w_hh, float *g_b, void *workspace,
                          void *stream);

void hag_free(hag_t *h);

int hag_stats(const hag_t *h, hag_stats_t *out);

/* Merge list in creation order; redundancy[i] = number of lists rewritten by merge i. */
int hag_get_merges(const hag_t *h, int64_t *n_merges, const int32_t **left, const int32_t **right,
                   const int32_t **redundancy);

/* Level-ordered forward form (what the device executes):
 *   agg_left/right [a]: inputs of aggregation node n+i, level-order ids;
 *   level_ptr [levels+1]: nodes n+level_ptr[l-1] .. n+level_ptr[l]-1 have depth l;
 *   hrowptr [n+1], hcol [h]: Nhat_v for v in V, level-order ids, ascending per row.
 * Any out pointer may be NULL. */
int hag_get_forward(const hag_t *h, const int32_t **agg_left, const int32_t **agg_right,
                    const int32_t **level_ptr, int32_t *n_levels,
                    const int64_t **hrowptr, const int32_t **hcol);

/* ------------------------------------------------------------- device ---- */

/* Copy the index arrays and launch schedules of h to the current device (once per
 * handle; allocates device memory that hag_free releases; synchronises). */
int hag_upload(hag_t *h, void *stream);

/* Bytes of caller-provided scratch that hag_forward / hag_backward need for this
 * op, dtype and d (aggregation-node rows, partial sums of split rows).  The
 * contents need not survive between calls: nothing is memorised for the backward
 * pass except argmax (Algorithm 2's caption). */
size_t hag_workspace_bytes(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d);

/* Algorithm 2 without the Update line: aggregation nodes level by level, then
 * y[v] = Aggregate over Nhat_v for every v in V.  x, y: device [n, d].
 * argmax: device int32 [n, d], required for HAG_MAX, ignored otherwise.
 * HAG_MEAN and HAG_GCN require HAG_F32. */
int hag_forward(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                const void *x, void *y, int32_t *argmax, void *workspace, void *stream);

/* Transposed pass (the hag_aggregate_grad operation of Section 5.1; by the
 * definition of equivalence in Section 3.2 it must return the gradient of the
 * naive aggregation): gx[u] = sum over consumers of u.  sum/mean run over the
 * transposed HAG, deepest level first; max uses only argmax
 * (gx[argmax[v,f], f] += gy[v,f], hardware atomics: fp32 order not fixed).
 * gx is overwritten. */
int hag_backward(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                 const void *gy, const int32_t *argmax, void *gx, void *workspace, void *stream);

/* The one-launch schedule (optional, off by default).  hag_forward and hag_backward can run
 * Algorithm 2's loop over V_A and its final loop (resp. their transposes) as ONE kernel launch:
 * workgroups draw units of work, phase by phase, from a device-wide ticket counter, and a unit of
 * a later phase waits, inside the kernel, until every unit of the earlier phases has been counted as
 * finished.  The wait is bounded; if it ever gives up the pass still runs to its end (every access
 * in bounds) but its output is not valid, and hag_check reports it.  The pass keeps a few words of
 * device state per handle, so while this schedule is in use calls on ONE handle must not overlap in
 * time (enqueue them on one stream, or order the streams).  It is taken when: no row is cut into
 * pieces, d <= 256, at most 7 stages, and the pass has at most HAG_OPT_ONE_LAUNCH_MAX_ITEMS rows.
 * On MI355X it is slower than one launch per stage (a device-wide atomic update of one address
 * completes about every 9 ns whoever issues it, and a pass needs one per unit of work; rows handed
 * from one phase to the next must bypass the per-XCD L2s), hence off by default.
 *
 * hag_set_option changes a handle's launch options (host state only; affects later calls):
 *   HAG_OPT_ONE_LAUNCH_MAX_ITEMS  largest pass, in rows, that takes the one-launch schedule (0 = never, the
 *                                 default; the environment's HAG_FUSE_MAX_ITEMS when the handle was built);
 *   HAG_OPT_SPIN_LIMIT            polls, about a microsecond apart, after which a wait gives up (default 262144);
 *   HAG_OPT_TEST_WAIT_UNREACHABLE tests only: every wait is for a count that cannot be reached, so it gives up
 *                                 after the spin limit and hag_check must report HAG_ETIMEOUT;
 *   HAG_OPT_PARTITION_SHIFT       0..7: in a launch whose long rows are cut into 8 classes of source ids, workgroup b takes
 *                                 the sources of class (b + shift) mod 8 (any value gives the same results);
 *   HAG_OPT_DETERMINISTIC_MAX_BACKWARD  non-zero: the backward pass of max adds up in a fixed order
 *                                 (a gather over the transposed input graph filtered by argmax) instead
 *                                 of with atomics; slower, bit-reproducible.
 * hag_check synchronises `stream` and returns HAG_OK, or HAG_ETIMEOUT if a one-launch pass on this handle
 * gave up waiting since the last check (and clears that state). */
enum { HAG_OPT_ONE_LAUNCH_MAX_ITEMS = 1, HAG_OPT_SPIN_LIMIT = 2, HAG_OPT_TEST_WAIT_UNREACHABLE = 3,
       HAG_OPT_DETERMINISTIC_MAX_BACKWARD = 4, HAG_OPT_PARTITION_SHIFT = 5, HAG_OPT_SEQ_ONE_LAUNCH = 6 };
int hag_set_option(hag_t *h, int32_t option, int64_t value);
int hag_check(const hag_t *h, void *stream);

/* The same two calls restricted to some of their phases, for per-kernel timing: a later
 * phase reads what an earlier call left in `workspace`.  HAG_PHASE_LEVELS = the
 * aggregation-node levels (forward: Algorithm 2's loop over V_A; backward: their
 * gradient rows); HAG_PHASE_GATHER = the per-node gather over V; HAG_PHASE_FOLD = the small
 * launches that add up the partial rows of rows that were cut into pieces. */
enum { HAG_PHASE_LEVELS = 1, HAG_PHASE_GATHER = 2, HAG_PHASE_FOLD = 4, HAG_PHASE_ALL = 7 };
int hag_forward_phases(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                       const void *x, void *y, int32_t *argmax, void *workspace, void *stream,
                       uint32_t phases);
int hag_backward_phases(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                        const void *gy, const int32_t *argmax, void *gx, void *workspace, void *stream,
                        uint32_t phases);

/* The GNN-graph baseline (Algorithm 1's Aggregate line; a HAG with V_A empty):
 * same arguments, same kernels, run on the input CSR and its transpose. */
int hag_naive_forward(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                      const void *x, void *y, int32_t *argmax, void *workspace, void *stream);
int hag_naive_backward(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                       const void *gy, const int32_t *argmax, void *gx, void *workspace, void *stream);

/* For callers that cannot allocate or hand over scratch memory (code under HIP graph capture
 * that owns no buffer pool, tight serving loops, harnesses that forbid hipMalloc): hag_forward
 * with the workspace taken from a fixed device array inside the library instead of from the
 * caller.  The array holds HAG_STATIC_SCRATCH_BYTES per GPU from the moment the library is loaded
 * until the process ends.  HAG_EINVAL (nothing is launched) when
 * hag_workspace_bytes(h, op, dtype, d) exceeds it; HAG_ESTATE before hag_upload.  The call
 * allocates nothing, on the host or on the device.  All calls on one GPU share the one array:
 * calls that may overlap in time (different streams, different threads) race on it and must be
 * serialised by the caller; its contents are left over from the last call and nothing is
 * expected of them (every row of it that a pass reads was written by that pass before). */
#define HAG_STATIC_SCRATCH_BYTES (64u << 20)
int hag_forward_static_scratch(const hag_t *h, hag_op_t op, hag_dtype_t dtype, int64_t d,
                               const void *x, void *y, int32_t *argmax, void *stream);

/* Algorithmic bytes one call moves (every HAG edge one row read, every produced
 * row one write, plus index reads), for roofline accounting.  which: 0 hag_forward,
 * 1 hag_backward, 2 hag_naive_forward, 3 hag_naive_backward. */
int64_t hag_algorithmic_bytes(const hag_t *h, int which, hag_op_t op, int64_t d);

/* Measurement helpers (nothing of the paper's method): kernels that only move bytes in the
 * access shape of the aggregation kernels, so that a benchmark run can state the ceilings its
 * roofline fractions are measured against.
 * hag_probe_rows: every sub-group of lanes (as many lanes as a row of d fp32 features has
 * 16-byte vectors, a power of two from 4 to 64) of `workgroups` 256-thread workgroups reads
 * `reads` pseudo-random rows of the device matrix src [n_rows, d] (n_rows a power of two,
 * d a multiple of 4 up to 256, reads a multiple of 4) and writes its sum to sink (device,
 * workgroups * 1024 floats).  The matrix size decides which memory level serves the rows;
 * from_lds = 1 copies as many rows as fit 16 KB into LDS first and reads those instead;
 * from_lds = 2 adds a row held in registers into pseudo-random LDS rows instead (each sub-group
 * into rows of its own: 16-byte read, add, 16-byte write), from_lds = 3 does the same with LDS
 * atomic adds: what accumulators kept in LDS cost per row.
 * Returns the number of row bytes read or accumulated (>= 0) or a negative status.
 * hag_probe_copy: dst[0..bytes) = src[0..bytes), device pointers, 16-byte granularity.
 * hag_probe_mfma_f32: every wavefront of `workgroups` 256-thread workgroups issues iters x 4 independent
 * v_mfma_f32_32x32x2_f32 on register operands and writes a checksum to sink (device, workgroups * 256
 * floats); returns the flops of the launch: the fp32 matrix-core rate the LSTM aggregator is priced against. */
int64_t hag_probe_rows(const void *src, int64_t n_rows, int64_t d, int64_t reads, int32_t from_lds,
                       int64_t workgroups, void *sink, void *stream);
int hag_probe_copy(const void *src, void *dst, int64_t bytes, void *stream);
int64_t hag_probe_mfma_f32(int64_t iters, int64_t workgroups, void *sink, void *stream);

const char *hag_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HAG_H */
