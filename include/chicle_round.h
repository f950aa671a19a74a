/*
 * chicle_round.h - C ABI of the CoCoA round for generalised linear models on one MI355X.
 *
 * One round (paper Section 2.2 "CoCoA", Eq. 1 and Eq. 2; trainer/solver protocol of
 * Section 4.1-4.2; Section 5.1 "CoCoA" for the hyper-parameters) is
 *
 *     K local solvers each make one stochastic-coordinate pass (L = 1, H = all local samples)
 *     over the rows of the data chunks they own, starting from the shared vector w
 *  -> their updates Delta w_k are combined into w (adding; sigma = K makes the plain sum safe)
 *  -> the duality gap P(w) - D(alpha) is evaluated.
 *
 * Problem solved:   P(w) = lambda/2 |w|^2 + 1/n sum_i loss_i(x_i . w)
 *                   D(a) = -lambda/2 |w(a)|^2 - 1/n sum_i loss_i^*(-a_i),  w(a) = 1/(lambda n) sum_i a_i s_i x_i
 *   hinge   : loss_i(z) = max(0, 1 - y_i z), y_i in {-1,+1}, s_i = y_i, a_i in [0,1]
 *   squared : loss_i(z) = (z - y_i)^2 / 2,  s_i = 1,  a_i real
 *   logistic: loss_i(z) = log(1 + exp(-y_i z)), y_i in {-1,+1}, s_i = y_i, a_i in [0,1]; its coordinate
 *             step has no closed form: the scalar equation is solved numerically (a wavefront evaluates it at
 *             64 points of a bracket and narrows the bracket 63-fold per evaluation)
 *
 * Data live in HBM as chunks (Section 3 "Uni-tasks", Section 4.4 "In-memory chunk data
 * format"): a chunk is one contiguous block holding a run of rows (CSR or dense) together with
 * its per-row state (label, dual variable alpha, squared norm).  Chunks are the unit that the
 * scheduler hands to solvers; the state always stays inside its chunk.  The ownership contract
 * of Section 3 is enforced as a state machine:
 *
 *     LOADING --assign--> READY --local_epoch--> EPOCH_DONE --aggregate--> READY
 *
 *   - between iterations (READY, LOADING) the scheduler owns the chunks: load, assign, set_alpha,
 *     set_w are legal;
 *   - during an iteration (EPOCH_DONE: the solvers' updates are not merged yet) they are not.
 *
 * Conventions
 *   - every function returns CHICLE_OK (0) or a negative chicle_status; nothing throws or aborts;
 *     chicle_last_error() gives a message for the last failure on that context;
 *   - "host" pointers are ordinary CPU memory, read or written before the call returns; the caller
 *     keeps ownership;  "device" pointers are HBM addresses valid on the context's GPU;
 *   - columns are addressed by the caller's ids in every call; inside the chunk store sparse columns
 *     are renumbered by popularity (done once, at the first assign), which the get/set calls undo;
 *   - the library allocates no device memory: it carves everything out of the arena handed to
 *     chicle_create (size it with chicle_arena_bytes); the arena and the HIP stream are borrowed for
 *     the lifetime of the context; all work is enqueued on that stream; the context itself holds 32 bytes
 *     of pinned host memory, into which the gap's last kernel writes its sums;
 *   - calls that return values to the host (gap, get_*) wait for the stream; the others only enqueue;
 *   - a context is not thread-safe.
 */
#ifndef CHICLE_ROUND_H
#define CHICLE_ROUND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct chicle_ctx chicle_ctx;

enum chicle_status {
    CHICLE_OK = 0,
    CHICLE_EINVAL = -1,   /* bad argument, malformed chunk, bad table */
    CHICLE_ENOMEM = -2,   /* arena too small */
    CHICLE_ESTATE = -3,   /* call not legal in the current state (ownership contract) */
    CHICLE_EDEVICE = -4   /* HIP error, or a kernel flagged bad input (e.g. perm entry out of range) or gave
                             up a bounded wait between the workgroups that share a solver */
};

enum chicle_loss { CHICLE_LOSS_HINGE = 0, CHICLE_LOSS_SQUARED = 1, CHICLE_LOSS_LOGISTIC = 2 };

/* Which local-solver kernel chicle_local_epoch launches (both visit the coordinates in exactly the
 * given order; they differ only in floating-point summation order). */
enum chicle_solver_kind {
    CHICLE_SOLVER_AUTO = 0,       /* choose from the data shape */
    CHICLE_SOLVER_ROWWISE = 1,    /* one coordinate step at a time; where sparse rows are long (more than 96 entries
                                     on average) and the chip has more compute units than solvers, several
                                     workgroups share every solver, each owning a range of columns (Section 4.2:
                                     a solver may use all processors of its node) */
    CHICLE_SOLVER_BATCHED = 2,    /* blocks of 64 rows via their Gram matrix, same sequence of steps: sparse rows
                                     of at most 48 entries (dense rows that short are stored that way), or dense
                                     rows of at most 320 columns; else EINVAL at the pass.  Where the columns do
                                     not all fit the part of the private vector a compute unit keeps on chip and
                                     the chip has compute units to spare, two workgroups share every solver: one
                                     owns the popular columns and runs the steps, the other owns the rest */
    CHICLE_SOLVER_ROWWISE_ONE_CU = 3, /* row-wise with every solver on one compute unit */
    CHICLE_SOLVER_BATCHED_ONE_CU = 4  /* batched with every solver on one compute unit */
};

/* Timed segments reported by chicle_last_kernel_ms. */
enum chicle_segment {
    CHICLE_SEG_LOCAL_EPOCH = 0,   /* everything chicle_local_epoch enqueued */
    CHICLE_SEG_AGGREGATE = 1,
    CHICLE_SEG_GAP = 2,
    CHICLE_SEG_EPOCH_GRAM = 3,    /* batched solver only: the Gram-block kernel */
    CHICLE_SEG_EPOCH_CHAIN = 4,   /* the kernel that runs the coordinate steps */
    CHICLE_SEG_COUNT = 5
};

/* Bytes of device arena a context needs (host, pure).  total_entries = stored matrix entries over all
 * chunks (CSR non-zeros, or n_total*d for dense chunks).  Returns 0 on bad arguments. */
size_t chicle_arena_bytes(int64_t n_total, int64_t total_entries, int32_t d, int32_t n_chunks,
                          int32_t max_solvers, int32_t dense);

/* Create a context in state LOADING with alpha = 0, w = 0.
 *   loss          chicle_loss
 *   n_total       number of rows over all chunks (the n of the objective)
 *   d             number of columns (length of w)
 *   lambda        normalised regulariser (> 0)
 *   n_chunks      chunk ids are 0 .. n_chunks-1
 *   max_solvers   largest K that will ever be assigned
 *   dense         1: all chunks dense row-major, 0: all chunks CSR
 *   device_arena  device pointer, 256-byte aligned, arena_bytes long, borrowed
 *   hip_stream    hipStream_t (NULL = the default stream), borrowed
 * Errors: EINVAL (arguments), ENOMEM (arena smaller than chicle_arena_bytes), EDEVICE. */
int chicle_create(chicle_ctx **out, int32_t loss, int64_t n_total, int32_t d, double lambda,
                  int32_t n_chunks, int32_t max_solvers, int32_t dense, int64_t total_entries,
                  void *device_arena, size_t arena_bytes, void *hip_stream);

/* Copy one chunk into the chunk store (Section 4.4).  All pointers are host arrays.
 *   row_ptr  n_rows+1 chunk-local offsets, row_ptr[0] = 0, non-decreasing
 *   col      row_ptr[n_rows] column ids in [0, d), strictly ascending inside a row
 *   val      matching values;  y  n_rows labels (+-1 for hinge and logistic) or targets
 *   alpha0   initial dual variables or NULL for zeros (hinge, logistic: must lie in [0,1])
 * Legal in LOADING only.  Errors: EINVAL (malformed arrays, id out of range or already loaded,
 * label not +-1 where the loss asks for it), ENOMEM (store full), ESTATE. */
int chicle_load_chunk_csr(chicle_ctx *ctx, int32_t chunk_id, int32_t n_rows, const int32_t *row_ptr,
                          const int32_t *col, const float *val, const float *y, const float *alpha0);

/* Dense variant: X is row-major n_rows x d (host). */
int chicle_load_chunk_dense(chicle_ctx *ctx, int32_t chunk_id, int32_t n_rows, const float *X,
                            const float *y, const float *alpha0);

/* Greedy balanced chunk -> solver table (host, pure, integers only): chunks by (load descending, id
 * ascending), each to the solver that would finish it earliest, (L_k + load)/speed_k, ties to the
 * smallest solver index.  speed_q: K positive integer speed weights or NULL for equal speeds.
 * This is the elastic-scaling / load-balancing step of Section 3 reduced to one deterministic rule
 * (the paper's policies of Section 4.5 pick chunks randomly or shift them gradually). */
int chicle_balance(const int64_t *chunk_load, int32_t n_chunks, int32_t K, const int32_t *speed_q,
                   int32_t *chunk_to_solver_out);

/* Iteration time under the projection model of the evaluation (Sections 5.3 and 5.4), in units of
 * "one task that holds 1/base_nodes of the data, on a full-speed node" (host, pure).
 *   K_tasks     > 0: that many equal micro-tasks run in waves over the nodes; 0: uni-tasks, one per
 *               node, each sized to its node's speed
 *   nodes       nodes available;  n_slow of them take slow_factor (> 0) times as long per task
 * Equal nodes: base/K * ceil(K/nodes) for micro-tasks, base/nodes for uni-tasks.  Mixed nodes: the
 * shortest schedule with i tasks on every slow and j on every fast node, max(i*slow_factor, j)*base/K;
 * uni-tasks finish together, base / (n_fast + n_slow/slow_factor).  Returns a negative value for
 * invalid arguments. */
double chicle_projected_iteration_time(int32_t K_tasks, int32_t nodes, int32_t n_slow, double slow_factor,
                                       int32_t base_nodes);

/* Elastic scaling policy, growing from K_old to K_new solvers (Section 4.5; Section 5.3 adds that the
 * chunks moved to new tasks are picked randomly from each old task).  Host, pure, integers only.
 * Every old solver hands over floor(count * (K_new - K_old) / K_new) of its chunks: those with the
 * smallest draw[chunk] (ties: smaller chunk id).  Handed-over chunks, old solver by old solver in pick
 * order, go to solvers K_old, K_old+1, .., K_new-1, K_old, .. in turn.  draw: one caller-supplied random
 * word per chunk.  in and out may not overlap.  Errors: EINVAL. */
int chicle_scale_out(const int32_t *chunk_to_solver, int32_t n_chunks, int32_t K_old, int32_t K_new,
                     const uint32_t *draw, int32_t *chunk_to_solver_out);

/* Elastic scaling policy, shrinking to K_new < K_old solvers (Section 4.5: chunks of the workers to be
 * freed are redistributed round robin).  Chunks of solvers K_new .. K_old-1, freed solver by freed
 * solver in ascending chunk id, go to solvers 0, 1, .., K_new-1, 0, .. in turn.  Errors: EINVAL. */
int chicle_scale_in(const int32_t *chunk_to_solver, int32_t n_chunks, int32_t K_old, int32_t K_new,
                    int32_t *chunk_to_solver_out);

/* Rebalancing policy (Section 4.5), one call between two iterations.  Host, pure.
 *   chunk_load   load of every chunk (stored entries)
 *   unit_time    n_iterations x K row-major: runtime per unit of load that solver k showed in each of
 *                the last n_iterations iterations (> 0); a solver's rate is the median of its column
 *   max_moves    chunks moved at most in this call (the policy shifts load over several iterations)
 *   chunk_to_solver  table, updated in place;  n_moved_out (may be NULL) receives the number moved
 * Repeatedly the solver with the longest projected time rate*load gives its lightest chunk (ties: the
 * larger chunk id) to the solver with the shortest one, and stops when their difference is no larger
 * than the time that chunk would take on the receiver.  Errors: EINVAL. */
int chicle_rebalance(const int64_t *chunk_load, int32_t n_chunks, int32_t K, const double *unit_time,
                     int32_t n_iterations, int32_t max_moves, int32_t *chunk_to_solver, int32_t *n_moved_out);

/* When to scale in (host, pure).  Section 2.2 cites that starting with many partitions and reducing them
 * after a few iterations speeds up convergence, and the evaluation's summary that such changes pay once
 * convergence slows down; the rule itself is this library's: a round has stalled when the gap after it is
 * more than stall_ratio times the gap before it, and after `patience` stalled rounds in a row the number
 * of solvers is halved (rounded up, not below K_min).
 *   gap           the duality gap before the first round and after every round so far (n_gaps entries)
 *   since_change  rounds run with the current K (only those count towards patience)
 * Returns the number of solvers for the next round (K when nothing changes), or a negative value for
 * invalid arguments (null gap, n_gaps < 1, K < 1, K_min < 1, stall_ratio outside (0, 1], patience < 1,
 * since_change < 0). */
int32_t chicle_next_solver_count(const double *gap, int32_t n_gaps, int32_t K, int32_t K_min,
                                 double stall_ratio, int32_t patience, int32_t since_change);

/* Scheduler step between iterations (Section 3 "Uni-tasks": between iterations the scheduler owns the
 * chunks and may hand them to other tasks; Section 5.1: sigma is the number of tasks): give every chunk
 * to one of K solvers (host table of n_chunks entries in [0, K)); sigma becomes K; every solver's
 * update starts from nothing (its private vector equals w).  A solver
 * may own no chunk.  alpha is not touched.  A solver's local rows are its chunks in ascending chunk id,
 * rows ascending inside a chunk.  Legal in LOADING (all chunks loaded, row counts summing to n_total)
 * and READY.  Errors: EINVAL, ESTATE. */
int chicle_assign(chicle_ctx *ctx, int32_t K, const int32_t *chunk_to_solver);

/* Runtime of every solver's last local pass in milliseconds (host out, K entries), from the device's
 * constant-rate clock read at the start and at the end of the solver's workgroup: the task runtimes
 * the rebalancing policy learns from (Section 4.5).  Synchronises the stream.  Errors: ESTATE before
 * the first local epoch, EDEVICE. */
int chicle_solver_ms(chicle_ctx *ctx, float *ms_out);

/* Rows owned by each solver under the current assignment (host out, K entries). */
int chicle_solver_rows(chicle_ctx *ctx, int64_t *rows_out);

/* Select the local-solver kernel (chicle_solver_kind); default AUTO. */
int chicle_set_solver(chicle_ctx *ctx, int32_t kind);

/* Elastic net (Section 2.2: the method covers generalised linear models with a strongly convex
 * regulariser): the objective becomes (1/n) sum_i loss_i(x_i . w) + lambda (|w|^2 / 2 + l1 |w|_1).  The
 * solvers' updates then add up in the dual image v (kept in double), the shared vector every solver
 * starts from is w_j = sign(v_j) max(|v_j| - l1, 0), the local pass is unchanged, the primal value gains
 * lambda l1 |w|_1 and the dual value uses |w|^2 / 2 as the regulariser's conjugate at v.  l1 = 0 (the
 * default) is the plain L2 round.  Legal in LOADING and READY; in READY the shared vector is recomputed
 * from v with the new threshold.  Afterwards chicle_set_w is refused while l1 > 0 (w does not determine
 * v).  Errors: EINVAL (negative or not finite), ESTATE (between local_epoch and aggregate). */
int chicle_set_l1(chicle_ctx *ctx, double l1);

/* One local pass of all K solvers, concurrently, each from the current w (Section 2.2; Section 4.2).
 * perm_device: device array of n_total int32: solver 0's visiting order (a permutation of
 * [0, rows_0)), then solver 1's, and so on.  Commits alpha in the chunks and leaves the solver's update
 * in its private vector, which is stored as the difference u_k = v_k - w = sigma * Delta w_k (v_k being
 * the solver's private copy of the shared vector).  READY -> EPOCH_DONE.
 * An out-of-range perm entry is skipped and reported as EDEVICE by the next synchronising call. */
int chicle_local_epoch(chicle_ctx *ctx, const int32_t *perm_device);

/* Same, and perm_next_device (may be NULL) announces the orders of the following local pass.  They are
 * copied into the context on the context's stream (the caller's buffer is an ordinary stream-ordered input
 * of this call and is not referred to afterwards), and work for that pass which depends on the data and the
 * orders alone (the Gram blocks of the batched solver) is started on a stream of the library's own, ordered
 * after everything enqueued on the context's stream before this call, and runs beside this pass.
 * perm_device may be NULL: the pass then runs with the orders that the previous call announced, from the
 * context's copy, and uses the work prepared for them.  A non-NULL perm_device discards what was announced;
 * so does an assign.  Errors: EINVAL (perm_device NULL with nothing announced), ESTATE. */
int chicle_local_epoch_ahead(chicle_ctx *ctx, const int32_t *perm_device, const int32_t *perm_next_device);

/* Same as chicle_local_epoch with the orders given as a host array (copied to a staging area first). */
int chicle_local_epoch_host_perm(chicle_ctx *ctx, const int32_t *perm_host);

/* Trainer step (Section 4.1: merge updates, broadcast the model): w <- w + sum_k Delta w_k, then every
 * solver's private copy equals w again (its stored difference u_k is cleared).  EPOCH_DONE -> READY. */
int chicle_aggregate(chicle_ctx *ctx);

/* The convergence metric that solvers report to the trainer every iteration (Section 4.1) and that the
 * evaluation follows, the duality gap (Section 5.1): P(w), D(alpha) and P - D at the current state, with the
 * objectives stated at the top of this file (host outs, any may be NULL).  Legal in READY.  Synchronises.
 * Errors: ESTATE, EDEVICE. */
int chicle_gap(chicle_ctx *ctx, double *primal, double *dual, double *gap);

/* chicle_gap for callers that cannot allocate device memory or hand over a workspace for this call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * kernels and same results as chicle_gap; the kernels' partial sums go to a fixed array in the library's
 * code object (136 KB, one copy per GPU, held until the process ends) instead of the arena.  The call
 * allocates nothing.  Limit: at most 4096 chunks (EINVAL beyond).  All contexts on one GPU share that
 * array: every call overwrites what it reads later, so nothing needs clearing, but two such calls that
 * overlap in time on one GPU (different streams or threads) race.  Errors as chicle_gap, plus EINVAL for
 * the limit and EDEVICE when the array's address could not be obtained at chicle_create. */
int chicle_gap_noalloc(chicle_ctx *ctx, double *primal, double *dual, double *gap);

/* State access: the shared vector, and the per-sample state that lives inside its chunk and moves with it
 * (Section 4.4 "In-memory chunk data format"); what a trainer checkpoints or restores between iterations.
 * Host arrays of d floats / n_rows-of-that-chunk floats.  get_* synchronise.
 * set_alpha is legal in READY/LOADING, set_w in READY; get_delta_w in EPOCH_DONE only:
 * solver >= 0 gives Delta w_solver = (v_solver - w)/sigma, solver = -1 gives sum_k Delta w_k. */
int chicle_get_w(chicle_ctx *ctx, float *w_out);
int chicle_set_w(chicle_ctx *ctx, const float *w_in);
int chicle_get_delta_w(chicle_ctx *ctx, int32_t solver, float *dw_out);
int chicle_get_alpha(chicle_ctx *ctx, int32_t chunk_id, float *alpha_out);
int chicle_set_alpha(chicle_ctx *ctx, int32_t chunk_id, const float *alpha_in);
int chicle_get_assignment(chicle_ctx *ctx, int32_t *chunk_to_solver_out, int32_t *K_out);

/* Diagnostic: run only the Gram-block kernel of the batched solver for the given visiting orders and
 * copy its output to the host.  Blocks of 64 consecutive steps of a solver form one tile of 128 x 64
 * floats laid out [jp][i]: T[jp][i] couples step i of the block with step jp of the previous block
 * (jp < 64) or with step jp - 64 of the same block (entries with jp - 64 >= i are zero);
 * T = -y_i y_j (x_i . x_j) / |x_i|^2 for hinge, -(x_i . x_j) / (lambda n / sigma + |x_i|^2) for squared loss.
 * Tiles are ordered by solver, then by block.  tiles_out may be NULL to query *n_tiles_out only.
 * Legal in READY.  Errors: EINVAL (data not eligible for the batched solver, capacity), ESTATE. */
int chicle_debug_gram(chicle_ctx *ctx, const int32_t *perm_device, float *tiles_out,
                      int64_t capacity_floats, int32_t *n_tiles_out);

/* Wait for the stream; report any deferred kernel error. */
int chicle_sync(chicle_ctx *ctx);

/* Event timing of the library's own launches.  With profiling on, every call records HIP events on the
 * context's stream around each segment; chicle_last_kernel_ms waits for the segment's end event and
 * returns the duration of its most recent execution in milliseconds. */
int chicle_set_profiling(chicle_ctx *ctx, int32_t on);
int chicle_last_kernel_ms(chicle_ctx *ctx, int32_t segment, float *ms_out);

const char *chicle_last_error(chicle_ctx *ctx);
void chicle_destroy(chicle_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* CHICLE_ROUND_H */
