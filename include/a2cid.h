/*
 * a2cid.h -- C ABI of the MI355X (gfx950) continuous-momentum gossip engine.
 *
 * The library applies the event-based dynamic of A2CiD2 (arXiv 2306.08289, Eq. (1),
 * realised event by event as in Algorithm 1) to n simulated workers.  Worker i owns row i
 * of two caller-provided device buffers: x (parameters) and xt (the momentum copy, written
 * x-tilde in the paper), d fp32 values each, plus a host-side time stamp t_i at which the row
 * was last brought up to date.  Three kinds of update exist:
 *
 *   mixing flow  (x_i, xt_i) <- exp((t - t_i) [[-eta, eta], [eta, -eta]]) (x_i, xt_i)
 *                applied to a worker right before any jump that touches it (Algorithm 1); the
 *                elapsed time t - t_i is multiplied by the speed of worker i's own clock, which
 *                is 1 unless the caller sets it (a2cid_op.clock_rate);
 *   gradient     x_i -= gamma g,  xt_i -= gamma g                  (Eq. (1), dN^i term)
 *                with g = gscale * h .* (x_i - c) + xi evaluated AFTER the mixing;
 *   gossip       m = x_i - x_j;  x_i -= alpha m;  x_j += alpha m;
 *                xt_i -= alpha_tilde m;  xt_j += alpha_tilde m     (Eq. (1), dM^ij term)
 *                with m evaluated AFTER both workers have been mixed.
 *
 * Conventions
 *   - "device pointer": memory of the GPU that is current when a2cid_create is called; "host
 *     pointer": ordinary process memory.  The library never allocates, frees or reallocates
 *     x, xt, xi or c; it owns only a small device scratch area (operation tables and
 *     reduction partials) that lives as long as the context.
 *   - All work is enqueued on the HIP stream given at creation.  a2cid_apply_events and
 *     a2cid_flush return as soon as the work is enqueued; a2cid_stats waits for its result.
 *   - Every function returns A2CID_OK (0) or a negative A2CID_E* code and a2cid_last_error()
 *     (thread-local) describes the cause.  Everything a call can check -- arguments, batch
 *     structure, time order, pointers, sizes -- is checked before the call enqueues anything or
 *     moves a time stamp, so a call that fails one of these checks has applied nothing.  If a HIP
 *     call fails after that point, part of the work may already be in the stream while the time
 *     stamps were not advanced: the context is then marked unusable and every later
 *     a2cid_apply_events / flush / stats / average on it returns A2CID_EHIP.  No exception, abort
 *     or signal crosses this boundary.
 *   - A context must not be used from two threads at once.
 */
#ifndef A2CID_H
#define A2CID_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define A2CID_OK          0
#define A2CID_EINVAL     -1   /* null pointer, size out of range, non-finite parameter          */
#define A2CID_EGRAPH     -2   /* edge list malformed (u >= v, duplicate, out of range, rate < 0) */
#define A2CID_EORDER     -3   /* an event is earlier than its worker's current time stamp       */
#define A2CID_EMATCHING  -4   /* two operations of one level share a worker, or bad level table  */
#define A2CID_EALIGN     -5   /* pointer not 16-byte aligned or ld not a multiple of 4           */
#define A2CID_EHIP       -6   /* a HIP runtime call failed (message holds the HIP error string) */
#define A2CID_ENOMEM     -7   /* host allocation failed                                        */

#define A2CID_KIND_GRADIENT 0
#define A2CID_KIND_GOSSIP   1

#define A2CID_MAX_WORKERS 1024

#define A2CID_ORDER_EQ1     0   /* jumps evaluated after the mixing: Eq. (1) (default)          */
#define A2CID_ORDER_LISTING 1   /* jumps evaluated before it: the line order of Algorithm 1     */

typedef struct a2cid_ctx a2cid_ctx;
typedef struct a2cid_sched a2cid_sched;

/* Undirected communication graph with one Poisson rate per edge (Definition 3.1: the rates
 * are the lambda^{ij} of the instantaneous expected Laplacian).  Host pointers, n_edges
 * entries each, u[e] < v[e], no duplicates.  Borrowed for the duration of the call only. */
typedef struct {
    int32_t n_edges;
    const int32_t *u;
    const int32_t *v;
    const double *rate;
} a2cid_graph;

/* The state buffers.  x and xt are device pointers to n rows of ld floats (row-major, row i =
 * worker i, the first d entries of a row are used, the rest is never read or written).  Both
 * must be 16-byte aligned and ld must be a multiple of 4, so that every row is 16-byte aligned.
 * hip_stream is a hipStream_t (NULL: the default stream).  Owned by the caller and must outlive
 * the context. */
typedef struct {
    float *x;
    float *xt;
    int64_t ld;
    void *hip_stream;
} a2cid_buffers;

/* One event of the dynamic.
 *   t       absolute time of the event (same clock for all workers).
 *   kind    A2CID_KIND_GRADIENT (worker i; j ignored, conventionally -1) or
 *           A2CID_KIND_GOSSIP (edge {i, j} of the graph, either orientation).
 *   gamma   step size of a gradient event (Eq. (1)); ignored for gossip.
 *   gscale  slope s of the affine gradient model g = s h .* (x_i - c) + xi.  s = 0 with xi = the
 *           gradient computed elsewhere is the general case; s = 1 with c = c_i is the
 *           quadratic f_i = 1/2 ||x - c_i||^2; with a curvature vector h it is the gradient of
 *           f_i(x) = s/2 sum_k h_k (x_k - c_k)^2, which is (s min h)-strongly convex and
 *           (s max h)-smooth: the first setting of Proposition 3.2.
 *   xi, c, h  device pointers to d floats, 16-byte aligned, or NULL (xi, c: zeros; h: ones).
 *           Read when the stream reaches the operation; the caller keeps them alive until
 *           then.  c and h are not read when gscale = 0.
 *   clock_rate  gradient events only; 0: nothing changes.  > 0: from this event on worker i's own
 *           clock runs at this speed against the clock of the event times, i.e. the mixing of
 *           worker i between two of its events (or up to t_sync, or up to the t_now of a2cid_stats,
 *           a2cid_flush, a2cid_average) lasts clock_rate times the difference of the two times.
 *           This is the time normalisation of the section "Practical implementation of the
 *           dynamic" (a running average of the durations of the previous gradient steps) read per
 *           worker: the caller passes 1 / (average duration of worker i's steps so far).  The
 *           mixing up to this event itself still uses the previous speed.  Every worker starts at
 *           speed 1 (a2cid_set_clock_rates changes that).
 *   id      opaque to the library (the scheduler stores the serial event index here). */
typedef struct {
    double t;
    int32_t kind;
    int32_t i;
    int32_t j;
    float gamma;
    float gscale;
    float clock_rate;
    const float *xi;
    const float *c;
    const float *h;
    int64_t id;
} a2cid_op;

/* A batch of events arranged in levels.  ops[level_off[l] .. level_off[l+1]) is level l;
 * level_off has n_levels + 1 entries, level_off[0] = 0, level_off[n_levels] = n_ops.
 * Operations of one level must touch pairwise distinct workers (a matching plus singletons).
 * Every worker meets its events in the order given; operations on distinct workers commute
 * exactly, and the library is free to interleave them in any order that respects this (mode 0
 * applies level after level, the other modes walk the batch per column tile: a2cid_set_tuning).
 * Times must be non-decreasing per worker (across batches too).  All host pointers, borrowed for
 * the call.
 *   t_sync  if finite: after its last operation in this batch every worker touched by the
 *           batch is additionally mixed up to t_sync (fused into that operation's pass, the
 *           "mix -> jump -> mix" form) and its time stamp becomes t_sync; must be >= every
 *           event time of the batch.  NaN: no trailing mix. */
typedef struct {
    int64_t n_ops;
    const a2cid_op *ops;
    int32_t n_levels;
    const int64_t *level_off;
    double t_sync;
} a2cid_event_batch;

/* Observables (appendix "Notations": ||pi x||_F^2 = sum_i ||x_i - xbar||^2; Eq. (2) for the
 * role of the sums).  sum_x and sum_xt are caller-allocated host arrays of n doubles. */
typedef struct {
    double consensus_x;
    double consensus_xt;
    double *sum_x;
    double *sum_xt;
} a2cid_stats_out;

/* Per-operation coefficients produced by the host planner (exposed for testing and for
 * callers that want to inspect a plan).  b = (1 - exp(-2 eta tau)) / 2 is the off-diagonal
 * entry of exp(tau [[-eta, eta], [eta, -eta]]) = [[1 - b, b], [b, 1 - b]]. */
typedef struct {
    float b_pre_i, b_pre_j;    /* mixing to the event time, worker i / worker j (j: gossip only) */
    float b_post_i, b_post_j;  /* trailing mixing to t_sync (0 when none)                        */
} a2cid_coef;

/* ---- hyper-parameters ----------------------------------------------------------------- */

/* chi_1 = 1 / (smallest non-zero eigenvalue of the Laplacian), chi_2 = half the largest
 * effective resistance over the edges (the two definitions after Definition 3.1), and the
 * accelerated setting of Proposition 3.2: eta = 1 / (2 sqrt(chi_1 chi_2)),
 * alpha_tilde = sqrt(chi_1 / chi_2) / 2 (alpha is 1/2).  Any output pointer may be NULL.
 * A2CID_EGRAPH if the graph is malformed or not connected.  Host only. */
int a2cid_graph_params(const a2cid_graph *graph, int32_t n,
                       double *chi1, double *chi2, double *eta, double *alpha_tilde);

/* ---- engine ---------------------------------------------------------------------------- */

/* Creates a context for n workers (2 <= n <= A2CID_MAX_WORKERS) of d >= 1 parameters on the
 * current HIP device, which must own x and xt (checked: a2cid_check_device_span).  eta >= 0,
 * alpha and alpha_tilde finite: the three constants of Eq. (1), fixed for the life of the context.
 * All t_i start at 0 (Algorithm 1, initialisation).  The graph is copied. */
int a2cid_create(a2cid_ctx **out, int32_t n, int64_t d, const a2cid_graph *graph,
                 double eta, double alpha, double alpha_tilde, const a2cid_buffers *buf);

/* Validates the batch (levels, edges, time order, alignment, and that every xi, c and h it will read
 * is d floats of device memory: see a2cid_check_device_span), computes the mixing coefficients from
 * the time stamps, advances the time stamps and enqueues the kernels (Algorithm 1, both threads, for
 * every event of the batch).  When validation fails nothing is enqueued and no time stamp moves.
 * The device that was current at a2cid_create must be current (A2CID_EINVAL otherwise); the same
 * holds for a2cid_flush, a2cid_stats and a2cid_average. */
int a2cid_apply_events(a2cid_ctx *ctx, const a2cid_event_batch *batch);

/* Chooses from which values a jump is formed, for all later batches.  A2CID_ORDER_EQ1: the
 * gradient g and the difference m = x_i - x_j are evaluated after the workers have been mixed to
 * the event time, as Eq. (1) prescribes (its jump terms act on x_t).  A2CID_ORDER_LISTING: they
 * are evaluated from the stored values, then the workers are mixed, then the jump is applied --
 * the order in which Algorithm 1 lists its lines, where g is as stale as the mixing it skipped.
 * The two coincide when eta = 0. */
int a2cid_set_order(a2cid_ctx *ctx, int32_t order);

/* Consensus distances and per-worker sums of the state as it would be if every worker were
 * mixed up to t_now (>= max_i t_i); x, xt and the time stamps are left untouched.  Blocks
 * until the result is in *out. */
int a2cid_stats(a2cid_ctx *ctx, double t_now, a2cid_stats_out *out);

/* a2cid_stats for callers that cannot allocate device memory or wait for the stream (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same observables of
 * the same virtually mixed state, written to caller-provided DEVICE memory, asynchronously on the
 * context's stream, by the same kernels.  out: 2 n + 2 doubles, 8-byte aligned, device memory of
 * the context's GPU: [0, n) the sums of x_i, [n, 2n) the sums of xt_i, [2n] and [2n + 1] the
 * consensus distances of x and xt.  The call makes no hipMalloc / hipFree and no host allocation,
 * uploads nothing (the n pending mixing coefficients travel in the kernel's argument block) and
 * does not synchronise.  Its only scratch, the per-workgroup partial sums, is a fixed array of
 * 2 129 920 bytes inside the library's code object: every GPU the library runs on holds one copy
 * until the process ends, and all calls on a GPU share it.  Each call rewrites every entry it later
 * reads, so nothing has to be cleared between calls, but two calls that overlap on one GPU (two
 * contexts or streams) race on it: serialise them.  At most A2CID_STATS_STATIC_MAX_WORKERS workers
 * (A2CID_EINVAL beyond); for more than 64 workers fewer workgroups than a2cid_stats would use share
 * the scratch, which changes the summation order (last bits) but not the result otherwise. */
#define A2CID_STATS_STATIC_MAX_WORKERS 256
int a2cid_stats_static(a2cid_ctx *ctx, double t_now, double *out);

/* Mixes every worker up to t_now (>= max_i t_i) in place and sets all t_i = t_now: the state
 * Algorithm 1 returns at its final time. */
int a2cid_flush(a2cid_ctx *ctx, double t_now);

/* Consensus step of the experimental protocol (section "Experimental Setup": the workers are
 * averaged once before and once after training): mixes every worker up to t_now
 * (>= max_i t_i), then replaces every x_i by the mean of the x_j and every xt_i by the mean of the
 * xt_j, and sets all t_i = t_now.  Both means, hence Eq. (2)'s tracker, are unchanged by it; the
 * consensus distances become 0.  Asynchronous like a2cid_flush (16 n d bytes). */
int a2cid_average(a2cid_ctx *ctx, double t_now);

/* Copies the n time stamps t_i into the host array t. */
int a2cid_get_times(const a2cid_ctx *ctx, double *t);

/* Replaces the n time stamps (resuming from a saved state). */
int a2cid_set_times(a2cid_ctx *ctx, const double *t);

/* The speeds of the n workers' own clocks (a2cid_op.clock_rate): get, and set (finite, > 0; e.g. the
 * nominal step rates before any gradient step has been measured, or a saved state). */
int a2cid_get_clock_rates(const a2cid_ctx *ctx, double *rate);
int a2cid_set_clock_rates(a2cid_ctx *ctx, const double *rate);

/* Waits until everything enqueued so far has finished. */
int a2cid_synchronize(a2cid_ctx *ctx);

void a2cid_destroy(a2cid_ctx *ctx);

/* ---- host-only planner (no GPU needed) -------------------------------------------------- */

/* The validation and coefficient step of a2cid_apply_events as a pure host function:
 * t (n doubles) is read and, on success, advanced; coef receives one entry per operation.
 * Same error codes as a2cid_apply_events. */
int a2cid_plan_batch(int32_t n, const a2cid_graph *graph, double eta, double *t,
                     const a2cid_event_batch *batch, a2cid_coef *coef);
/* The same with worker clocks: rate (n doubles, the speed of every worker's own clock, see
 * a2cid_op.clock_rate) is read and, on success, updated by the batch's gradient events.
 * a2cid_plan_batch is this function with every speed 1 at the start of the batch. */
int a2cid_plan_batch_clocks(int32_t n, const a2cid_graph *graph, double eta, double *t, double *rate,
                            const a2cid_event_batch *batch, a2cid_coef *coef);

/* The programme the chain kernel (a2cid_set_tuning, mode 3) runs for a batch, as a pure host
 * function.  Eq. (1) lets operations on disjoint workers commute, so any order that keeps every
 * worker's own operations in sequence yields the same state bit for bit; the library picks one in
 * which an operation finds its workers' columns close by as often as it can: in the workgroup's
 * carry registers (A2CID_LOC_CARRY: handed from one operation to the very next) or parked in one of
 * lds_slots LDS slots (A2CID_LOC_SLOT0 + s), instead of device memory (A2CID_LOC_MEMORY).
 * A step with op >= 0 applies batch->ops[op] with its workers presented as (row_i, row_j) (row_j = -1
 * for a gradient event; the carried worker is always row_i), reads them from src_i / src_j and leaves
 * them in dst_i / dst_j.  A step with op = -1 writes the worker row_i parked in slot src_i back to
 * memory.  After the last step every worker's columns are in memory (a worker's last operation
 * of the batch always leaves it there).
 * steps (capacity entries; 3 n_ops always suffice) may be NULL to query *n_steps only;
 * *bytes_per_column (may be NULL) receives what the launch moves per column: 8 per row read from or
 * written to memory, 4 per gradient input read.  Only kinds, worker indices and the xi / c / h / gscale
 * fields of the operations are read (the level table is not).  0 <= lds_slots <= 16.
 * a2cid_apply_events plans pieces of at most 5456 operations (whole levels) independently. */
#define A2CID_LOC_MEMORY 0
#define A2CID_LOC_CARRY  1
#define A2CID_LOC_SLOT0  2
typedef struct a2cid_chain_step {
    int32_t op;
    int32_t row_i, row_j;
    uint8_t src_i, src_j, dst_i, dst_j;
} a2cid_chain_step;
int a2cid_plan_chain(int32_t n, const a2cid_event_batch *batch, int32_t lds_slots, a2cid_chain_step *steps,
                     int64_t capacity, int64_t *n_steps, double *bytes_per_column);

/* The programmes the resident kernel (a2cid_set_tuning, mode 2) runs for one launch, as a pure host
 * function.  waves wavefronts share a tile of 64 * cols columns that stays in LDS for the whole launch;
 * the operations of a level touch disjoint workers, so they are dealt to the waves, and a workgroup
 * barrier separates levels.  Every wave gets its own linear programme of 16-byte slots, typed by
 * position (fp32 values as their bit patterns):
 *   control:  x = gossip operations | gradient operations << 8 that follow, after a barrier (a level);
 *             or 0x10000: continue with the next set of 64 slots; or 0x20000: the end.  In the first slot
 *             of a programme also y = ordinal of the wave's first gradient event (0xffffffff: none),
 *             z, w = low and high word of that event's xi;
 *   gossip:   x, y = LDS byte offsets of worker i's and j's row (512 * cols * position in rows),
 *             z, w = mixing coefficients b_pre_i, b_pre_j; if any operation of the batch has a trailing
 *             mix, a second slot follows with x, y = b_post_i, b_post_j;
 *   gradient: two slots: x = LDS byte offset of the worker's row, y = b_pre_i, z = gamma, w = gscale;
 *             then x = ordinal of the wave's next gradient event (0xffffffff: none), y = b_post_i,
 *             z, w = that event's xi.  An xi of 1 stands for "no xi" (zeros).
 * All programmes hold the same number of levels; a level never straddles a set of 64 slots; a
 * programme has 256 (waves = 16) or 512 slots, end slots included, so one call takes as many whole
 * levels (levels of more than 31 * waves operations in parts) from operation first_op on as fit, and
 * *next_op is where the next launch starts (first_op must be the start of a level or a former
 * *next_op).  Gradient events are numbered in the order of gradient_ops (their indices in the batch).
 * *waves = 0 lets the library choose waves and cols from the batch (as a2cid_apply_events does) and
 * returns the choice.  slots: *waves * (256 or 512) entries, wave after wave (8192 always suffice);
 * rows: n entries; gradient_ops: n_ops entries.  coef: the batch's coefficients from a2cid_plan_batch. */
typedef struct a2cid_resident_slot {
    uint32_t x, y, z, w;
} a2cid_resident_slot;
int a2cid_plan_resident(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int32_t *waves, int32_t *cols,
                        int64_t first_op, a2cid_resident_slot *slots, int32_t *rows, int32_t *n_rows,
                        int64_t *gradient_ops, int32_t *n_gradient_ops, int64_t *next_op);

/* The programme the register-file kernel (a2cid_set_tuning, mode 4; n <= 64) runs for one launch, as a
 * pure host function.  A wavefront keeps its 64 columns of every worker's x and xt in vector registers
 * for the whole launch, so all wavefronts run the same linear programme, the batch's operations in the
 * batch's order from first_op on, as 16-byte slots whose kind is x >> 8 (fp32 values as bit patterns):
 *   0 gossip:   x = i, y = j, z, w = b_pre_i, b_pre_j;
 *   1 gradient: x = i | 1 << 8, y = b_pre_i, z = gamma, w = gscale; gradient events are numbered in the
 *               order of gradient_ops (their indices in the batch), 8 to a chunk;
 *   2 mix:      x = worker | 2 << 8, y = b_post: a trailing mix, directly after its operation (one slot
 *               per worker with b_post != 0);
 *   3 control:  x = 3 << 8, y = 2: the end; y = 0: filler; y = 1 or 3, in the first slot of a block of 8
 *               slots only: a request block.
 * Request block q (in programme order) names the inputs of chunk q: its slots 1-4 hold the 8 xi pointers
 * (two to a slot: x, y = low and high word of the first, z, w of the second), the rest is filler; if
 * full != 0 a second block follows with the c pointers in slots 0-3 and the h pointers in slots 4-7.  A
 * pointer with bit 0 set is the address of one float that stands for every column: zero_one for an
 * absent xi or c and for events past the last, zero_one + 1 for an absent h (zero_one: device address
 * of a float 0 followed by a float 1; only recorded here).  The programme begins with request blocks 0
 * and 1 (y = 3); request block k + 1 (y = 1) stands before the first gradient event of chunk k >= 1,
 * where the kernel waits for chunk k's inputs, requests chunk k + 1 into the registers chunk k - 1 used,
 * and turns to chunk k.  The programme is fetched in blocks of 8 slots, ends with an end slot and is
 * padded to a whole block.
 * One call takes as many operations as fit into max_slots slots (a multiple of 8, at least 32, with full
 * 48; the library uses 8192); *next_op is where the next launch starts.  touched: bit r set iff worker
 * r is used.  full must be set if any gradient event of the batch has a c or an h and gscale != 0.
 * slots: max_slots entries; gradient_ops: n_ops entries.  coef: the batch's coefficients from
 * a2cid_plan_batch.  The batch's level table is not read: any order that keeps every worker's own
 * operations in sequence gives the same bits (Eq. (1) couples no other), and the batch's order does. */
int a2cid_plan_registers(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int64_t first_op,
                         int64_t max_slots, int32_t full, const float *zero_one, a2cid_resident_slot *slots,
                         int64_t *n_slots, int64_t *gradient_ops, int32_t *n_gradient_ops, uint64_t *touched,
                         int64_t *next_op);

/* The check every register-file programme passes before it is launched (the kernel adds worker indices
 * to register numbers and trusts the block structure, so a malformed programme must never reach it):
 * whole blocks of 8 slots, the two first request blocks, worker indices below n <= 64, at most 8
 * gradient events between two switch slots, switch slots only at the head of a block and followed by
 * their pointer block(s), an end slot in the last block.  A2CID_OK or A2CID_EINVAL.  Host only. */
int a2cid_check_registers(int32_t n, int32_t full, const a2cid_resident_slot *slots, int64_t n_slots);

/* ---- event scheduler (host only) ------------------------------------------------------- */

/* Independent Poisson clocks (Assumption 3.1): one per worker (gradient events, rate
 * node_rate[i] >= 0) and one per edge (gossip events, rate graph->rate[e] >= 0); a rate of 0
 * never fires.  The k-th waiting time of clock c (workers first, then edges in list order)
 * is -log1p(-u) / rate, u the 53-bit uniform built from the first two words of
 * Philox4x32-10(counter = (k_lo, k_hi, c, 0x0A2C1D20), key = (seed_lo, seed_hi)); arrival
 * times are running fp64 sums; simultaneous arrivals are ordered by clock id.  The merged
 * stream is therefore a pure function of (n, graph, node_rate, seed). */
int a2cid_sched_create(a2cid_sched **out, int32_t n, const a2cid_graph *graph,
                       const double *node_rate, uint64_t seed);

/* The event source of the paper's implementation instead of Assumption 3.1's clocks (section
 * "Practical implementation of the dynamic"; appendix "Uniform neighbor selection check"):
 * every worker computes gradient steps back to back (the k-th step of worker i lasts
 * (1 / node_rate[i]) (1 + jitter (2u - 1)), u uniform; its end is a gradient event) and at each
 * step's end adds a Poisson(comm_per_grad) number of p2p averagings to do; a worker that is not
 * inside an averaging and still has some to do is available and joins the tail of one queue; the
 * coordinator pairs the oldest available worker with its oldest available graph neighbour as long
 * as such pairs exist (a gossip event at that moment; both partners are then busy for comm_time).
 * Simultaneous completions are ordered (time, averaging-end before step-end, worker).  The graph's
 * rates are ignored.  Streams: Philox4x32-10 as for a2cid_sched_create with counter tags
 * 0x0A2C1D21 (durations) and 0x0A2C1D22 (Poisson counts, product-of-uniforms method).
 * normalize = 1 stamps the events with normalised time instead of real time, as the same section
 * describes (a running average of the duration of the previous gradient steps normalises time, so
 * that a gradient step takes one unit as the analysis assumes): the stamp advances by (real time
 * elapsed) / (average duration of all gradient steps completed so far, by any worker; before the
 * first completion: the mean of 1 / node_rate[i]); a step's duration enters the average after the
 * events of its own completion are stamped.  Durations and comm_time stay in real time.
 * normalize = 2 reads the same sentence per worker: the stamps stay in real time, and every gradient
 * event carries in clock_rate the speed of its worker's own clock from then on, 1 / (average duration
 * of that worker's steps completed so far, the one just finished included), as a float; the context
 * that consumes the stream should start from a2cid_set_clock_rates(node_rate).  The
 * returned scheduler is used with a2cid_sched_next / skip / counts / destroy like any other. */
int a2cid_sched_create_fifo(a2cid_sched **out, int32_t n, const a2cid_graph *graph, const double *node_rate,
                           double comm_per_grad, double comm_time, double jitter, int32_t normalize,
                           uint64_t seed);

/* Takes the next max_events events of the serial stream and packs them into levels: an
 * event's level is one more than the highest level of an earlier event of this batch sharing
 * a worker with it; inside a level events keep serial order.  The returned batch (ops,
 * level_off) points into memory owned by the scheduler and stays valid until the next call
 * on the same scheduler; the caller may fill in gamma, gscale, xi, c in place.  ops[k].id is
 * the serial index of the event (0-based since creation); t_sync is NaN. */
int a2cid_sched_next(a2cid_sched *s, int64_t max_events, a2cid_event_batch *out);

/* Skips the next n_events events of the serial stream without producing them. */
int a2cid_sched_skip(a2cid_sched *s, int64_t n_events);

/* Number of events of each clock produced so far (n + n_edges entries): the communication
 * history of the appendix "Uniform neighbor selection check" for the edge part. */
int a2cid_sched_counts(const a2cid_sched *s, int64_t *counts);

void a2cid_sched_destroy(a2cid_sched *s);

/* ---- diagnostics and measurement ------------------------------------------------------- */

/* Launch shape of the event kernels: unroll = 16-byte pieces per lane and row (1, 2 or 4),
 * nontemporal != 0 selects non-temporal loads and stores of the state (modes 0 and 1), threads =
 * workgroup size (64 ... 1024, a power of two), mode =
 *  -1: chosen by the library from the shape (default): 4 for up to 64 workers, 2 for up to 160; beyond
 *      that 1 for rows of at most 4096 parameters and 3 for everything else;
 *   0: one launch per level;
 *   1: one launch per batch in which every workgroup walks all operations, in level order, for its
 *      own columns, each operation reading and writing its rows in device memory (32 d bytes per
 *      gossip event);
 *   3: as 1, but following the programme of a2cid_plan_chain: a worker shared by consecutive
 *      operations stays in registers and workers that come back soon are parked in LDS (16 d bytes
 *      for a gossip event that finds one worker there and leaves one there);
 *   2: as 1, but the workgroup keeps its columns of all touched rows in LDS for the whole batch, so
 *      the state is read and written once per batch instead of once per event (at most 320
 *      workers: 512 bytes of LDS per worker and column-per-lane);
 *   4: as 2, but every wavefront keeps its 64 columns of all workers in its vector registers and
 *      runs the whole programme of a2cid_plan_registers on them, with no LDS and no barrier (at most
 *      64 workers, rows of at most 2^29 parameters).
 * Default: 1, 0, 256, -1 (tiles shrink automatically for short rows).  All modes compute the same
 * operations in the same per-worker order and give the same state bit for bit.  In every mode the
 * gradient inputs of a batch must hold their final values, in stream order, before
 * a2cid_apply_events is called. */
int a2cid_set_tuning(a2cid_ctx *ctx, int32_t unroll, int32_t nontemporal, int32_t threads, int32_t mode);

/* Mode 3 only: LDS slots in which a workgroup parks workers between operations (0 ... 16; each
 * takes unroll x threads x 32 bytes of the CU's 160 KiB of LDS per resident workgroup, so 5 leaves
 * room for four workgroups of 256 lanes on a CU: more slots save more traffic but leave fewer
 * columns in flight).  0: only the carry registers are used.  Default: 5. */
int a2cid_set_chain_slots(a2cid_ctx *ctx, int32_t slots);

/* Mode 1 only: at most workgroups_per_cu workgroups of the walk kernel share a compute unit (0, the
 * default: as many as fit, 8 of 256 lanes).  Fewer resident workgroups mean fewer columns in flight
 * and a smaller memory footprint per operation, so that a row written by one operation is more often
 * still in the last-level cache when a later operation reads it; which effect wins depends on how soon
 * rows come back in the event stream. */
int a2cid_set_walk_occupancy(a2cid_ctx *ctx, int32_t workgroups_per_cu);

/* Mode 2 only: group = waves per workgroup, i.e. how many operations of one level a column tile
 * processes concurrently (1, 2, 4, 8 or 16); cols = columns per lane (1, 2 or 4; group = 1 goes with
 * cols = 1 only): a tile is 64 * cols columns wide and needs 512 * cols bytes of the CU's 160 KiB of
 * LDS per worker.  group = 0 (the default; cols is then ignored): the library chooses both for every
 * batch from the average number of operations per level and the number of workers. */
int a2cid_set_resident_group(a2cid_ctx *ctx, int32_t group, int32_t cols);

/* Launch shape of the observables kernel: pieces = 16-byte pieces per lane and row (1 or 2), rows =
 * rows whose loads are issued together (1, 2 or 4), blocks = workgroups (grid-stride over column
 * tiles, 1 ... 8192), nontemporal != 0 selects non-temporal loads.  Default: 2, 2, 2048, 1.  The
 * first three change the summation order, hence the last bits of the results. */
int a2cid_set_stats_tuning(a2cid_ctx *ctx, int32_t pieces, int32_t rows, int32_t blocks, int32_t nontemporal);

/* The check the library applies to x and xt at creation and to every xi, c and h a batch will read:
 * A2CID_OK if [p, p + bytes) is device (or managed) memory of the context's GPU that does not run
 * past the end of its allocation, A2CID_EINVAL otherwise (a host pointer, another GPU's memory, a
 * span longer than what was allocated).  It sees allocations, not tensors: a span inside a
 * larger allocation, such as a caching allocator's segment, passes.  The runtime is asked on every
 * call (a2cid_apply_events asks once per allocation and batch).  Launches nothing. */
int a2cid_check_device_span(a2cid_ctx *ctx, const void *p, int64_t bytes);

/* Measurement aid, independent of any context: enqueues a plain copy of n floats (n a multiple
 * of 4) from src to dst (device pointers, 16-byte aligned, non-overlapping) on hip_stream, with
 * the same access shape as the event kernels.  It moves exactly 8 n bytes, which gives the
 * practical streaming ceiling of the machine at hand and the scale of its HBM byte counters. */
int a2cid_stream_probe(const float *src, float *dst, int64_t n, void *hip_stream);

/* Measurement aid: an in-place pass over the context's own state with the walk kernel's access shape and
 * (next to) no arithmetic.  n_ops times, every column tile reads the pieces of rows_per_op (1 or 2) consecutive
 * workers from x and xt, multiplies them by 1 and stores them back, the workers advancing cyclically, so that
 * a row comes back only after n / rows_per_op passes, beyond the reach of the chip's caches for the state sizes
 * this is meant for: the rate it reaches is the in-place HBM streaming rate of the machine at hand for the
 * shape of a gossip event (rows_per_op = 2: four row pieces in, four out) or of a mixing pass (1).  The state
 * is left unchanged bit for bit.  Asynchronous on the context's stream; *bytes (may be NULL) receives the
 * bytes the launch moves: n_ops * rows_per_op * 64 * floor(d / 4).  Needs 2 <= n, 1 <= n_ops. */
int a2cid_inplace_probe(a2cid_ctx *ctx, int32_t rows_per_op, int32_t n_ops, double *bytes);

/* Work enqueued since creation or the last reset: gossip and gradient events, kernel launches,
 * the byte count of one pass per event (32 d for a gossip event; 16 d for a gradient event plus
 * 4 d for each of xi, c and h that it reads; 16 d per worker mixed by a2cid_flush; 16 n d for
 * a2cid_average), and the bytes the launched kernels move by construction: the same for modes 0
 * and 1; for mode 3, 8 d for every row read from or written to memory (a2cid_plan_chain) plus the
 * gradient inputs; for modes 2 and 4, 16 d
 * per touched row and launch plus the gradient inputs.  Any output pointer may be NULL. */
int a2cid_counters(a2cid_ctx *ctx, int64_t *n_gossip, int64_t *n_gradient, int64_t *n_launches,
                   double *one_pass_bytes, double *moved_bytes, int32_t reset);

/* While enabled, every event-kernel launch and every observables-kernel launch (a2cid_stats,
 * a2cid_stats_static) is bracketed by a pair of HIP events on the context's stream.
 * a2cid_profile_read waits for the stream, returns the number of event-kernel launches timed
 * since the previous read and the sum of their durations in milliseconds, and forgets them;
 * a2cid_profile_read_stats does the same for the observables kernel (the pass over x and xt, not
 * the small kernel that adds the partial sums). */
int a2cid_profile(a2cid_ctx *ctx, int32_t enable);
int a2cid_profile_read(a2cid_ctx *ctx, int64_t *n_launches, double *kernel_ms);
int a2cid_profile_read_stats(a2cid_ctx *ctx, int64_t *n_launches, double *kernel_ms);

const char *a2cid_last_error(void);
const char *a2cid_version(void);

#ifdef __cplusplus
}
#endif
#endif /* A2CID_H */
