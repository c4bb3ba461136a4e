/*
 * sailor.h -- C ABI of the batched plan evaluator (HIP, gfx950).
 *
 * The library evaluates every candidate training-job plan of a planning problem
 * through the runtime / memory / cost simulator of Sailor (SOSP '25, Sec. 4.3) and
 * selects the best valid plans under an objective and an optional constraint
 * (Sec. 4, Sec. 4.2).  All evaluation runs in GPU kernels; the host only validates,
 * uploads tables, launches and decodes the winning indices into plan tuples.
 *
 * Conventions
 *   - every call returns a sailor_status; out-parameters are untouched on error
 *   - "host" / "device" says where a pointer must live; device pointers belong to the
 *     HIP device that was current when the plan was created
 *   - units: seconds, bytes, bytes/second, $/hour, $/byte
 *   - a plan object is not thread-safe; different plans are independent
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream)
 *
 * Candidate space (plan tuple of Sec. 4.2: stages P, one data-parallel degree D for all
 * stages, a (GPU type, TP, zone) choice per stage, one microbatch size).  A plan's P
 * stages are cut into 1..3 contiguous segments; each segment runs on one pool
 * a = zone * n_types + type; neighbouring segments use different pools; one TP degree
 * per plan.  Candidates are numbered block by block, blocks ordered by pp index, then
 * by segment count s (a block exists when s <= max_segments, s <= P and, for s = 3,
 * P <= seg3_max_pp).  Inside a block the index is mixed radix, least significant digit
 * first:
 *     mb index, tp index, dp index, pool of segment 1,
 *     [s >= 2: r2 in [0, ZG-1), pool2 = (pool1 + 1 + r2) mod ZG],
 *     [s == 3: r3 in [0, ZG-1), pool3 = (pool2 + 1 + r3) mod ZG],
 *     [s == 2: k - 1 in [0, P-1), segment 1 = stages [0, k)],
 *     [s == 3: rank of (k1, k2), 1 <= k1 < k2 <= P-1, in lexicographic order],
 *     partition index q in [0, n_partitions[pp index]).
 * The numbering is part of the contract: the tie rule prefers the lowest index.
 *
 * per_segment_tp = 1 gives every segment its own TP degree, the (GPU type, TP, zone)
 * choice per stage of Sec. 4.2 under H1 (a TP group consists of one GPU type, and a
 * segment runs on one).  The "tp index" digit above is then segment 1's, and the digit
 * "tp index of the segment" follows r2 (segment 2) and r3 (segment 3).  A stage's
 * memory shard, activation bytes, profiled times, node-size check, gradient shard,
 * GPU count and rent use the degree of its segment.
 *
 * mixed_types = 1 lets the D replicas of a stage be of two GPU types (the D tuples of the plan,
 * Sec. 4.2; H5 / H6 keep them in one zone).  A segment then chooses among G' = G + G (G - 1) / 2
 * extended types: the G plain ones, then every pair a < b in lexicographic order, half of the
 * replicas on each (D must be even).  Wherever the numbering above says "pool" it is
 * zone * G' + extended type, and ZG = n_zones * G' (at most SAILOR_MAX_POOLS).  A stage of a
 * pair runs, and updates, at the pace of its slower type (the straggler of Sec. 4.3); both
 * types must fit their memory and node size; every real (zone, type) pool must hold what all
 * segments of the plan together take from it, else OVER_QUOTA; the rent is the mean of the
 * two prices.
 *
 * Beyond the enumerated space (further down): sailor_search places the stages of a pipeline one
 * by one -- a pool per stage, optionally a second pool for half of its replicas, a TP degree of
 * its own, or both -- with lower bounds and a beam (Sec. 4.2.1, 4.2.2); sailor_eval_placements and
 * sailor_eval_replica_placements run the simulator of Sec. 4.3 on listed plans of that kind, down
 * to a pool per replica of every stage; sailor_simulate_1f1b replays a plan's 1F1B schedule op by op.
 *
 * Mask bits of an evaluated candidate (0 = valid plan)
 *   bit 0 OOM               some stage's worker exceeds its GPU's memory (Sec. 4.3)
 *   bit 1 OVER_QUOTA        a pool needs more GPUs than are available (Sec. 4)
 *   bit 2 BATCH_INDIVISIBLE global batch not divisible by D * mb; then time = cost =
 *                           +inf, mem = 0 and no other bit is set
 *   bit 3 TP_EXCEEDS_NODE   heuristic H1 (Sec. 4.2.1)
 *   bit 5 CONSTRAINT        the optional bound is violated (Sec. 4.2)
 */
#ifndef SAILOR_H
#define SAILOR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sailor_plan sailor_plan; /* opaque, owned by the library */

typedef enum {
  SAILOR_OK = 0,
  SAILOR_EINVAL = -1,      /* NULL pointer, malformed list or table, limit exceeded */
  SAILOR_ENOMEM = -2,      /* host or device allocation failed, or an internal buffer overflowed */
  SAILOR_EDEVICE = -3,     /* a HIP call failed */
  SAILOR_ERANGE = -4,      /* candidate index or range outside [0, N) */
  SAILOR_ENOFEASIBLE = -5  /* no candidate has mask == 0 */
} sailor_status;

typedef enum { SAILOR_MAX_THROUGHPUT = 0, SAILOR_MIN_COST = 1 } sailor_objective;

enum {
  SAILOR_MASK_OOM = 1u << 0,
  SAILOR_MASK_OVER_QUOTA = 1u << 1,
  SAILOR_MASK_BATCH_INDIVISIBLE = 1u << 2,
  SAILOR_MASK_TP_EXCEEDS_NODE = 1u << 3,
  SAILOR_MASK_CONSTRAINT = 1u << 5
};

/* Limits checked by sailor_plan_create. */
enum {
  SAILOR_MAX_POOLS = 128, /* n_zones * n_types, and n_zones * G' with mixed_types; the records of
                             3 * pools * n_mb (segment, pool, microbatch size) triples, 36 bytes
                             each, and n_mb * n_zones^2 transfer entries of 16 bytes must also fit
                             the 160 KiB of local memory of a compute unit */
  SAILOR_MAX_TYPES = 16,
  SAILOR_MAX_ZONES = 16,
  SAILOR_MAX_MB = 8,
  SAILOR_MAX_TP = 8,
  SAILOR_MAX_DP = 24,
  SAILOR_MAX_STAGES = 256,
  SAILOR_MAX_SHAPES = 1 << 20, /* (layer split, cut points) combinations over all pp */
  SAILOR_MAX_BW_COEF = 8, /* coefficients of a link's bandwidth polynomial */
  SAILOR_MAX_K = 4096,    /* largest k of sailor_topk */
  SAILOR_STATIC_SCRATCH_BYTES = 8 << 20, /* device array behind sailor_simulate_1f1b_static */
  SAILOR_STATIC_MAX_PLANS = 4096         /* most plans one call of it takes */
};

/*
 * The planning problem: job profile, cluster, search lists (inputs of the planner,
 * Sec. 4 and Sec. 4.1).  All arrays are host memory, row-major, caller-owned and copied
 * during sailor_plan_create; the caller may free them when it returns.
 * G = n_types, Z = n_zones, Lc = uniform_layers ? 1 : n_layers.
 */
typedef struct {
  int32_t n_layers, n_types, n_zones, n_mb, n_tp, n_dp, n_pp;
  int32_t max_segments;    /* 1, 2 or 3 */
  int32_t seg3_max_pp;     /* a third segment only for pp <= this */
  int32_t uniform_layers;  /* 1: time tables hold a single per-layer column */
  int32_t per_segment_tp;  /* 1: every segment has its own TP digit; 0: one TP per plan */
  int32_t n_bw_coef;       /* coefficients per link in bw_poly, 0..SAILOR_MAX_BW_COEF; 0: every
                              message sees bandwidth[a][b] */
  int32_t mixed_types;     /* 1: a segment's replicas may be split over two GPU types */
  int64_t global_batch;    /* never changed by the planner (Sec. 4.2) */
  const int32_t *mb_values, *tp_values, *dp_values, *pp_values; /* positive, strictly ascending */
  const int32_t *n_partitions;     /* [n_pp], >= 1 */
  const int32_t *partition_layers; /* for each pp index, n_partitions rows of pp layer counts,
                                      each >= 1, each row summing to n_layers */
  const uint64_t *layer_params;    /* [n_layers] parameters per layer */
  uint64_t embed_params, head_params; /* charged to the first / the last stage */
  uint32_t bytes_per_param;        /* weights + gradients + optimizer state per parameter */
  uint32_t grad_bytes_per_param;   /* bytes all-reduced per parameter */
  const double *t_fwd, *t_bwd;     /* [G][n_mb][n_tp][Lc] seconds per layer */
  const double *t_upd;             /* [G][n_tp][Lc] seconds per layer */
  const uint64_t *act_store_bytes; /* [n_mb][n_tp] stored activations per layer per
                                      in-flight microbatch */
  const uint64_t *p2p_bytes;       /* [n_mb] activation bytes sent between two stages */
  const uint64_t *mem_capacity;    /* [G] */
  const uint64_t *mem_reserved;    /* [G] buffers / fragmentation, added to every worker */
  const int32_t *gpus_per_node;    /* [G] */
  const double *price_per_hour;    /* [G] */
  const int32_t *avail;            /* [Z][G] GPUs available now, >= 0 */
  const double *bandwidth;         /* [Z][Z] bytes/s from row zone to column zone, > 0;
                                      the diagonal is the intra-zone link */
  const double *egress_per_byte;   /* [Z][Z] $/byte, >= 0, or NULL for zeros */
  const double *bw_poly;           /* [Z][Z][n_bw_coef], lowest power first, finite; NULL when
                                      n_bw_coef = 0.  Message-size profile of a link (cluster
                                      profiling, Sec. 4.1): a message of S >= 1 bytes from zone a
                                      to zone b sees the polynomial's value at x = log2(S),
                                      limited to [bandwidth[a][b] / 1000, bandwidth[a][b]], and
                                      takes S / that.  Used for activation / gradient transfers
                                      between stages (S = p2p_bytes[mb]) and for the gradient
                                      all-reduce of a stage (S = its gradient buffer), Sec. 4.3 */
} sailor_problem;

/* Optional bound: SAILOR_MAX_THROUGHPUT -> bound is the largest allowed $/iteration;
 * SAILOR_MIN_COST -> bound is the smallest allowed iterations/second. */
typedef struct {
  double bound;
  int32_t has_bound;
} sailor_constraint;

/* One decoded (and, where stated, evaluated) plan. */
typedef struct {
  uint64_t index;
  uint64_t peak_mem_bytes;
  double iter_time_s, cost_per_iter; /* evaluated in fp64 on the device */
  uint32_t mask;
  int32_t pp, tp, dp, mb;
  int32_t pp_index, tp_index, dp_index, mb_index;
  int32_t partition, n_segments;
  int32_t cut[2];  /* first stage of segment 2 / 3; unused entries = pp */
  int32_t pool[3]; /* zone * G' + (extended) type, G' = n_types unless mixed_types;
                      unused entries = -1 */
  int32_t seg_tp[3];       /* TP degree of each segment; unused entries = 0 */
  int32_t seg_tp_index[3]; /* its index in tp_values; unused entries = -1;
                              tp / tp_index above are those of segment 1 */
  int32_t zone[3];         /* zone of each segment; unused entries = -1 */
  int32_t type_a[3];       /* GPU type of each segment's replicas ... */
  int32_t type_b[3];       /* ... and of the other half of them (= type_a unless mixed) */
} sailor_result;

/* The planner's inputs (Sec. 4: job profile, quotas and current availability, prices; Sec. 4.1:
 * per-layer times and memory per GPU type, link bandwidths) become a plan object.
 * Build a plan: validate, copy the problem to the current HIP device, build the static
 * per-stage and per-segment tables there, and run three to four passes over the space that
 * decide how later scans are launched (which pieces of the space can never hold a valid plan,
 * how long the others take); results do not depend on that.  *out receives the plan.
 * (sailor_set_scan_unit_parts overrides how the pieces are cut.)
 * Errors: SAILOR_EINVAL (see limits and field comments), SAILOR_ENOMEM, SAILOR_EDEVICE. */
sailor_status sailor_plan_create(const sailor_problem *problem, sailor_plan **out);

/* Tuning and testing, process-wide, for plans created afterwards: n = 0 (default) lets the
 * times measured at plan creation decide which pieces of the space are cut into parts for the
 * scan; n = 1..255 cuts every piece into n parts instead.  Results never depend on it.
 * SAILOR_EINVAL outside 0..255. */
sailor_status sailor_set_scan_unit_parts(int32_t n);

/* Free everything the plan owns (host and device).  NULL is accepted. */
sailor_status sailor_plan_destroy(sailor_plan *plan);

/* Replace the availability table ([Z][G], host) -- the only input that changes between
 * re-plans when resources come and go (Sec. 4, Sec. 4.4).  Tables that do not depend on
 * availability are kept (cf. the reuse noted under H2, Sec. 4.2.1).  The table is copied
 * before the call returns; it reaches the device, and the quota table derived from it is
 * rebuilt there, at the start of the next evaluation or selection call, on that call's
 * stream. */
sailor_status sailor_plan_set_avail(sailor_plan *plan, const int32_t *avail);

/* Re-planning (Sec. 4.4: the planner is invoked again whenever the availability changes;
 * H2, Sec. 4.2.1: what does not depend on the availability is reused).  The library keeps, for
 * every piece of the space (one layer split and cut, one TP degree per segment, a range of
 * pools), the best key of its last full evaluation.  While the query (objective and bound) stays
 * the same, sailor_best_plan / sailor_topk evaluate again only the pieces in which some plan's
 * validity can have changed: a piece gathers, as always, the bits that say for which
 * data-parallel degrees each of its segments fits each pool (memory, quota, node size, batch),
 * compares them with those of its last evaluation -- integers only -- and is evaluated again
 * only if one differs.  The other pieces contribute their kept minima.  Results are identical
 * to a full evaluation.  (sailor_plan_last_scan copies a small per-piece table from the device
 * and waits for it.)
 * on = 0 (default): every call evaluates the whole space; on = 1: minima are kept and reused.
 * What it buys depends on the stream: the pieces whose validity changes are mostly the ones
 * that hold many valid plans, and those set the duration of a pass over the space, while a
 * pass that reuses minima needs one more small kernel to list the pieces near the minimum;
 * on the synthetic streams measured here it shortens the pass by a third and the call not at
 * all. */
sailor_status sailor_plan_set_incremental(sailor_plan *plan, int32_t on);

/* Pieces of the space the last successful sailor_best_plan / sailor_topk evaluated, and how
 * many there are.  Not counted as evaluated: pieces whose minima were reused, and pieces passed
 * over because a bound computed at sailor_plan_create proves that they hold nothing for the
 * query (the smallest cost, or time, of any plan of the piece whatever the availability
 * already violates the constraint; for the best plan also: its smallest objective value
 * cannot come within the tie band of a plan already seen) -- Sec. 4.2.1, H3, applied to a
 * piece instead of a partial plan.  When a query's constraint leaves at most 128
 * pieces alive the library visits exactly those in one pass and keeps every valid plan of
 * theirs (no pass over the other pieces, no threshold); units_evaluated is then their number.
 * Copies a small per-piece table from the device and waits for it.  Host pointers, either may
 * be NULL.  SAILOR_EINVAL before the first
 * successful selection. */
sailor_status sailor_plan_last_scan(sailor_plan *plan, uint32_t *units_evaluated,
                                    uint32_t *units_total);

/* Number of candidates N. */
sailor_status sailor_plan_num_candidates(const sailor_plan *plan, uint64_t *out);

/* Decode an index into the configuration fields of *out (host only, nothing is
 * evaluated: peak_mem_bytes, times, cost and mask are set to 0).  SAILOR_ERANGE if
 * index >= N. */
sailor_status sailor_plan_decode(const sailor_plan *plan, uint64_t index, sailor_result *out);

/* Evaluate candidates (Sec. 4.3: memory footprint, iteration time, cost per iteration,
 * plus the validity mask).  d_indices == NULL evaluates first .. first+count-1, otherwise
 * the count indices stored in device memory at d_indices (first is ignored).  Output
 * arrays are device memory of count elements; any may be NULL.  fp32 time and cost,
 * exact 64-bit bytes.  Asynchronous on hip_stream.  constraint may be NULL.
 * Errors: SAILOR_ERANGE if the range leaves [0, N); an index >= N inside d_indices yields
 * mask = 0xFFFFFFFF, time = cost = +inf, mem = 0. */
sailor_status sailor_eval_batch(sailor_plan *plan, uint64_t first, uint64_t count,
                                const uint64_t *d_indices, sailor_objective objective,
                                const sailor_constraint *constraint, float *d_time,
                                float *d_cost, uint64_t *d_mem, uint32_t *d_mask,
                                void *hip_stream);

/* Best valid plan over the whole space (Sec. 4.2: order by the objective, return the
 * best): the minimum key (iteration time or cost) over mask == 0, then the lowest index
 * whose key is within a relative 1e-5 of that minimum.  *out (host) is filled completely.
 * Returns when the result has arrived in host memory: everything enqueued on hip_stream
 * before the call has finished by then, the call's last dispatch may still be retiring.
 * SAILOR_ENOFEASIBLE when no candidate is valid. */
sailor_status sailor_best_plan(sailor_plan *plan, sailor_objective objective,
                               const sailor_constraint *constraint, sailor_result *out,
                               void *hip_stream);

/* Sec. 4.2: the planner "sorts the configurations according to the objective"; this returns the
 * head of that order.
 * The k best valid plans in ascending (key, index) order; out (host) has room for k
 * entries, *n_found receives how many exist (<= k).  1 <= k <= SAILOR_MAX_K.
 * Keys, and the constrained quantity against the bound, are the fp64 values reported in out:
 * plans whose values agree to the last few bits (or a value that equals the bound to the
 * last bit) are ordered (decided) by those bits, which depend on the order of the additions.
 * Waits like sailor_best_plan.  SAILOR_ENOFEASIBLE (with *n_found = 0) when none is valid. */
sailor_status sailor_topk(sailor_plan *plan, sailor_objective objective,
                          const sailor_constraint *constraint, int32_t k, sailor_result *out,
                          int32_t *n_found, void *hip_stream);

/* Resize the device scratch of the selection: the list of candidates that survive the fp32
 * scan (24 B each, default 4 Mi entries) and the list re-evaluated in fp64 (40 B each,
 * default 256 Ki entries).  sailor_topk searches for a tighter threshold when the first
 * list would overflow; a call fails with SAILOR_ENOMEM only when more candidates than fit
 * lie within the rounding band of the k-th key (or, for sailor_best_plan, within the tie
 * tolerance of the minimum).  Waits for the device.  SAILOR_EINVAL for a zero size. */
sailor_status sailor_plan_set_scratch(sailor_plan *plan, uint32_t max_survivors,
                                      uint32_t max_refined);

/* Measurement only.  mode 0 (default): no events are recorded.  mode 1: the dominant kernel
 * of each call (the full-space scan of sailor_best_plan / sailor_topk, the evaluation kernel
 * of sailor_eval_batch) is launched with start and stop events on its stream.  mode 2: in
 * addition two events bracket all kernels of a sailor_best_plan / sailor_topk call.  A
 * dispatch that carries events is completed and timestamped apart from its neighbours, which
 * lengthens the call by some 15 us: time a sample of the calls, not every one. */
sailor_status sailor_plan_set_timing(sailor_plan *plan, int32_t mode);

/* Milliseconds measured by the last call on this plan under the timing mode above:
 * *total_ms (mode 2, else 0) and *kernel_ms (mode >= 1).  Waits for the events.
 * SAILOR_EINVAL if the last call recorded nothing. */
sailor_status sailor_plan_last_timing(sailor_plan *plan, float *total_ms, float *kernel_ms);

/* The 1F1B schedule of one pipeline of each listed plan, op by op (warm-up, steady and
 * cool-down phases, Sec. 4.3), beside the closed form sum_i t_i + (N_b - 1) max_i t_i that the
 * evaluator uses for T_pp (Sec. 4.2.2), on the same stage times.  A forward of stage i takes
 * its layers' forward time plus the transfer to stage i + 1, a backward its backward time plus
 * the transfer to stage i - 1; a forward waits for the previous stage's forward of the same
 * microbatch, a backward for the next stage's backward.  Quantifies the closed form's error
 * for plans that a selection returned.
 *   d_indices  device, [count] candidate indices
 *   d_event    device, [count] fp64 makespan of the schedule, or NULL
 *   d_closed   device, [count] fp64 closed form, or NULL (not both NULL)
 * A plan whose batch does not divide yields +inf, an index outside [0, N) NaN.  Work per plan
 * is about 2 (N_b + P) dependent steps of one workgroup.  Asynchronous on hip_stream, except
 * for pipelines deeper than about 60 stages, whose working set is allocated, used and freed
 * inside the call (it then synchronises the stream).
 * SAILOR_ERANGE: count > 2^31 - 1, or more than 2^24 microbatches per pipeline. */
sailor_status sailor_simulate_1f1b(sailor_plan *plan, uint64_t count, const uint64_t *d_indices,
                                   double *d_event, double *d_closed, void *hip_stream);

/* sailor_simulate_1f1b for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  (sailor_simulate_1f1b itself
 * allocates, synchronises and frees inside the call when a pipeline is deeper than about 60
 * stages.)  Same arguments, same results bit for bit; the schedule's working set -- per plan two
 * rings of end times per stage -- always lives in one file-scope device array of
 * SAILOR_STATIC_SCRATCH_BYTES that every GPU the library runs on holds from load to exit.  The
 * call allocates and frees nothing, never synchronises, and only enqueues kernels on
 * hip_stream; plans are processed in batches of as many as fit the array, one launch per batch.
 * Nothing in the array has to start at zero (a slot is read only after the stage that produces
 * it has written it in the same launch), so nothing is cleared.  All calls on one GPU share the
 * array: calls that overlap on one GPU (different streams or host threads) race and must be
 * serialised by the caller.
 * SAILOR_ERANGE (with a message on stderr): count > SAILOR_STATIC_MAX_PLANS, the rings of one
 * plan of the deepest pipeline exceed the array, or more than 2^24 microbatches per pipeline. */
sailor_status sailor_simulate_1f1b_static(sailor_plan *plan, uint64_t count,
                                          const uint64_t *d_indices, double *d_event,
                                          double *d_closed, void *hip_stream);

/* ---- plans whose stages choose their pools freely ---------------------------------------- */

/* Options of sailor_search. */
typedef struct {
  int32_t beam_width;     /* 1 .. 1024: longest frontier kept per sub-problem */
  int32_t max_runs;       /* 0: any placement; n: at most n runs of consecutive stages on one pool
                             (3 = the candidate space of sailor_best_plan when that space allows
                             three segments at every depth) */
  int32_t use_incumbent;  /* 0: none; 1: `incumbent` below; 2: sailor_best_plan runs first and its
                             key, times 1 + 1e-9, is the incumbent */
  double incumbent;       /* placements whose bound exceeds it are dropped, complete plans too */
  int32_t allow_split;    /* 1: a stage may put half of its D replicas on a second pool, also of
                             another zone (see sailor_eval_placements); a stage then has
                             (pools)^2 choices (a, b) */
  int32_t stage_tp;       /* 1: every stage chooses its TP degree too (tp_ij of Sec. 4.2.2, taken
                             per stage): a stage has pools x n_tp choices, TP is no longer part
                             of the sub-problem, a pool's quota counts the GPUs of one replica.
                             Together with allow_split a stage chooses (a, b, TP degree): two
                             (GPU type, zone) tuples and one degree for both halves,
                             (pools)^2 x n_tp choices */
} sailor_search_options;

/* A plan with one pool per stage (plan tuple of Sec. 4.2). */
typedef struct {
  int32_t found;          /* 1: a valid plan (no worse than the incumbent, if any) exists */
  int32_t exact;          /* 1: no frontier was cut, the plan is the optimum over all placements */
  int32_t pp, tp, dp, mb;
  int32_t pp_index, tp_index, dp_index, mb_index, partition;
  uint32_t mask;            /* of the winner's re-evaluation (0) */
  uint64_t peak_mem_bytes;  /* of the winner's re-evaluation */
  double iter_time_s, cost_per_iter; /* as the search accumulated them (stage order, fp64) */
  double eval_time_s, eval_cost;     /* the same plan through sailor_eval_placements */
  uint64_t expanded;        /* placements (partial and complete) generated */
  int32_t incumbent_used;
  double incumbent;
  int32_t pool[SAILOR_MAX_STAGES]; /* zone * n_types + type of every stage; unused entries -1 */
  int32_t pool_b[SAILOR_MAX_STAGES]; /* pool of the other half of the stage's replicas (= pool[i]
                                        unless the stage is split) */
  int32_t stage_tp_index[SAILOR_MAX_STAGES]; /* index of every stage's TP degree (= tp_index unless
                                        the stages choose their own; then tp / tp_index are
                                        stage 0's) */
} sailor_stage_plan;

/* Search on top of the evaluator for spaces too large to enumerate (Sec. 4.2.2: resources are
 * assigned stage by stage, Eq. (1); Sec. 4.2.1, H3 / H4: stop where nothing better can follow;
 * Sec. 4.2.3: the budget prunes partial assignments).  Every stage chooses its pool freely,
 * all D replicas of a stage on it (H5), one TP degree per plan.  For every sub-problem
 * (pipeline depth, layer split, TP, D, microbatch size) the stages are placed in order; a
 * partial placement carries a lower bound on T_iter and C_iter (Sec. 4.3) of all its
 * completions -- placed stages at their cost, later stages at their cheapest admissible choice
 * (memory, node size), the open stage's forward transfer as zero -- and is dropped when the
 * bound breaks the constraint or exceeds the incumbent; a frontier longer than beam_width keeps
 * the smallest bounds (ties: the order of generation).  While no frontier is cut (*out.exact)
 * the result is the optimum over all placements; otherwise it is the best plan these steps
 * reach.  Equal keys: the first sub-problem in the order pp, layer split, TP, D, microbatch
 * size.  All arithmetic is fp64 in stage order, so the reported values are those of the plan.
 * With allow_split the two halves of the replicas form two kinds of pipeline, kept apart in the
 * bounds (the slower counts, Sec. 4.3), and the D tuples of a stage (Sec. 4.2) may lie in two
 * zones; unsplit stages cost what they cost without the option.  With stage_tp a run of the run
 * limit ends where the pool or the degree changes, and "cheapest admissible choice" runs over the
 * (type, TP) pairs that fit.  With both, both hold: two kinds of pipeline at the stage's degree,
 * a pool's quota counting the GPUs of one replica once per half.
 * per_segment_tp only shapes the enumerated space (and the incumbent taken from it); the search
 * does not look at it.  Not for problems with mixed_types or bw_poly, more than 64 pools or 255
 * stages (SAILOR_EINVAL).  Waits for the device.  SAILOR_ENOFEASIBLE (out->found = 0, exact and
 * expanded still set) when no valid plan is found. */
sailor_status sailor_search(sailor_plan *plan, sailor_objective objective,
                            const sailor_constraint *constraint,
                            const sailor_search_options *options, sailor_stage_plan *out,
                            void *hip_stream);

/* The simulator (Sec. 4.3) for listed plans of that kind, fp64, exact bytes:
 *   d_desc    device, [count][5]: pp index, partition, TP index, D index, microbatch index
 *   d_pools   device, [count][pool_stride]: pool of every stage (pool_stride >= pp)
 *   d_pools_b device, same shape, or NULL.  Given, a stage's D replicas are split, half on
 *             d_pools' pool and half on d_pools_b's -- any two pools, also of different zones
 *             (the D tuples (GPU, TP, zone) of a stage, Sec. 4.2); equal entries = not split.
 *             The replicas on the first pools and those on the second pools form two kinds of
 *             pipeline and T_iter = max over them + T_sync + T_update (Sec. 4.3); the all-reduce
 *             of a split stage is a ring through both pools at the pace of its slowest link
 *             (both zones' own links and the two between them); traffic between zones is paid
 *             for: the pipelines' (each kind carries D / 2 replicas) and the ring's two
 *             crossings of 2 (D - 1) / D x gradient bytes; memory and node size hold for both
 *             halves, quotas count halves, an odd D with a split stage is OVER_QUOTA
 *   d_tps     device, same shape, or NULL.  Given, stage i runs at TP degree tp_values[d_tps[..][i]]
 *             instead of the descriptor's: its memory shard, activation bytes, profiled times,
 *             node-size check, gradient shard, GPUs against its pool's quota and rent use it
 *             (tp_ij of Sec. 4.2.2).  Together with d_pools_b both halves of a stage run at
 *             the stage's degree: two (GPU type, zone) tuples and a TP degree per stage
 *   outputs   device, [count], any may be NULL
 * A descriptor, pool or TP index out of range yields mask = 0xFFFFFFFF, time = cost = +inf, mem = 0; a
 * batch that does not divide mask = BATCH_INDIVISIBLE with +inf and 0.  Asynchronous on
 * hip_stream.  SAILOR_EINVAL for mixed_types problems or more than 64 pools. */
sailor_status sailor_eval_placements(sailor_plan *plan, uint64_t count, const int32_t *d_desc,
                                     const int32_t *d_pools, const int32_t *d_pools_b,
                                     const int32_t *d_tps, uint32_t pool_stride,
                                     sailor_objective objective,
                                     const sailor_constraint *constraint, double *d_time,
                                     double *d_cost, uint64_t *d_mem, uint32_t *d_mask,
                                     void *hip_stream);

/* The plan tuple in full (Sec. 4.2: a stage has D tuples (GPU, TP, zone), one per replica): every
 * replica of every stage names its pool -- uneven splits of a stage's replicas, any number of
 * pools per stage.
 *   d_desc    device, [count][5]: pp index, partition, TP index, D index, microbatch index
 *   d_pools   device, [count][stride] with stride >= P x D: the pool of replica r of stage i at
 *             i * D + r
 *   d_tps     device, [count][tps_stride] with tps_stride >= P, or NULL: the TP index of every
 *             stage, at which all replicas of the stage run, instead of the descriptor's (the
 *             stage's memory shard, activation bytes, profiled times, node-size check, gradient
 *             shard, GPUs against the quotas and rent use it)
 * Replica r of all stages forms pipeline r, with its own stage times and transfers, and
 * T_iter = max over the D pipelines + T_sync + T_update (Sec. 4.3).  The gradient all-reduce of
 * a stage is a ring through its replicas in their order (0 -> 1 -> ... -> D - 1 -> 0) at the
 * pace of its slowest link, 2 (D - 1) / D x gradient bytes over it.  Traffic between zones is
 * paid for where a pipeline crosses (both directions' prices per microbatch, as everywhere) and
 * where a ring link crosses (that direction's price).  Memory and node size hold for every
 * replica's GPU type, a pool's quota counts the GPUs it gives, one TP degree per plan or per
 * stage.  With all replicas of a stage on one pool the values are those of
 * sailor_eval_placements.
 * Outputs and errors as for sailor_eval_placements (an invalid row also when stride < P x D,
 * tps_stride < P or D > 65 536).
 * Asynchronous on hip_stream.  SAILOR_EINVAL for mixed_types problems or more than 64 pools. */
sailor_status sailor_eval_replica_placements(sailor_plan *plan, uint64_t count, const int32_t *d_desc,
                                             const int32_t *d_pools, uint64_t stride,
                                             const int32_t *d_tps, uint32_t tps_stride,
                                             sailor_objective objective,
                                             const sailor_constraint *constraint, double *d_time,
                                             double *d_cost, uint64_t *d_mem, uint32_t *d_mask,
                                             void *hip_stream);

/* Sizes of the intermediate lists of the last successful sailor_best_plan / sailor_topk
 * (the selection of Sec. 4.2 runs as fp32 scan -> survivors -> fp64 re-evaluation):
 * candidates kept by the fp32 threshold, candidates re-evaluated in fp64, and how many of
 * those were valid.  Host pointers, any may be NULL.  SAILOR_EINVAL before the first
 * successful selection. */
sailor_status sailor_plan_last_counts(const sailor_plan *plan, uint32_t *survivors,
                                      uint32_t *refined, uint32_t *feasible);

#ifdef __cplusplus
}
#endif
#endif
