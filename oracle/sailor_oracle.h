/*
 * CPU oracle for the batched plan evaluator -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 / exact-integer implementation of what the planner's hot path
 * computes for every candidate plan, written from the paper (Sailor, SOSP '25):
 *   - plan tuple: stages P, data-parallel degree D shared by all stages, a
 *     (GPU type, TP, zone) choice per stage, one microbatch size      (Sec. 4.2)
 *   - heuristics H1 (TP inside a node), H5 (a stage's replicas stay in one region),
 *     H6 (zones of a region merged)                                   (Sec. 4.2.1)
 *   - memory M_peak = M_model + M_activation per worker, per stage   (Sec. 4.3)
 *   - T_iter = max(T_pp) + T_sync + T_update, 1F1B with the steady phase set by
 *     the straggler; T_total composition                             (Sec. 4.3, 4.2.2)
 *   - C_iter = C_comp + C_comm                                        (Sec. 4.3, 4.2.3)
 *   - sort by objective, return the best valid plan                   (Sec. 4.2)
 *
 * It shares no code with the HIP library and is never called by it.  Only the tests,
 * the smoke check and the benchmark's CPU-baseline leg may use it.
 *
 * Optional per-segment tensor parallelism (per_segment_tp = 1): every stage of the plan
 * tuple may carry its own TP degree (Sec. 4.2); with H1 a TP group is made of one GPU
 * type, so each contiguous segment (one pool) gets its own TP digit.  Memory shards,
 * activation bytes, profiled times, the node-size check, the gradient all-reduce, the
 * GPU count against the quota and the rent all use the degree of the stage's segment.
 *
 * Optional message-size dependent bandwidth (n_bw_coef > 0): the profiler fits, per link,
 * a polynomial of the bandwidth over the message size (Sec. 4.1) and the simulator uses
 * it for peer-to-peer transfers and collectives (Sec. 4.3).  Here the polynomial is in
 * x = log2(bytes); its value is limited to [peak / 1000, peak] with peak = bandwidth[a][b].
 * A transfer of S bytes takes S / bw(S); the all-reduce of a stage uses its gradient
 * buffer as the message size, and T_sync is the maximum over the stages.
 *
 * Optional mixed replicas (mixed_types = 1): the D replicas of a stage need not be of one GPU
 * type (the D tuples of Sec. 4.2); H5 / H6 keep them in one zone.  Here a segment may use an
 * extended type: a pair of GPU types a < b of its zone, half of the replicas on each (D must
 * be even).  Extended types are numbered after the G plain ones, pairs in lexicographic
 * order, and a pool is zone * G' + extended type with G' = G + G (G - 1) / 2.  A stage's time,
 * and its update time, are those of its slower replica type (the straggler, Sec. 4.3); both
 * types must fit their memory and node size; every real pool must hold what all segments
 * together take from it; rent is the mean of the two prices.
 *
 * Parity pins (tests/test_oracle_*.py): homogeneous 1F1B closed form, discrete-event
 * 1F1B schedule, ring all-reduce limits, big-integer memory bytes, cost identities,
 * feasibility monotonicity, brute-force selection, enumeration bijection; per-segment
 * TP: agreement with the shared-TP mode on equal degrees, hand-computed time / sync /
 * cost on mixed degrees, Python-integer memory and quota, count formula; bandwidth
 * polynomial: reduction to the constant model, hand-computed transfers and all-reduce
 * with numpy's polynomial evaluation, both limits, per-stage maximum of T_sync.
 * Against numeric outputs of the paper's own simulator: parity unpinned (the paper
 * prints no worked input -> output example).
 *
 * Units: seconds, bytes, bytes/second, $/hour, $/byte.
 */
#ifndef SAILOR_ORACLE_H
#define SAILOR_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t n_layers, n_types, n_zones, n_mb, n_tp, n_dp, n_pp;
  int32_t max_segments, seg3_max_pp, uniform_layers;
  int32_t per_segment_tp;          /* 1: every segment has its own TP degree (digit) */
  int32_t n_bw_coef;               /* 0: constant bandwidth; else coefficients per zone pair */
  int32_t mixed_types;             /* 1: a segment's replicas may be split over two GPU types */
  int64_t global_batch;
  const int32_t *mb_values, *tp_values, *dp_values, *pp_values;
  const int32_t *n_partitions;     /* [n_pp] */
  const int32_t *partition_layers; /* rows of pp layer counts, pp-major then partition */
  const uint64_t *layer_params;    /* [n_layers] */
  uint64_t embed_params, head_params;
  uint32_t bytes_per_param, grad_bytes_per_param;
  const double *t_fwd, *t_bwd;     /* [G][n_mb][n_tp][Lc], Lc = uniform ? 1 : n_layers */
  const double *t_upd;             /* [G][n_tp][Lc] */
  const uint64_t *act_store_bytes; /* [n_mb][n_tp] */
  const uint64_t *p2p_bytes;       /* [n_mb] */
  const uint64_t *mem_capacity, *mem_reserved; /* [G] */
  const int32_t *gpus_per_node;    /* [G] */
  const double *price_per_hour;    /* [G] */
  const int32_t *avail;            /* [Z][G] */
  const double *bandwidth;         /* [Z][Z] */
  const double *egress_per_byte;   /* [Z][Z] or NULL */
  const double *bw_poly;           /* [Z][Z][n_bw_coef], lowest power first, or NULL */
} so_problem;

/* a decoded candidate */
typedef struct {
  int32_t pp, pp_idx, n_segments, partition;
  int32_t cut[2];  /* first stage of segment 2 / segment 3 (unused entries = pp) */
  int32_t pool[3]; /* zone * G' + (extended) type, -1 if the segment is absent */
  int32_t dp, tp, mb, dp_idx, tp_idx, mb_idx; /* tp, tp_idx: those of segment 1 */
  int32_t seg_tp[3], seg_tp_idx[3];           /* TP degree per segment (0 / -1 if absent) */
} so_config;

typedef struct {
  uint64_t index;
  uint32_t mask;
  uint64_t peak_mem;
  double iter_time, cost;
} so_eval;

enum { SO_MAX_THROUGHPUT = 0, SO_MIN_COST = 1 };
enum {
  SO_BIT_OOM = 1u << 0, SO_BIT_QUOTA = 1u << 1, SO_BIT_BATCH = 1u << 2,
  SO_BIT_TP_NODE = 1u << 3, SO_BIT_CONSTRAINT = 1u << 5
};

typedef struct so_ctx so_ctx;

so_ctx *so_create(const so_problem *p); /* borrows the arrays; NULL on bad input */
void so_destroy(so_ctx *c);
uint64_t so_num_candidates(const so_ctx *c);

int so_decode(const so_ctx *c, uint64_t index, so_config *out);     /* 0 ok, -1 range */
int so_encode(const so_ctx *c, const so_config *cfg, uint64_t *out); /* 0 ok, -1 invalid */
/* nested-loop enumeration in index order; fills at most max_out configs, returns total */
uint64_t so_enumerate(const so_ctx *c, so_config *out, uint64_t max_out);

/* one candidate; has_bound = 0 ignores bound */
int so_eval_one(const so_ctx *c, uint64_t index, int objective, int has_bound, double bound,
                so_eval *out);
/* Discrete-event 1F1B schedule of one pipeline of the plan (the three phases Sec. 4.3 names,
 * op by op) beside the closed form sum_i t_i + (N_b - 1) max_i t_i on the same stage times.
 * 0 ok, -1 bad index, 1 batch not divisible (both outputs +inf). */
int so_simulate_1f1b(const so_ctx *c, uint64_t index, double *t_event, double *t_closed);

/* indices == NULL means first .. first+count-1 ; any output pointer may be NULL */
int so_eval_batch(const so_ctx *c, uint64_t first, uint64_t count, const uint64_t *indices,
                  int objective, int has_bound, double bound, double *time, double *cost,
                  uint64_t *mem, uint32_t *mask, int n_threads);

/* best plan over [first, first+count): min key over mask == 0, then the lowest index
 * whose key <= min * (1 + 1e-5).  Returns 1 if found, 0 if nothing is feasible. */
int so_best(const so_ctx *c, uint64_t first, uint64_t count, int objective, int has_bound,
            double bound, int n_threads, so_eval *out);
/* ascending (key, index) over mask == 0, first k; returns how many were found */
int so_topk(const so_ctx *c, uint64_t first, uint64_t count, int objective, int has_bound,
            double bound, int k, int n_threads, so_eval *out);

/* ---- plans whose stages choose their pools freely (Sec. 4.2: a (GPU, TP, zone) choice per
 * stage; Sec. 4.2.2: resources are assigned stage by stage) -------------------------------- */

/* One such plan through the simulator: pools[i] = zone * G' + extended type of stage i, one TP
 * degree for all stages.  0 ok, -1 value out of range. */
int so_eval_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx, int tp_idx,
                       const int32_t *pools, int objective, int has_bound, double bound,
                       so_eval *out);
const so_problem *so_problem_of(const so_ctx *c);

/* The same with a TP degree per stage (tp_ij of Sec. 4.2.2 taken per stage): tp_idx[i] = index
 * of stage i's degree in tp_values.  A stage's memory shard, activation bytes, profiled times,
 * node-size check, gradient shard, GPUs against its pool's quota and rent use its own degree. */
int so_eval_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                          const int32_t *tp_idx, const int32_t *pools, int objective, int has_bound,
                          double bound, so_eval *out);

/* The same with stages that may split their replicas over two pools, also of different zones:
 * pools_a[i] / pools_b[i] (equal = not split), half of the D replicas on each.  T_iter takes
 * the slower of the two kinds of pipeline (Sec. 4.3: max over pipelines), a split stage's
 * all-reduce its slowest link, the cost includes the ring's traffic between the zones. */
int so_eval_split_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                             int tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                             int objective, int has_bound, double bound, so_eval *out);

/* Both at once: two pools and a TP degree per stage (tp_idx[i], the same for both halves of the
 * stage) -- the free per-stage (GPU type, zone, TP) choice of Sec. 4.2 with two tuples per stage. */
int so_eval_split_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                const int32_t *tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                                int objective, int has_bound, double bound, so_eval *out);

/* The plan tuple in full (Sec. 4.2: D tuples per stage): every replica of every stage names its
 * pool, pools[i * D + r] for stage i and replica r.  Replica r of all stages forms pipeline r;
 * T_iter = max over the D pipelines + T_sync + T_update (Sec. 4.3).  A stage's gradient all-reduce
 * is a ring through its replicas in their order (r -> r + 1 -> ... -> 0) at the pace of its
 * slowest link; traffic between zones is paid for where a pipeline or a ring crosses.  Quotas
 * count the GPUs every pool gives, memory and node size hold for every replica's type, one TP
 * degree per plan.  With all replicas of a stage on one pool this is so_eval_assignment, with
 * the first half on one pool and the second half on another so_eval_split_assignment (D >= 4).
 * Returns 0, -1 for a value out of range or a problem with extended types. */
int so_eval_replica_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                               int tp_idx, const int32_t *pools, int objective, int has_bound,
                               double bound, so_eval *out);

/* The same with a TP degree per stage (tp_idx[i]; all replicas of a stage run at it): the
 * D tuples (GPU type, TP, zone) of every stage with TP taken per stage. */
int so_eval_replica_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                  const int32_t *tp_idx, const int32_t *pools, int objective,
                                  int has_bound, double bound, so_eval *out);

#define SO_SEARCH_MAX_STAGES 256
typedef struct {
  int32_t found;                 /* 1: a valid plan exists (within the incumbent, if one was given) */
  int32_t truncated;             /* beam: some frontier was cut to the beam width */
  int32_t pp_idx, partition, tp_idx, dp_idx, mb_idx, pp;
  uint64_t expanded;             /* placements generated */
  double key, iter_time, cost;
  int32_t pools[SO_SEARCH_MAX_STAGES];
  int32_t pools_b[SO_SEARCH_MAX_STAGES]; /* pool of the other half of a stage's replicas (= pools[i]
                                            when the stage is not split) */
  int32_t tps[SO_SEARCH_MAX_STAGES];     /* index of every stage's TP degree (= tp_idx unless the
                                            stages choose their own) */
} so_search_result;

typedef struct {
  int32_t beam_width;            /* longest frontier kept per sub-problem */
  int32_t max_runs;              /* 0: any placement; n: at most n runs of equal pools */
  int32_t has_incumbent;         /* 1: placements whose bound exceeds `incumbent` are dropped */
  double incumbent;
  int32_t allow_split;           /* 1: a stage may put half of its replicas on a second pool, also
                                    of another zone (so_eval_split_assignment); a stage then has
                                    (pools)^2 choices (a, b), numbered a * pools + b */
  int32_t stage_tp;              /* 1: every stage chooses its TP degree too (so_eval_assignment_tp);
                                    a stage has pools x n_tp choices (a, t), numbered a * n_tp + t,
                                    and TP leaves the sub-problem.  Not together with allow_split */
} so_search_opts;

/* (sailor_search_oracle.c) sub-problems in the order pp, layer split, TP, D, microbatch size;
 * equal keys: the first sub-problem, inside it the first placement found.  0 ok, -1 when the
 * problem uses an option the search does not cover. */
int so_search_exhaustive(const so_ctx *c, int objective, int has_bound, double bound, int max_runs,
                         int allow_split, int stage_tp, so_search_result *out);
int so_search_beam(const so_ctx *c, int objective, int has_bound, double bound,
                   const so_search_opts *opt, so_search_result *out);
int so_search_prefix_bound(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                           int tp_idx, const int32_t *pools, int n_placed, int objective,
                           double *lb_time, double *lb_cost);
int so_search_prefix_bound_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                              const int32_t *tp_idx, const int32_t *pools, int n_placed, int objective,
                              double *lb_time, double *lb_cost);
int so_search_prefix_bound_split_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                    const int32_t *tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                                    int n_placed, int objective, double *lb_time, double *lb_cost);

#ifdef __cplusplus
}
#endif
#endif
