/*
 * CPU oracle of the search over per-stage placements -- TEST INFRASTRUCTURE ONLY.
 *
 * The planner assigns resources stage by stage (Sec. 4.2.2, Eq. (1): give stage i resources
 * r, leave R - r to the stages behind it, compose the times with T_total).  Here every stage
 * of a pipeline chooses its pool (zone, GPU type) freely, all D replicas of a stage on that
 * pool (H5), one TP degree per plan; (P, layer split, TP, D, microbatch size) is a
 * "sub-problem", as in the planner's outer loops (Sec. 4.2).
 *
 *   so_search_exhaustive   the definition: every placement of every sub-problem is evaluated
 *                          by the plain simulator (so_eval_assignment) and the smallest key
 *                          over valid plans wins.  Exponential; for tiny problems.
 *   so_search_beam         the algorithm, step by step: stages are placed in order, a frontier
 *                          of partial placements per sub-problem, each with a lower bound on
 *                          the key of every completion; partial placements whose bound exceeds
 *                          an incumbent (or violates the constraint) are dropped, and a
 *                          frontier longer than the beam width keeps the placements with the
 *                          smallest bounds.  While no frontier is cut the result is the
 *                          optimum (every dropped placement is provably no better than the
 *                          incumbent); otherwise it is what these steps produce.
 *
 * Bound of a partial placement (stages 0..i placed): every term of T_iter and C_iter
 * (Sec. 4.3) is monotone in the per-stage quantities, so the placed stages contribute what
 * they are known to cost and every later stage its cheapest admissible choice (memory and
 * node size respected, quotas ignored), the open stage's forward transfer counted as zero.
 * At i = P - 1 the bound is the plan's T_iter / C_iter itself, added up in stage order like
 * the simulator does.
 *
 * With stage_tp every stage also chooses its TP degree (tp_ij of Sec. 4.2.2, taken per stage):
 * a choice is (pool, TP), TP leaves the sub-problem, a pool's quota is counted in GPUs of one
 * replica, and "cheapest admissible choice" runs over (type, TP) pairs that fit.
 *
 * Pins (tests/test_oracle_search.py): beam with an unbounded width equals the exhaustive
 * search on tiny problems; restricted to three contiguous runs it equals the flat space's
 * optimum (so_best); the returned placement re-evaluates to the reported values; a wider beam
 * is never worse; bounds never exceed the value of any completion.
 */
#include "sailor_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define SS_MAX_STAGES 255
#define SS_MAX_POOLS 64

typedef struct {
  double sum;      /* stage times of the closed stages 0 .. i-1 */
  double maxt;     /* slowest closed stage */
  double c_open;   /* compute time of stage i (its forward transfer is not known yet) */
  double xb_open;  /* its backward transfer to stage i-1 */
  double msync, mupd, dol, comm;
  double lb_key, lb_T, lb_C;
  /* with split stages: the same four for the pipelines through the second pools */
  double sum_b, maxt_b, c_open_b, xb_open_b;
  uint16_t cnt[SS_MAX_POOLS]; /* stages placed on each pool (with split stages: halves of stages;
                                 with a TP degree per stage: GPUs of one replica) */
  uint8_t pool, runs;
  uint8_t pool_b;
  uint8_t tpi;                /* with a TP degree per stage: the open stage's */
  uint8_t path[SS_MAX_STAGES];
  uint8_t path_b[SS_MAX_STAGES];
  uint8_t path_t[SS_MAX_STAGES];
} ss_state;

typedef struct {
  /* the sub-problem */
  int P, G, Z, ZG, tp, tp_idx, mb_idx, dp_idx, pp_idx, partition;
  int64_t D, Nb;
  double p2p;
  /* per stage and type / zone / pool */
  double c[SS_MAX_STAGES][16], upd[SS_MAX_STAGES][16], dol[SS_MAX_STAGES][16];
  double sync[SS_MAX_STAGES][16];
  uint8_t ok[SS_MAX_STAGES][SS_MAX_POOLS];
  int cap_cnt[SS_MAX_POOLS];      /* stages a pool can host: avail / (tp * D) */
  int cap_half[SS_MAX_POOLS];     /* halves of stages: 2 avail / (tp * D) */
  double xfer[16][16], comm[16][16];
  double comm_half[16][16];       /* traffic cost of one kind of pipeline (half of the replicas) */
  double ring_bytes[SS_MAX_STAGES]; /* bytes a ring all-reduce of the stage moves over every link */
  double bw[16][16], ring_price[16][16], price[16];
  /* with a TP degree per stage: per stage, type / zone and TP index */
  int n_tp, tpv[8];
  double c3[SS_MAX_STAGES][16][8], upd3[SS_MAX_STAGES][16][8], sync3[SS_MAX_STAGES][16][8];
  double dol3[16][8];
  uint8_t ok3[SS_MAX_STAGES][16][8]; /* the stage fits the type's memory and node at this degree */
  int cap_gpus[SS_MAX_POOLS];        /* GPUs one replica can take from a pool: avail / D */
  /* ... and two pools per stage as well */
  double ring3[SS_MAX_STAGES][8];    /* bytes the stage's ring all-reduce moves over every link, per TP index */
  int cap_half_gpus[SS_MAX_POOLS];   /* GPUs of one replica, counted once per half of a stage: 2 avail / D */
  /* cheapest admissible choice of the stages behind stage i */
  double Ssum[SS_MAX_STAGES], Smax[SS_MAX_STAGES], Ssync[SS_MAX_STAGES], Supd[SS_MAX_STAGES],
      Sdol[SS_MAX_STAGES];
} ss_sub;

static double time_sum(const so_problem *p, const double *tab, int g, int im, int it, int first, int n) {
  if (p->uniform_layers) return (double)n * tab[(((size_t)g * p->n_mb + im) * p->n_tp + it)];
  const double *row = tab + (((size_t)g * p->n_mb + im) * p->n_tp + it) * p->n_layers;
  double s = 0.0;
  for (int l = first; l < first + n; ++l) s += row[l];
  return s;
}

static double upd_sum(const so_problem *p, int g, int it, int first, int n) {
  if (p->uniform_layers) return (double)n * p->t_upd[(size_t)g * p->n_tp + it];
  const double *row = p->t_upd + ((size_t)g * p->n_tp + it) * p->n_layers;
  double s = 0.0;
  for (int l = first; l < first + n; ++l) s += row[l];
  return s;
}

static const int32_t *layers_of(const so_problem *p, int pp_idx, int partition) {
  size_t row = 0;
  for (int ip = 0; ip < pp_idx; ++ip) row += (size_t)p->n_partitions[ip] * p->pp_values[ip];
  return p->partition_layers + row + (size_t)partition * p->pp_values[pp_idx];
}

/* What lies behind stage i at the least: every later stage at its cheapest admissible choice
 * (sums for the pipeline time and the rent, maxima for the straggler, all-reduce and update). */
static void behind_every_stage(ss_sub *s, const double *cmin, const double *smin, const double *umin,
                               const double *dmin) {
  const int P = s->P;
  s->Ssum[P - 1] = s->Smax[P - 1] = s->Ssync[P - 1] = s->Supd[P - 1] = s->Sdol[P - 1] = 0.0;
  for (int i = P - 2; i >= 0; --i) {
    s->Ssum[i] = s->Ssum[i + 1] + cmin[i + 1];
    s->Smax[i] = fmax(s->Smax[i + 1], cmin[i + 1]);
    s->Ssync[i] = fmax(s->Ssync[i + 1], smin[i + 1]);
    s->Supd[i] = fmax(s->Supd[i + 1], umin[i + 1]);
    s->Sdol[i] = s->Sdol[i + 1] + dmin[i + 1];
  }
}

/* Tables of one sub-problem.  Returns 0 when it cannot hold a valid plan at all (the batch
 * does not divide, or some stage fits no pool). */
static int sub_setup(const so_problem *p, ss_sub *s, int pp_idx, int partition, int tp_idx, int dp_idx,
                     int mb_idx) {
  s->P = p->pp_values[pp_idx];
  s->G = p->n_types;
  s->Z = p->n_zones;
  s->ZG = s->G * s->Z;
  s->pp_idx = pp_idx; s->partition = partition; s->tp_idx = tp_idx; s->dp_idx = dp_idx; s->mb_idx = mb_idx;
  s->tp = p->tp_values[tp_idx];
  s->D = p->dp_values[dp_idx];
  const int64_t mb = p->mb_values[mb_idx];
  if (p->global_batch % (s->D * mb) != 0) return 0;
  s->Nb = p->global_batch / (s->D * mb);
  s->p2p = (double)p->p2p_bytes[mb_idx];
  const int P = s->P, G = s->G, Z = s->Z;
  const int32_t *nl = layers_of(p, pp_idx, partition);
  for (int g = 0; g < s->G; ++g) s->price[g] = p->price_per_hour[g];
  for (int a = 0; a < s->ZG; ++a) {
    s->cap_cnt[a] = (int)((int64_t)p->avail[a] / ((int64_t)s->tp * s->D));
    s->cap_half[a] = (int)(2 * (int64_t)p->avail[a] / ((int64_t)s->tp * s->D));
  }
  for (int z = 0; z < Z; ++z)
    for (int y = 0; y < Z; ++y) {
      s->xfer[z][y] = s->p2p / p->bandwidth[(size_t)z * Z + y];
      s->comm[z][y] = 0.0;
      s->comm_half[z][y] = 0.0;
      s->ring_price[z][y] = 0.0;
      s->bw[z][y] = p->bandwidth[(size_t)z * Z + y];
      if (p->egress_per_byte && z != y) {
        const double both = p->egress_per_byte[(size_t)z * Z + y] + p->egress_per_byte[(size_t)y * Z + z];
        s->comm[z][y] = (double)s->Nb * (double)s->D * s->p2p * both;
        s->comm_half[z][y] = (double)s->Nb * (0.5 * (double)s->D) * s->p2p * both;
        s->ring_price[z][y] = both;
      }
    }
  int first = 0;
  for (int i = 0; i < P; ++i) {
    uint64_t params = 0;
    for (int l = first; l < first + nl[i]; ++l) params += p->layer_params[l];
    if (i == 0) params += p->embed_params;
    if (i == P - 1) params += p->head_params;
    const uint64_t shard = (params + (uint64_t)s->tp - 1) / (uint64_t)s->tp;
    const int64_t alive = (P - i) < s->Nb ? (P - i) : s->Nb;
    const uint64_t bytes = shard * (uint64_t)p->bytes_per_param +
                           (uint64_t)alive * (uint64_t)nl[i] *
                               p->act_store_bytes[(size_t)mb_idx * p->n_tp + tp_idx];
    for (int g = 0; g < G; ++g) {
      const double f = time_sum(p, p->t_fwd, g, mb_idx, tp_idx, first, nl[i]);
      const double b = time_sum(p, p->t_bwd, g, mb_idx, tp_idx, first, nl[i]);
      s->c[i][g] = f + b;
      s->upd[i][g] = upd_sum(p, g, tp_idx, first, nl[i]);
      s->dol[i][g] = (double)(s->D * s->tp) * p->price_per_hour[g];
      const int fits = bytes + p->mem_reserved[g] <= p->mem_capacity[g] && s->tp <= p->gpus_per_node[g];
      for (int z = 0; z < Z; ++z) s->ok[i][z * G + g] = (uint8_t)fits;
    }
    s->ring_bytes[i] = 0.0;
    if (s->D > 1)
      s->ring_bytes[i] = 2.0 * (double)(s->D - 1) / (double)s->D * ((double)shard * (double)p->grad_bytes_per_param);
    for (int z = 0; z < Z; ++z) {
      double sync = 0.0;
      if (s->D > 1) {
        const double grad = (double)shard * (double)p->grad_bytes_per_param;
        sync = 2.0 * (double)(s->D - 1) / (double)s->D * grad / p->bandwidth[(size_t)z * Z + z];
      }
      s->sync[i][z] = sync;
    }
    first += nl[i];
  }
  /* the cheapest admissible choice of every stage, then what lies behind stage i */
  double cmin[SS_MAX_STAGES], smin[SS_MAX_STAGES], umin[SS_MAX_STAGES], dmin[SS_MAX_STAGES];
  for (int i = 0; i < P; ++i) {
    int any = 0;
    cmin[i] = smin[i] = umin[i] = dmin[i] = INFINITY;
    for (int a = 0; a < s->ZG; ++a) {
      if (!s->ok[i][a]) continue;
      any = 1;
      const int g = a % G, z = a / G;
      if (s->c[i][g] < cmin[i]) cmin[i] = s->c[i][g];
      if (s->sync[i][z] < smin[i]) smin[i] = s->sync[i][z];
      if (s->upd[i][g] < umin[i]) umin[i] = s->upd[i][g];
      if (s->dol[i][g] < dmin[i]) dmin[i] = s->dol[i][g];
    }
    if (!any) return 0;
  }
  behind_every_stage(s, cmin, smin, umin, dmin);
  return 1;
}

/* Lower bounds of the state's completions; the plan's own values when stage P - 1 is placed. */
static void bounds(const ss_sub *s, int i, ss_state *st, int objective) {
  const double t_open = st->c_open + st->xb_open;
  const double tsum = (st->sum + t_open) + s->Ssum[i];
  const double tmax = fmax(fmax(st->maxt, t_open), s->Smax[i]);
  st->lb_T = ((tsum + (double)(s->Nb - 1) * tmax) + fmax(st->msync, s->Ssync[i])) + fmax(st->mupd, s->Supd[i]);
  st->lb_C = (st->dol + s->Sdol[i]) / 3600.0 * st->lb_T + st->comm;
  st->lb_key = objective == SO_MAX_THROUGHPUT ? st->lb_T : st->lb_C;
}

/* stage 0 on pool a */
static int first_state(const ss_sub *s, int a, int objective, ss_state *st) {
  if (!s->ok[0][a] || s->cap_cnt[a] < 1) return 0;
  const int g = a % s->G, z = a / s->G;
  memset(st, 0, sizeof *st);
  st->c_open = s->c[0][g];
  st->msync = s->sync[0][z];
  st->mupd = s->upd[0][g];
  st->dol = s->dol[0][g];
  st->cnt[a] = 1;
  st->pool = (uint8_t)a;
  st->runs = 1;
  st->path[0] = (uint8_t)a;
  bounds(s, 0, st, objective);
  return 1;
}

/* stage i + 1 on pool a behind the state par (stages 0 .. i placed) */
static int extend(const ss_sub *s, int i, const ss_state *par, int a, int max_runs, int objective,
                  ss_state *st) {
  if (!s->ok[i + 1][a] || par->cnt[a] + 1 > s->cap_cnt[a]) return 0;
  const int runs = par->runs + (a != par->pool ? 1 : 0);
  if (max_runs > 0 && runs > max_runs) return 0;
  const int g = a % s->G, z = a / s->G, zp = par->pool / s->G;
  *st = *par;
  const double t_closed = par->c_open + (s->xfer[zp][z] + par->xb_open); /* forward, then backward */
  st->sum = par->sum + t_closed;
  st->maxt = fmax(par->maxt, t_closed);
  st->c_open = s->c[i + 1][g];
  st->xb_open = s->xfer[z][zp];
  st->msync = fmax(par->msync, s->sync[i + 1][z]);
  st->mupd = fmax(par->mupd, s->upd[i + 1][g]);
  st->dol = par->dol + s->dol[i + 1][g];
  if (zp != z) st->comm = par->comm + s->comm[zp][z];
  st->cnt[a] = (uint16_t)(par->cnt[a] + 1);
  st->pool = (uint8_t)a;
  st->runs = (uint8_t)runs;
  st->path[i + 1] = (uint8_t)a;
  bounds(s, i + 1, st, objective);
  return 1;
}

/* dropped: the bound already violates the constraint, or cannot beat the incumbent */
static int pruned(const ss_state *st, int objective, int has_bound, double bound, int has_inc, double inc) {
  if (has_bound) {
    if (objective == SO_MAX_THROUGHPUT) { if (st->lb_C > bound) return 1; }
    else if (1.0 / st->lb_T < bound) return 1;
  }
  return has_inc && st->lb_key > inc;
}

/* ---- stages that may split their replicas over two pools (a, b), half on each ------------ */

/* bounds with two kinds of pipeline: the slower one counts (Sec. 4.3) */
static void bounds2(const ss_sub *s, int i, ss_state *st, int objective) {
  const double ta = st->c_open + st->xb_open, tb = st->c_open_b + st->xb_open_b;
  const double pa = ((st->sum + ta) + s->Ssum[i]) + (double)(s->Nb - 1) * fmax(fmax(st->maxt, ta), s->Smax[i]);
  const double pb = ((st->sum_b + tb) + s->Ssum[i]) + (double)(s->Nb - 1) * fmax(fmax(st->maxt_b, tb), s->Smax[i]);
  st->lb_T = (fmax(pa, pb) + fmax(st->msync, s->Ssync[i])) + fmax(st->mupd, s->Supd[i]);
  st->lb_C = (st->dol + s->Sdol[i]) / 3600.0 * st->lb_T + st->comm;
  st->lb_key = objective == SO_MAX_THROUGHPUT ? st->lb_T : st->lb_C;
}

/* what stage j costs on the pools (a, b) by itself: all-reduce over the slowest link of the
 * ring, the slower update, the mean rent, the ring's traffic between the zones */
static void stage_terms2(const ss_sub *s, int j, int a, int b, double *sync, double *upd, double *dol,
                         double *ring_cost) {
  const int ga = a % s->G, za = a / s->G, gb = b % s->G, zb = b / s->G;
  double link = s->bw[za][za];
  if (zb != za) link = fmin(fmin(link, s->bw[zb][zb]), fmin(s->bw[za][zb], s->bw[zb][za]));
  *sync = s->ring_bytes[j] / link;
  *upd = fmax(s->upd[j][ga], s->upd[j][gb]);
  *dol = (double)(s->D * s->tp) * (0.5 * (s->price[ga] + s->price[gb]));
  *ring_cost = zb != za ? s->ring_bytes[j] * s->ring_price[za][zb] : 0.0;
}

static int admissible2(const ss_sub *s, int j, const uint16_t *cnt, int a, int b) {
  if (!s->ok[j][a] || !s->ok[j][b]) return 0;
  if (a == b) return cnt[a] + 2 <= s->cap_half[a];
  if (s->D % 2 != 0) return 0; /* D replicas cannot be halved */
  return cnt[a] + 1 <= s->cap_half[a] && cnt[b] + 1 <= s->cap_half[b];
}

static int first_state2(const ss_sub *s, int a, int b, int objective, ss_state *st) {
  memset(st, 0, sizeof *st);
  if (!admissible2(s, 0, st->cnt, a, b)) return 0;
  double sync, upd, dol, ring;
  stage_terms2(s, 0, a, b, &sync, &upd, &dol, &ring);
  st->c_open = s->c[0][a % s->G];
  st->c_open_b = s->c[0][b % s->G];
  st->msync = sync; st->mupd = upd; st->dol = dol; st->comm = ring;
  st->cnt[a] += 1; st->cnt[b] += 1;
  st->pool = (uint8_t)a; st->pool_b = (uint8_t)b;
  st->runs = 1;
  st->path[0] = (uint8_t)a; st->path_b[0] = (uint8_t)b;
  bounds2(s, 0, st, objective);
  return 1;
}

static int extend2(const ss_sub *s, int i, const ss_state *par, int a, int b, int max_runs, int objective,
                   ss_state *st) {
  if (!admissible2(s, i + 1, par->cnt, a, b)) return 0;
  const int runs = par->runs + ((a != par->pool || b != par->pool_b) ? 1 : 0);
  if (max_runs > 0 && runs > max_runs) return 0;
  const int za = a / s->G, zb = b / s->G, pza = par->pool / s->G, pzb = par->pool_b / s->G;
  *st = *par;
  const double ta = par->c_open + (s->xfer[pza][za] + par->xb_open);
  const double tb = par->c_open_b + (s->xfer[pzb][zb] + par->xb_open_b);
  st->sum = par->sum + ta;
  st->maxt = fmax(par->maxt, ta);
  st->sum_b = par->sum_b + tb;
  st->maxt_b = fmax(par->maxt_b, tb);
  st->c_open = s->c[i + 1][a % s->G];
  st->c_open_b = s->c[i + 1][b % s->G];
  st->xb_open = s->xfer[za][pza];
  st->xb_open_b = s->xfer[zb][pzb];
  double sync, upd, dol, ring;
  stage_terms2(s, i + 1, a, b, &sync, &upd, &dol, &ring);
  st->msync = fmax(par->msync, sync);
  st->mupd = fmax(par->mupd, upd);
  st->dol = par->dol + dol;
  double comm = par->comm;
  if (pza != za) comm += s->comm_half[pza][za];
  if (pzb != zb) comm += s->comm_half[pzb][zb];
  st->comm = comm + ring;
  st->cnt[a] += 1; st->cnt[b] += 1;
  st->pool = (uint8_t)a; st->pool_b = (uint8_t)b;
  st->runs = (uint8_t)runs;
  st->path[i + 1] = (uint8_t)a; st->path_b[i + 1] = (uint8_t)b;
  bounds2(s, i + 1, st, objective);
  return 1;
}

/* ---- stages that choose their TP degree too: a choice is (pool a, TP index t) -------------- */

/* Tables of one sub-problem (pp, layer split, D, microbatch size).  Returns 0 when it cannot
 * hold a valid plan at all. */
static int sub_setup_tp(const so_problem *p, ss_sub *s, int pp_idx, int partition, int dp_idx, int mb_idx) {
  s->P = p->pp_values[pp_idx];
  s->G = p->n_types;
  s->Z = p->n_zones;
  s->ZG = s->G * s->Z;
  s->pp_idx = pp_idx; s->partition = partition; s->tp_idx = -1; s->dp_idx = dp_idx; s->mb_idx = mb_idx;
  s->tp = 0;
  s->n_tp = p->n_tp;
  if (p->n_tp > 8) return 0;
  for (int t = 0; t < p->n_tp; ++t) s->tpv[t] = p->tp_values[t];
  s->D = p->dp_values[dp_idx];
  const int64_t mb = p->mb_values[mb_idx];
  if (p->global_batch % (s->D * mb) != 0) return 0;
  s->Nb = p->global_batch / (s->D * mb);
  s->p2p = (double)p->p2p_bytes[mb_idx];
  const int P = s->P, G = s->G, Z = s->Z;
  const int32_t *nl = layers_of(p, pp_idx, partition);
  for (int a = 0; a < s->ZG; ++a) {
    s->cap_gpus[a] = (int)((int64_t)p->avail[a] / s->D);
    s->cap_half_gpus[a] = (int)(2 * (int64_t)p->avail[a] / s->D);
  }
  for (int g = 0; g < G; ++g) s->price[g] = p->price_per_hour[g];
  for (int z = 0; z < Z; ++z)
    for (int y = 0; y < Z; ++y) {
      s->xfer[z][y] = s->p2p / p->bandwidth[(size_t)z * Z + y];
      s->bw[z][y] = p->bandwidth[(size_t)z * Z + y];
      s->comm[z][y] = s->comm_half[z][y] = s->ring_price[z][y] = 0.0;
      if (p->egress_per_byte && z != y) {
        const double both = p->egress_per_byte[(size_t)z * Z + y] + p->egress_per_byte[(size_t)y * Z + z];
        s->comm[z][y] = (double)s->Nb * (double)s->D * s->p2p * both;
        s->comm_half[z][y] = (double)s->Nb * (0.5 * (double)s->D) * s->p2p * both;
        s->ring_price[z][y] = both;
      }
    }
  for (int g = 0; g < G; ++g)
    for (int t = 0; t < s->n_tp; ++t) s->dol3[g][t] = (double)(s->D * s->tpv[t]) * p->price_per_hour[g];
  double cmin[SS_MAX_STAGES], smin[SS_MAX_STAGES], umin[SS_MAX_STAGES], dmin[SS_MAX_STAGES];
  int first = 0;
  for (int i = 0; i < P; ++i) {
    uint64_t params = 0;
    for (int l = first; l < first + nl[i]; ++l) params += p->layer_params[l];
    if (i == 0) params += p->embed_params;
    if (i + 1 == P) params += p->head_params;
    const int64_t alive = (P - i) < s->Nb ? (P - i) : s->Nb;
    int any = 0;
    cmin[i] = smin[i] = umin[i] = dmin[i] = INFINITY;
    for (int t = 0; t < s->n_tp; ++t) {
      const uint64_t shard = (params + (uint64_t)s->tpv[t] - 1) / (uint64_t)s->tpv[t];
      const uint64_t bytes = shard * (uint64_t)p->bytes_per_param +
                             (uint64_t)alive * (uint64_t)nl[i] * p->act_store_bytes[(size_t)mb_idx * p->n_tp + t];
      s->ring3[i][t] = 0.0;
      if (s->D > 1)
        s->ring3[i][t] = 2.0 * (double)(s->D - 1) / (double)s->D * ((double)shard * (double)p->grad_bytes_per_param);
      int fits_some = 0;
      for (int g = 0; g < G; ++g) {
        s->c3[i][g][t] = time_sum(p, p->t_fwd, g, mb_idx, t, first, nl[i]) + time_sum(p, p->t_bwd, g, mb_idx, t, first, nl[i]);
        s->upd3[i][g][t] = upd_sum(p, g, t, first, nl[i]);
        s->ok3[i][g][t] = (uint8_t)(bytes + p->mem_reserved[g] <= p->mem_capacity[g] && s->tpv[t] <= p->gpus_per_node[g]);
        if (!s->ok3[i][g][t]) continue;
        fits_some = 1;
        if (s->c3[i][g][t] < cmin[i]) cmin[i] = s->c3[i][g][t];
        if (s->upd3[i][g][t] < umin[i]) umin[i] = s->upd3[i][g][t];
        if (s->dol3[g][t] < dmin[i]) dmin[i] = s->dol3[g][t];
      }
      for (int z = 0; z < Z; ++z) {
        double sync = 0.0;
        if (s->D > 1) {
          const double grad = (double)shard * (double)p->grad_bytes_per_param;
          sync = 2.0 * (double)(s->D - 1) / (double)s->D * grad / p->bandwidth[(size_t)z * Z + z];
        }
        s->sync3[i][z][t] = sync;
        if (fits_some && sync < smin[i]) smin[i] = sync;
      }
      any |= fits_some;
    }
    if (!any) return 0;
    first += nl[i];
  }
  behind_every_stage(s, cmin, smin, umin, dmin);
  return 1;
}

/* stage 0 on pool a at TP index t */
static int first_state_tp(const ss_sub *s, int a, int t, int objective, ss_state *st) {
  const int g = a % s->G, z = a / s->G;
  if (!s->ok3[0][g][t] || s->tpv[t] > s->cap_gpus[a]) return 0;
  memset(st, 0, sizeof *st);
  st->c_open = s->c3[0][g][t];
  st->msync = s->sync3[0][z][t];
  st->mupd = s->upd3[0][g][t];
  st->dol = s->dol3[g][t];
  st->cnt[a] = (uint16_t)s->tpv[t];
  st->pool = (uint8_t)a;
  st->tpi = (uint8_t)t;
  st->runs = 1;
  st->path[0] = (uint8_t)a;
  st->path_t[0] = (uint8_t)t;
  bounds(s, 0, st, objective);
  return 1;
}

/* stage i + 1 on pool a at TP index t behind the state par; a run ends where the pool or the
 * degree changes */
static int extend_tp(const ss_sub *s, int i, const ss_state *par, int a, int t, int max_runs, int objective,
                     ss_state *st) {
  const int g = a % s->G, zone = a / s->G, before = par->pool / s->G;
  if (!s->ok3[i + 1][g][t] || par->cnt[a] + s->tpv[t] > s->cap_gpus[a]) return 0;
  const int runs = par->runs + ((a != par->pool || t != par->tpi) ? 1 : 0);
  if (max_runs > 0 && runs > max_runs) return 0;
  *st = *par;
  const double t_closed = par->c_open + (s->xfer[before][zone] + par->xb_open); /* forward, then backward */
  st->sum = par->sum + t_closed;
  st->maxt = fmax(par->maxt, t_closed);
  st->c_open = s->c3[i + 1][g][t];
  st->xb_open = s->xfer[zone][before];
  st->msync = fmax(par->msync, s->sync3[i + 1][zone][t]);
  st->mupd = fmax(par->mupd, s->upd3[i + 1][g][t]);
  st->dol = par->dol + s->dol3[g][t];
  if (before != zone) st->comm = par->comm + s->comm[before][zone];
  st->cnt[a] = (uint16_t)(par->cnt[a] + s->tpv[t]);
  st->pool = (uint8_t)a;
  st->tpi = (uint8_t)t;
  st->runs = (uint8_t)runs;
  st->path[i + 1] = (uint8_t)a;
  st->path_t[i + 1] = (uint8_t)t;
  bounds(s, i + 1, st, objective);
  return 1;
}

/* ---- two pools and a TP degree per stage: a choice is (pool a, pool b, TP index t); both halves
 * of the stage run at the degree, a pool's quota counts the GPUs of one replica once per half ---- */

static int admissible2_tp(const ss_sub *s, int j, const uint16_t *cnt, int a, int b, int t) {
  if (!s->ok3[j][a % s->G][t] || !s->ok3[j][b % s->G][t]) return 0;
  const int width = s->tpv[t];
  if (a == b) return cnt[a] + 2 * width <= s->cap_half_gpus[a];
  if (s->D % 2 != 0) return 0; /* D replicas cannot be halved */
  return cnt[a] + width <= s->cap_half_gpus[a] && cnt[b] + width <= s->cap_half_gpus[b];
}

/* what stage j costs on the pools (a, b) at TP index t by itself */
static void stage_terms2_tp(const ss_sub *s, int j, int a, int b, int t, double *sync, double *upd,
                            double *dol, double *ring_cost) {
  const int ga = a % s->G, za = a / s->G, gb = b % s->G, zb = b / s->G;
  double link = s->bw[za][za];
  if (zb != za) link = fmin(fmin(link, s->bw[zb][zb]), fmin(s->bw[za][zb], s->bw[zb][za]));
  *sync = s->ring3[j][t] / link;
  *upd = fmax(s->upd3[j][ga][t], s->upd3[j][gb][t]);
  *dol = (double)(s->D * s->tpv[t]) * (0.5 * (s->price[ga] + s->price[gb]));
  *ring_cost = zb != za ? s->ring3[j][t] * s->ring_price[za][zb] : 0.0;
}

static int first_state2_tp(const ss_sub *s, int a, int b, int t, int objective, ss_state *st) {
  memset(st, 0, sizeof *st);
  if (!admissible2_tp(s, 0, st->cnt, a, b, t)) return 0;
  double sync, upd, dol, ring;
  stage_terms2_tp(s, 0, a, b, t, &sync, &upd, &dol, &ring);
  st->c_open = s->c3[0][a % s->G][t];
  st->c_open_b = s->c3[0][b % s->G][t];
  st->msync = sync; st->mupd = upd; st->dol = dol; st->comm = ring;
  st->cnt[a] = (uint16_t)(st->cnt[a] + s->tpv[t]);
  st->cnt[b] = (uint16_t)(st->cnt[b] + s->tpv[t]);
  st->pool = (uint8_t)a; st->pool_b = (uint8_t)b; st->tpi = (uint8_t)t;
  st->runs = 1;
  st->path[0] = (uint8_t)a; st->path_b[0] = (uint8_t)b; st->path_t[0] = (uint8_t)t;
  bounds2(s, 0, st, objective);
  return 1;
}

/* stage i + 1 behind the state par; a run ends where a pool or the degree changes */
static int extend2_tp(const ss_sub *s, int i, const ss_state *par, int a, int b, int t, int max_runs,
                      int objective, ss_state *st) {
  if (!admissible2_tp(s, i + 1, par->cnt, a, b, t)) return 0;
  const int runs = par->runs + ((a != par->pool || b != par->pool_b || t != par->tpi) ? 1 : 0);
  if (max_runs > 0 && runs > max_runs) return 0;
  const int za = a / s->G, zb = b / s->G, pza = par->pool / s->G, pzb = par->pool_b / s->G;
  *st = *par;
  const double ta = par->c_open + (s->xfer[pza][za] + par->xb_open);   /* forward, then backward */
  const double tb = par->c_open_b + (s->xfer[pzb][zb] + par->xb_open_b);
  st->sum = par->sum + ta;
  st->maxt = fmax(par->maxt, ta);
  st->sum_b = par->sum_b + tb;
  st->maxt_b = fmax(par->maxt_b, tb);
  st->c_open = s->c3[i + 1][a % s->G][t];
  st->c_open_b = s->c3[i + 1][b % s->G][t];
  st->xb_open = s->xfer[za][pza];
  st->xb_open_b = s->xfer[zb][pzb];
  double sync, upd, dol, ring;
  stage_terms2_tp(s, i + 1, a, b, t, &sync, &upd, &dol, &ring);
  st->msync = fmax(par->msync, sync);
  st->mupd = fmax(par->mupd, upd);
  st->dol = par->dol + dol;
  double comm = par->comm;
  if (pza != za) comm += s->comm_half[pza][za];
  if (pzb != zb) comm += s->comm_half[pzb][zb];
  st->comm = comm + ring;
  st->cnt[a] = (uint16_t)(st->cnt[a] + s->tpv[t]);
  st->cnt[b] = (uint16_t)(st->cnt[b] + s->tpv[t]);
  st->pool = (uint8_t)a; st->pool_b = (uint8_t)b; st->tpi = (uint8_t)t;
  st->runs = (uint8_t)runs;
  st->path[i + 1] = (uint8_t)a; st->path_b[i + 1] = (uint8_t)b; st->path_t[i + 1] = (uint8_t)t;
  bounds2(s, i + 1, st, objective);
  return 1;
}

typedef struct { double key; uint32_t id; uint32_t pos; } ss_order; /* id: generation order; pos: where it is stored */

static int by_key_then_id(const void *x, const void *y) {
  const ss_order *a = (const ss_order *)x, *b = (const ss_order *)y;
  if (a->key < b->key) return -1;
  if (a->key > b->key) return 1;
  return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

static void take(so_search_result *out, const ss_sub *s, const ss_state *st) {
  out->found = 1;
  out->pp_idx = s->pp_idx; out->partition = s->partition; out->tp_idx = s->tp_idx;
  out->dp_idx = s->dp_idx; out->mb_idx = s->mb_idx; out->pp = s->P;
  out->key = st->lb_key; out->iter_time = st->lb_T; out->cost = st->lb_C;
  for (int i = 0; i < s->P; ++i) {
    out->pools[i] = st->path[i];
    out->pools_b[i] = st->path[i];
    out->tps[i] = s->tp_idx;
  }
}

static void take2(so_search_result *out, const ss_sub *s, const ss_state *st) {
  take(out, s, st);
  for (int i = 0; i < s->P; ++i) out->pools_b[i] = st->path_b[i];
}

static void take_tp(so_search_result *out, const ss_sub *s, const ss_state *st) {
  take(out, s, st);
  out->tp_idx = st->path_t[0];
  for (int i = 0; i < s->P; ++i) out->tps[i] = st->path_t[i];
}

static void take2_tp(so_search_result *out, const ss_sub *s, const ss_state *st) {
  take_tp(out, s, st);
  for (int i = 0; i < s->P; ++i) out->pools_b[i] = st->path_b[i];
}

int so_search_beam(const so_ctx *c, int objective, int has_bound, double bound,
                   const so_search_opts *opt, so_search_result *out) {
  const so_problem *p = so_problem_of(c);
  memset(out, 0, sizeof *out);
  if (p->mixed_types || p->n_bw_coef > 0 || !opt || opt->beam_width < 1) return -1;
  if (p->n_types > 16 || p->n_zones > 16 || p->n_types * p->n_zones > SS_MAX_POOLS) return -1;
  const int W = opt->beam_width, ZG = p->n_types * p->n_zones;
  const int split = opt->allow_split ? 1 : 0, stp = opt->stage_tp ? 1 : 0, NT = p->n_tp;
  const int both = split && stp;
  /* choices per stage: a pool; a pair (a, b) = a * ZG + b; a pool and a TP index (a, t) = a * NT + t;
   * a pair and a TP index (a, b, t) = (a * ZG + b) * NT + t */
  const int NCH = both ? ZG * ZG * NT : split ? ZG * ZG : (stp ? ZG * NT : ZG);
  /* room for a frontier of `cap` placements and its cap * NCH extensions; grows with the
   * frontier (a beam width far beyond what a problem can fill costs nothing) */
  size_t cap = (size_t)(W < 1024 ? W : 1024);
  ss_sub *s = (ss_sub *)malloc(sizeof(ss_sub));
  ss_state *cur = (ss_state *)malloc(sizeof(ss_state) * cap);
  ss_state *all = (ss_state *)malloc(sizeof(ss_state) * cap * (size_t)NCH);
  ss_order *ord = (ss_order *)malloc(sizeof(ss_order) * cap * (size_t)NCH);
  if (!s || !cur || !all || !ord) { free(s); free(cur); free(all); free(ord); return -1; }
  for (int ip = 0; ip < p->n_pp; ++ip) {
    if (p->pp_values[ip] > SS_MAX_STAGES) continue;
    for (int q = 0; q < p->n_partitions[ip]; ++q)
      for (int it = 0; it < (stp ? 1 : p->n_tp); ++it)
        for (int id = 0; id < p->n_dp; ++id)
          for (int im = 0; im < p->n_mb; ++im) {
            if (!(stp ? sub_setup_tp(p, s, ip, q, id, im) : sub_setup(p, s, ip, q, it, id, im))) continue;
            /* level 0, then one level per further stage */
            int n = 0, n_all = 0;
            for (int a = 0; a < NCH; ++a)
              if (both    ? first_state2_tp(s, a / NT / ZG, a / NT % ZG, a % NT, objective, &all[n_all])
                  : split ? first_state2(s, a / ZG, a % ZG, objective, &all[n_all])
                  : stp ? first_state_tp(s, a / NT, a % NT, objective, &all[n_all])
                        : first_state(s, a, objective, &all[n_all])) {
                out->expanded += 1;
                if (!pruned(&all[n_all], objective, has_bound, bound, opt->has_incumbent, opt->incumbent)) {
                  ord[n_all].key = all[n_all].lb_key;
                  ord[n_all].id = (uint32_t)a;
                  ord[n_all].pos = (uint32_t)n_all;
                  n_all += 1;
                }
              }
            for (int i = 0;; ++i) { /* `all` holds the surviving placements of stages 0 .. i */
              if (i == s->P - 1) {  /* complete plans: the smallest (key, id) */
                int bi = -1;
                for (int k = 0; k < n_all; ++k)
                  if (bi < 0 || by_key_then_id(&ord[k], &ord[bi]) < 0) bi = k;
                if (bi >= 0 && (!out->found || all[bi].lb_key < out->key)) {
                  if (both) take2_tp(out, s, &all[bi]);
                  else if (split) take2(out, s, &all[bi]);
                  else if (stp) take_tp(out, s, &all[bi]);
                  else take(out, s, &all[bi]);
                }
                break;
              }
              const size_t keep = (size_t)(n_all > W ? W : n_all);
              if (keep > cap) { /* (the kept placements are copied out of `all` first) */
                ss_state *c2 = (ss_state *)realloc(cur, sizeof(ss_state) * keep);
                if (!c2) { free(s); free(cur); free(all); free(ord); return -1; }
                cur = c2;
              }
              if (n_all > W) { /* keep the W smallest bounds, in that order */
                qsort(ord, (size_t)n_all, sizeof(ss_order), by_key_then_id);
                out->truncated = 1;
                for (int k = 0; k < W; ++k) cur[k] = all[ord[k].pos];
                n = W;
              } else { /* all of them, in the order they were generated */
                for (int k = 0; k < n_all; ++k) cur[k] = all[k];
                n = n_all;
              }
              if (keep > cap) {
                ss_state *a2 = (ss_state *)realloc(all, sizeof(ss_state) * keep * (size_t)NCH);
                if (a2) all = a2;
                ss_order *o2 = (ss_order *)realloc(ord, sizeof(ss_order) * keep * (size_t)NCH);
                if (o2) ord = o2;
                if (!a2 || !o2) { free(s); free(cur); free(all); free(ord); return -1; }
                cap = keep;
              }
              /* expand: candidate id = rank of the parent * NCH + choice */
              n_all = 0;
              for (int r = 0; r < n; ++r)
                for (int a = 0; a < NCH; ++a) {
                  ss_state *st = &all[n_all];
                  if (!(both    ? extend2_tp(s, i, &cur[r], a / NT / ZG, a / NT % ZG, a % NT, opt->max_runs, objective, st)
                        : split ? extend2(s, i, &cur[r], a / ZG, a % ZG, opt->max_runs, objective, st)
                        : stp ? extend_tp(s, i, &cur[r], a / NT, a % NT, opt->max_runs, objective, st)
                              : extend(s, i, &cur[r], a, opt->max_runs, objective, st)))
                    continue;
                  out->expanded += 1;
                  if (pruned(st, objective, has_bound, bound, opt->has_incumbent, opt->incumbent)) continue;
                  ord[n_all].key = st->lb_key;
                  ord[n_all].id = (uint32_t)(r * NCH + a);
                  ord[n_all].pos = (uint32_t)n_all;
                  n_all += 1;
                }
              if (n_all == 0) break;
            }
          }
  }
  free(s); free(cur); free(all); free(ord);
  return 0;
}

/* ---- the definition: every placement of every sub-problem through the plain simulator ---- */

static void place(const so_ctx *c, const so_problem *p, int ip, int q, int it, int id, int im,
                  int i, int runs, int max_runs, int32_t *pools, int32_t *pools_b, int split,
                  int objective, int has_bound, double bound, so_search_result *out) {
  const int P = p->pp_values[ip], ZG = p->n_types * p->n_zones;
  if (i == P) {
    so_eval e;
    out->expanded += 1;
    if ((split ? so_eval_split_assignment(c, ip, q, id, im, it, pools, pools_b, objective, has_bound, bound, &e)
               : so_eval_assignment(c, ip, q, id, im, it, pools, objective, has_bound, bound, &e)) != 0)
      return;
    if (e.mask != 0) return;
    const double key = objective == SO_MAX_THROUGHPUT ? e.iter_time : e.cost;
    if (out->found && !(key < out->key)) return; /* the first of equal keys stays */
    out->found = 1;
    out->pp_idx = ip; out->partition = q; out->tp_idx = it; out->dp_idx = id; out->mb_idx = im;
    out->pp = P; out->key = key; out->iter_time = e.iter_time; out->cost = e.cost;
    for (int k = 0; k < P; ++k) { out->pools[k] = pools[k]; out->pools_b[k] = pools_b[k]; }
    return;
  }
  for (int a = 0; a < ZG; ++a)
    for (int b = (split ? 0 : a); b < (split ? ZG : a + 1); ++b) {
      const int r = (i == 0) ? 1 : runs + ((a != pools[i - 1] || b != pools_b[i - 1]) ? 1 : 0);
      if (max_runs > 0 && r > max_runs) continue;
      pools[i] = a;
      pools_b[i] = b;
      place(c, p, ip, q, it, id, im, i + 1, r, max_runs, pools, pools_b, split, objective, has_bound, bound, out);
    }
}

/* the same with a TP index per stage */
static void place_tp(const so_ctx *c, const so_problem *p, int ip, int q, int id, int im, int i, int runs,
                     int max_runs, int32_t *pools, int32_t *tps, int objective, int has_bound, double bound,
                     so_search_result *out) {
  const int P = p->pp_values[ip], ZG = p->n_types * p->n_zones;
  if (i == P) {
    so_eval e;
    out->expanded += 1;
    if (so_eval_assignment_tp(c, ip, q, id, im, tps, pools, objective, has_bound, bound, &e) != 0) return;
    if (e.mask != 0) return;
    const double key = objective == SO_MAX_THROUGHPUT ? e.iter_time : e.cost;
    if (out->found && !(key < out->key)) return; /* the first of equal keys stays */
    out->found = 1;
    out->pp_idx = ip; out->partition = q; out->tp_idx = tps[0]; out->dp_idx = id; out->mb_idx = im;
    out->pp = P; out->key = key; out->iter_time = e.iter_time; out->cost = e.cost;
    for (int k = 0; k < P; ++k) { out->pools[k] = pools[k]; out->pools_b[k] = pools[k]; out->tps[k] = tps[k]; }
    return;
  }
  for (int a = 0; a < ZG; ++a)
    for (int t = 0; t < p->n_tp; ++t) {
      const int r = (i == 0) ? 1 : runs + ((a != pools[i - 1] || t != tps[i - 1]) ? 1 : 0);
      if (max_runs > 0 && r > max_runs) continue;
      pools[i] = a;
      tps[i] = t;
      place_tp(c, p, ip, q, id, im, i + 1, r, max_runs, pools, tps, objective, has_bound, bound, out);
    }
}

/* the same with two pools and a TP index per stage */
static void place2_tp(const so_ctx *c, const so_problem *p, int ip, int q, int id, int im, int i, int runs,
                      int max_runs, int32_t *pools, int32_t *pools_b, int32_t *tps, int objective,
                      int has_bound, double bound, so_search_result *out) {
  const int P = p->pp_values[ip], ZG = p->n_types * p->n_zones;
  if (i == P) {
    so_eval e;
    out->expanded += 1;
    if (so_eval_split_assignment_tp(c, ip, q, id, im, tps, pools, pools_b, objective, has_bound, bound, &e) != 0)
      return;
    if (e.mask != 0) return;
    const double key = objective == SO_MAX_THROUGHPUT ? e.iter_time : e.cost;
    if (out->found && !(key < out->key)) return; /* the first of equal keys stays */
    out->found = 1;
    out->pp_idx = ip; out->partition = q; out->tp_idx = tps[0]; out->dp_idx = id; out->mb_idx = im;
    out->pp = P; out->key = key; out->iter_time = e.iter_time; out->cost = e.cost;
    for (int k = 0; k < P; ++k) { out->pools[k] = pools[k]; out->pools_b[k] = pools_b[k]; out->tps[k] = tps[k]; }
    return;
  }
  for (int a = 0; a < ZG; ++a)
    for (int b = 0; b < ZG; ++b)
      for (int t = 0; t < p->n_tp; ++t) {
        const int r = (i == 0) ? 1
                               : runs + ((a != pools[i - 1] || b != pools_b[i - 1] || t != tps[i - 1]) ? 1 : 0);
        if (max_runs > 0 && r > max_runs) continue;
        pools[i] = a;
        pools_b[i] = b;
        tps[i] = t;
        place2_tp(c, p, ip, q, id, im, i + 1, r, max_runs, pools, pools_b, tps, objective, has_bound, bound, out);
      }
}

int so_search_exhaustive(const so_ctx *c, int objective, int has_bound, double bound, int max_runs,
                         int allow_split, int stage_tp, so_search_result *out) {
  const so_problem *p = so_problem_of(c);
  memset(out, 0, sizeof *out);
  if (p->mixed_types) return -1;
  int32_t pools[SO_SEARCH_MAX_STAGES], pools_b[SO_SEARCH_MAX_STAGES];
  if (allow_split && stage_tp) {
    int32_t tps[SO_SEARCH_MAX_STAGES];
    for (int ip = 0; ip < p->n_pp; ++ip) {
      if (p->pp_values[ip] > SS_MAX_STAGES) continue;
      for (int q = 0; q < p->n_partitions[ip]; ++q)
        for (int id = 0; id < p->n_dp; ++id)
          for (int im = 0; im < p->n_mb; ++im)
            place2_tp(c, p, ip, q, id, im, 0, 0, max_runs, pools, pools_b, tps, objective, has_bound, bound, out);
    }
    return 0;
  }
  if (stage_tp) {
    for (int ip = 0; ip < p->n_pp; ++ip) {
      if (p->pp_values[ip] > SS_MAX_STAGES) continue;
      for (int q = 0; q < p->n_partitions[ip]; ++q)
        for (int id = 0; id < p->n_dp; ++id)
          for (int im = 0; im < p->n_mb; ++im)
            place_tp(c, p, ip, q, id, im, 0, 0, max_runs, pools, pools_b, objective, has_bound, bound, out);
    }
    return 0;
  }
  for (int ip = 0; ip < p->n_pp; ++ip) {
    if (p->pp_values[ip] > SS_MAX_STAGES) continue;
    for (int q = 0; q < p->n_partitions[ip]; ++q)
      for (int it = 0; it < p->n_tp; ++it)
        for (int id = 0; id < p->n_dp; ++id)
          for (int im = 0; im < p->n_mb; ++im)
            place(c, p, ip, q, it, id, im, 0, 0, max_runs, pools, pools_b, allow_split ? 1 : 0, objective,
                  has_bound, bound, out);
  }
  return 0;
}

/* The bound of the first i + 1 stages of a placement (for the tests: it must not exceed the
 * value of the whole placement).  Returns 0, -1 when the prefix itself is not admissible. */
int so_search_prefix_bound(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                           int tp_idx, const int32_t *pools, int n_placed, int objective,
                           double *lb_time, double *lb_cost) {
  const so_problem *p = so_problem_of(c);
  if (p->mixed_types || p->n_bw_coef > 0) return -1;
  ss_sub *s = (ss_sub *)malloc(sizeof(ss_sub));
  ss_state a, b;
  int rc = -1;
  if (s && sub_setup(p, s, pp_idx, partition, tp_idx, dp_idx, mb_idx) && n_placed >= 1 &&
      n_placed <= s->P && first_state(s, pools[0], objective, &a)) {
    rc = 0;
    for (int i = 0; i + 1 < n_placed && rc == 0; ++i) {
      if (!extend(s, i, &a, pools[i + 1], 0, objective, &b)) rc = -1;
      a = b;
    }
    if (rc == 0) { *lb_time = a.lb_T; *lb_cost = a.lb_C; }
  }
  free(s);
  return rc;
}

int so_search_prefix_bound_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                              const int32_t *tp_idx, const int32_t *pools, int n_placed, int objective,
                              double *lb_time, double *lb_cost) {
  const so_problem *p = so_problem_of(c);
  if (p->mixed_types || p->n_bw_coef > 0) return -1;
  ss_sub *s = (ss_sub *)malloc(sizeof(ss_sub));
  ss_state a, b;
  int rc = -1;
  if (s && sub_setup_tp(p, s, pp_idx, partition, dp_idx, mb_idx) && n_placed >= 1 && n_placed <= s->P &&
      tp_idx[0] >= 0 && tp_idx[0] < s->n_tp && first_state_tp(s, pools[0], tp_idx[0], objective, &a)) {
    rc = 0;
    for (int i = 0; i + 1 < n_placed && rc == 0; ++i) {
      if (tp_idx[i + 1] < 0 || tp_idx[i + 1] >= s->n_tp ||
          !extend_tp(s, i, &a, pools[i + 1], tp_idx[i + 1], 0, objective, &b))
        rc = -1;
      a = b;
    }
    if (rc == 0) { *lb_time = a.lb_T; *lb_cost = a.lb_C; }
  }
  free(s);
  return rc;
}

int so_search_prefix_bound_split_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                    const int32_t *tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                                    int n_placed, int objective, double *lb_time, double *lb_cost) {
  const so_problem *p = so_problem_of(c);
  if (p->mixed_types || p->n_bw_coef > 0) return -1;
  ss_sub *s = (ss_sub *)malloc(sizeof(ss_sub));
  ss_state a, b;
  int rc = -1;
  if (s && sub_setup_tp(p, s, pp_idx, partition, dp_idx, mb_idx) && n_placed >= 1 && n_placed <= s->P &&
      tp_idx[0] >= 0 && tp_idx[0] < s->n_tp &&
      first_state2_tp(s, pools_a[0], pools_b[0], tp_idx[0], objective, &a)) {
    rc = 0;
    for (int i = 0; i + 1 < n_placed && rc == 0; ++i) {
      if (tp_idx[i + 1] < 0 || tp_idx[i + 1] >= s->n_tp ||
          !extend2_tp(s, i, &a, pools_a[i + 1], pools_b[i + 1], tp_idx[i + 1], 0, objective, &b))
        rc = -1;
      a = b;
    }
    if (rc == 0) { *lb_time = a.lb_T; *lb_cost = a.lb_C; }
  }
  free(s);
  return rc;
}
