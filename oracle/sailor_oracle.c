/*
 * CPU oracle -- TEST INFRASTRUCTURE ONLY (see sailor_oracle.h).
 *
 * Every candidate is evaluated from scratch, stage by stage, in the natural order of
 * the definitions: no tables of derived values, no blocking, no reordering.
 * Floating point is fp64, byte counts are exact unsigned 64-bit integers.
 */
#include "sailor_oracle.h"

#include <math.h>
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

#define SO_MAX_STAGES 512
#define SO_MAX_POOLS 256
#define SO_TIE_TOL 1e-5

struct so_ctx {
  so_problem p;
  int32_t GX;              /* types a segment can choose: G, or G + G (G - 1) / 2 with pairs */
  int32_t xa[SO_MAX_POOLS], xb[SO_MAX_POOLS]; /* the two real types of an extended type (equal
                                                 for a plain one)                             */
  int32_t ZG;              /* pools: n_zones * GX                                           */
  uint64_t inner;          /* n_mb * n_tp * n_dp * ZG : candidates per (shape, outer pools) */
  uint64_t *block_off;     /* [n_pp][3] : first index of block (pp_idx, s)                  */
  uint64_t *block_size;    /* [n_pp][3]                                                     */
  uint64_t *part_row;      /* [n_pp] : offset of the first partition row of pp_idx          */
  uint64_t n_candidates;
};

/* ---- candidate space (plan tuple of Sec. 4.2, restricted to contiguous segments) ------ */

static uint64_t n_cuts(int P, int s) {
  if (s == 1) return 1;
  if (s == 2) return (uint64_t)(P - 1);
  return (uint64_t)(P - 1) * (uint64_t)(P - 2) / 2;
}

static int segments_allowed(const so_problem *p, int P, int s) {
  if (s > p->max_segments) return 0;
  if (s > P) return 0;
  if (s == 3 && P > p->seg3_max_pp) return 0;
  return 1;
}

so_ctx *so_create(const so_problem *p) {
  if (!p || p->n_layers < 1 || p->n_types < 1 || p->n_zones < 1) return NULL;
  so_ctx *c = (so_ctx *)calloc(1, sizeof(so_ctx));
  if (!c) return NULL;
  c->p = *p;
  c->GX = 0;
  for (int a = 0; a < p->n_types && c->GX < SO_MAX_POOLS; ++a) { c->xa[c->GX] = a; c->xb[c->GX] = a; c->GX += 1; }
  if (p->mixed_types)
    for (int a = 0; a < p->n_types; ++a)
      for (int b = a + 1; b < p->n_types && c->GX < SO_MAX_POOLS; ++b) {
        c->xa[c->GX] = a;
        c->xb[c->GX] = b;
        c->GX += 1;
      }
  if (c->GX * p->n_zones > SO_MAX_POOLS) { free(c); return NULL; }
  c->ZG = p->n_zones * c->GX;
  c->inner = (uint64_t)p->n_mb * p->n_tp * p->n_dp * c->ZG;
  c->block_off = (uint64_t *)calloc((size_t)p->n_pp * 3, sizeof(uint64_t));
  c->block_size = (uint64_t *)calloc((size_t)p->n_pp * 3, sizeof(uint64_t));
  c->part_row = (uint64_t *)calloc((size_t)p->n_pp, sizeof(uint64_t));
  uint64_t off = 0, row = 0;
  for (int ip = 0; ip < p->n_pp; ++ip) {
    int P = p->pp_values[ip];
    if (P < 1 || P > p->n_layers || P > SO_MAX_STAGES) { so_destroy(c); return NULL; }
    c->part_row[ip] = row;
    row += (uint64_t)p->n_partitions[ip] * P;
    for (int s = 1; s <= 3; ++s) {
      uint64_t size = 0;
      if (segments_allowed(p, P, s)) {
        size = c->inner * n_cuts(P, s) * (uint64_t)p->n_partitions[ip];
        for (int j = 1; j < s; ++j) {
          size *= (uint64_t)(c->ZG - 1);
          if (p->per_segment_tp) size *= (uint64_t)p->n_tp; /* the segment's own TP digit */
        }
      }
      c->block_off[ip * 3 + (s - 1)] = off;
      c->block_size[ip * 3 + (s - 1)] = size;
      off += size;
    }
  }
  c->n_candidates = off;
  return c;
}

void so_destroy(so_ctx *c) {
  if (!c) return;
  free(c->block_off);
  free(c->block_size);
  free(c->part_row);
  free(c);
}

uint64_t so_num_candidates(const so_ctx *c) { return c->n_candidates; }

static void fill_values(const so_ctx *c, so_config *g) {
  g->pp = c->p.pp_values[g->pp_idx];
  g->dp = c->p.dp_values[g->dp_idx];
  g->tp = c->p.tp_values[g->tp_idx];
  for (int j = 0; j < 3; ++j) {
    if (j >= g->n_segments) { g->seg_tp_idx[j] = -1; g->seg_tp[j] = 0; continue; }
    if (!c->p.per_segment_tp || j == 0) g->seg_tp_idx[j] = g->tp_idx;
    g->seg_tp[j] = c->p.tp_values[g->seg_tp_idx[j]];
  }
  g->mb = c->p.mb_values[g->mb_idx];
}

/* index -> plan.  Digits, least significant first: mb, tp, dp, pool of segment 1,
 * [relative pool of segment 2], [relative pool of segment 3], [cut], partition.
 * With per-segment TP, "tp" is segment 1's and each later segment's own TP digit
 * follows that segment's relative pool. */
int so_decode(const so_ctx *c, uint64_t index, so_config *out) {
  const so_problem *p = &c->p;
  if (index >= c->n_candidates) return -1;
  int ip = 0, s = 1;
  for (int b = 0; b < p->n_pp * 3; ++b) {
    if (c->block_size[b] > 0 && index >= c->block_off[b] &&
        index < c->block_off[b] + c->block_size[b]) {
      ip = b / 3;
      s = b % 3 + 1;
    }
  }
  uint64_t r = index - c->block_off[ip * 3 + (s - 1)];
  so_config g;
  memset(&g, 0, sizeof g);
  g.pp_idx = ip;
  g.n_segments = s;
  int P = p->pp_values[ip];
  g.mb_idx = (int32_t)(r % p->n_mb); r /= p->n_mb;
  g.tp_idx = (int32_t)(r % p->n_tp); r /= p->n_tp;
  g.dp_idx = (int32_t)(r % p->n_dp); r /= p->n_dp;
  g.pool[0] = (int32_t)(r % c->ZG); r /= c->ZG;
  g.pool[1] = g.pool[2] = -1;
  g.cut[0] = g.cut[1] = P;
  if (s >= 2) {
    int rel = (int)(r % (c->ZG - 1)); r /= (c->ZG - 1);
    g.pool[1] = (g.pool[0] + 1 + rel) % c->ZG;
    if (p->per_segment_tp) { g.seg_tp_idx[1] = (int32_t)(r % p->n_tp); r /= p->n_tp; }
  }
  if (s == 3) {
    int rel = (int)(r % (c->ZG - 1)); r /= (c->ZG - 1);
    g.pool[2] = (g.pool[1] + 1 + rel) % c->ZG;
    if (p->per_segment_tp) { g.seg_tp_idx[2] = (int32_t)(r % p->n_tp); r /= p->n_tp; }
  }
  if (s == 2) {
    g.cut[0] = (int32_t)(r % (P - 1)) + 1; r /= (P - 1);
  } else if (s == 3) {
    uint64_t nc = n_cuts(P, 3);
    uint64_t ci = r % nc; r /= nc;
    /* pairs 1 <= k1 < k2 <= P-1 in lexicographic order */
    uint64_t seen = 0;
    for (int k1 = 1; k1 <= P - 2; ++k1)
      for (int k2 = k1 + 1; k2 <= P - 1; ++k2) {
        if (seen == ci) { g.cut[0] = k1; g.cut[1] = k2; }
        ++seen;
      }
  }
  g.partition = (int32_t)r;
  fill_values(c, &g);
  *out = g;
  return 0;
}

int so_encode(const so_ctx *c, const so_config *g, uint64_t *out) {
  const so_problem *p = &c->p;
  int ip = g->pp_idx, s = g->n_segments;
  if (ip < 0 || ip >= p->n_pp || s < 1 || s > 3) return -1;
  int P = p->pp_values[ip];
  if (c->block_size[ip * 3 + (s - 1)] == 0) return -1;
  uint64_t r = (uint64_t)g->partition;
  if (s == 2) {
    r = r * (P - 1) + (uint64_t)(g->cut[0] - 1);
  } else if (s == 3) {
    uint64_t ci = 0, seen = 0;
    for (int k1 = 1; k1 <= P - 2; ++k1)
      for (int k2 = k1 + 1; k2 <= P - 1; ++k2) {
        if (k1 == g->cut[0] && k2 == g->cut[1]) ci = seen;
        ++seen;
      }
    r = r * n_cuts(P, 3) + ci;
  }
  if (s == 3) {
    int rel = ((g->pool[2] - g->pool[1] - 1) % c->ZG + c->ZG) % c->ZG;
    if (p->per_segment_tp) r = r * p->n_tp + (uint64_t)g->seg_tp_idx[2];
    r = r * (c->ZG - 1) + (uint64_t)rel;
  }
  if (s >= 2) {
    int rel = ((g->pool[1] - g->pool[0] - 1) % c->ZG + c->ZG) % c->ZG;
    if (p->per_segment_tp) r = r * p->n_tp + (uint64_t)g->seg_tp_idx[1];
    r = r * (c->ZG - 1) + (uint64_t)rel;
  }
  r = r * c->ZG + (uint64_t)g->pool[0];
  r = r * p->n_dp + (uint64_t)g->dp_idx;
  r = r * p->n_tp + (uint64_t)g->tp_idx;
  r = r * p->n_mb + (uint64_t)g->mb_idx;
  *out = c->block_off[ip * 3 + (s - 1)] + r;
  return 0;
}

/* The same space as a loop nest (independent of so_decode): pp, then segment count,
 * then partition, cut, pools from the last segment inwards, dp, tp, mb innermost. */
uint64_t so_enumerate(const so_ctx *c, so_config *out, uint64_t max_out) {
  const so_problem *p = &c->p;
  uint64_t n = 0;
  int ZG = c->ZG;
  for (int ip = 0; ip < p->n_pp; ++ip) {
    int P = p->pp_values[ip];
    for (int s = 1; s <= 3; ++s) {
      if (!segments_allowed(p, P, s)) continue;
      for (int q = 0; q < p->n_partitions[ip]; ++q)
        for (int k1 = (s >= 2 ? 1 : P); k1 <= (s >= 2 ? P - (s - 1) : P); ++k1)
          for (int k2 = (s == 3 ? k1 + 1 : P); k2 <= (s == 3 ? P - 1 : P); ++k2)
            for (int t3 = 0; t3 < (s == 3 && p->per_segment_tp ? p->n_tp : 1); ++t3)
            for (int r3 = 0; r3 < (s == 3 ? ZG - 1 : 1); ++r3)
              for (int t2 = 0; t2 < (s >= 2 && p->per_segment_tp ? p->n_tp : 1); ++t2)
              for (int r2 = 0; r2 < (s >= 2 ? ZG - 1 : 1); ++r2)
                for (int a1 = 0; a1 < ZG; ++a1)
                  for (int id = 0; id < p->n_dp; ++id)
                    for (int it = 0; it < p->n_tp; ++it)
                      for (int im = 0; im < p->n_mb; ++im) {
                        if (n < max_out) {
                          so_config g;
                          memset(&g, 0, sizeof g);
                          g.pp_idx = ip; g.n_segments = s; g.partition = q;
                          g.cut[0] = k1; g.cut[1] = k2;
                          g.pool[0] = a1;
                          g.pool[1] = s >= 2 ? (a1 + 1 + r2) % ZG : -1;
                          g.pool[2] = s == 3 ? (g.pool[1] + 1 + r3) % ZG : -1;
                          g.dp_idx = id; g.tp_idx = it; g.mb_idx = im;
                          g.seg_tp_idx[1] = t2; g.seg_tp_idx[2] = t3;
                          fill_values(c, &g);
                          out[n] = g;
                        }
                        ++n;
                      }
    }
  }
  return n;
}

/* ---- simulator for one plan (Sec. 4.3) ------------------------------------------------- */

static const int32_t *partition_row(const so_ctx *c, const so_config *g) {
  return c->p.partition_layers + c->part_row[g->pp_idx] + (uint64_t)g->partition * g->pp;
}

static double layer_time_sum(const so_problem *p, const double *tab, int g, int im, int it,
                             int first_layer, int n) {
  /* tab is [G][n_mb][n_tp][Lc] */
  if (p->uniform_layers)
    return (double)n * tab[(((size_t)g * p->n_mb + im) * p->n_tp + it)];
  const double *row = tab + (((size_t)g * p->n_mb + im) * p->n_tp + it) * p->n_layers;
  double s = 0.0;
  for (int l = first_layer; l < first_layer + n; ++l) s += row[l];
  return s;
}

static double upd_time_sum(const so_problem *p, int g, int it, int first_layer, int n) {
  /* t_upd is [G][n_tp][Lc] */
  if (p->uniform_layers) return (double)n * p->t_upd[(size_t)g * p->n_tp + it];
  const double *row = p->t_upd + ((size_t)g * p->n_tp + it) * p->n_layers;
  double s = 0.0;
  for (int l = first_layer; l < first_layer + n; ++l) s += row[l];
  return s;
}

/* Bandwidth a message of `bytes` sees from zone a to zone b: the link's fitted polynomial
 * in log2(bytes) (Sec. 4.1), kept inside [peak / 1000, peak]; the constant peak when no
 * polynomial is given. */
static double link_bandwidth(const so_problem *p, int a, int b, double bytes) {
  const double peak = p->bandwidth[(size_t)a * p->n_zones + b];
  if (p->n_bw_coef <= 0 || !p->bw_poly || bytes < 1.0) return peak;
  const double *c = p->bw_poly + ((size_t)a * p->n_zones + b) * p->n_bw_coef;
  const double x = log2(bytes);
  double v = 0.0, xk = 1.0;
  for (int k = 0; k < p->n_bw_coef; ++k) {
    v += c[k] * xk;
    xk *= x;
  }
  if (!(v < peak)) v = peak;
  if (v < peak * 1e-3) v = peak * 1e-3;
  return v;
}

/* The simulator proper.  A plan is given stage by stage: pool_of[i] (zone * G' + extended
 * type) and the TP degree of stage i (tp_of[i], its list index tpi_of[i]); nl = layers per
 * stage; D, mb (list index mb_idx) as in the plan tuple. */
static void eval_stages(const so_ctx *c, int P, const int32_t *nl, const int *pool_of,
                        const int *tp_of, const int *tpi_of, int64_t D, int64_t mb, int mb_idx,
                        uint64_t index, int objective, int has_bound, double bound, so_eval *out) {
  const so_problem *p = &c->p;
  const int G = p->n_types, Z = p->n_zones;
  out->index = index;
  out->mask = 0;
  out->peak_mem = 0;

  /* microbatches per pipeline: the global batch is never changed (Sec. 4.2) */
  if (p->global_batch % (D * mb) != 0) {
    out->mask = SO_BIT_BATCH;
    out->iter_time = INFINITY;
    out->cost = INFINITY;
    return;
  }
  const int64_t Nb = p->global_batch / (D * mb);

  /* the stage's replicas are of type type_of[i], or half of them of type type_b[i] */
  int type_of[SO_MAX_STAGES], type_b[SO_MAX_STAGES], zone_of[SO_MAX_STAGES], first_layer[SO_MAX_STAGES];
  /* GPUs that one replica of the plan takes from every real (zone, type) pool, counted in
   * halves: a stage whose replicas are split over two types takes half a replica from each */
  int64_t half_gpus_on_pool[SO_MAX_POOLS];
  memset(half_gpus_on_pool, 0, sizeof half_gpus_on_pool);
  int layer = 0;
  for (int i = 0; i < P; ++i) {
    int pool = pool_of[i];
    type_of[i] = c->xa[pool % c->GX];
    type_b[i] = c->xb[pool % c->GX];
    zone_of[i] = pool / c->GX;
    if (type_b[i] == type_of[i]) {
      half_gpus_on_pool[zone_of[i] * G + type_of[i]] += 2 * tp_of[i];
    } else {
      half_gpus_on_pool[zone_of[i] * G + type_of[i]] += tp_of[i];
      half_gpus_on_pool[zone_of[i] * G + type_b[i]] += tp_of[i];
      if (D % 2 != 0) out->mask |= SO_BIT_QUOTA; /* D replicas cannot be halved */
    }
    first_layer[i] = layer;
    layer += nl[i];
  }

  /* H1: a tensor-parallel group stays inside one node (Sec. 4.2.1) */
  for (int i = 0; i < P; ++i)
    if (tp_of[i] > p->gpus_per_node[type_of[i]] || tp_of[i] > p->gpus_per_node[type_b[i]])
      out->mask |= SO_BIT_TP_NODE;

  /* quota: D replicas of every stage, tp GPUs each, from the stage's (zone, type) pool(s) */
  for (int a = 0; a < Z * G; ++a)
    if (half_gpus_on_pool[a] * D > 2 * (int64_t)p->avail[a]) out->mask |= SO_BIT_QUOTA;

  /* memory per worker of each stage: M_model + M_activation (+ reserved), Sec. 4.3 */
  uint64_t params_of[SO_MAX_STAGES];
  uint64_t peak = 0;
  for (int i = 0; i < P; ++i) {
    uint64_t params = 0;
    for (int l = first_layer[i]; l < first_layer[i] + nl[i]; ++l) params += p->layer_params[l];
    if (i == 0) params += p->embed_params;
    if (i == P - 1) params += p->head_params;
    uint64_t shard = (params + (uint64_t)tp_of[i] - 1) / (uint64_t)tp_of[i];
    params_of[i] = shard;
    uint64_t m_model = shard * (uint64_t)p->bytes_per_param;
    int64_t inflight = (P - i) < Nb ? (P - i) : Nb; /* 1F1B: microbatches kept alive */
    uint64_t m_act = (uint64_t)inflight * (uint64_t)nl[i] *
                     p->act_store_bytes[(size_t)mb_idx * p->n_tp + tpi_of[i]];
    uint64_t m = m_model + m_act + p->mem_reserved[type_of[i]];
    if (m > p->mem_capacity[type_of[i]]) out->mask |= SO_BIT_OOM;
    if (m > peak) peak = m;
    if (type_b[i] != type_of[i]) { /* the other half of the replicas */
      uint64_t m2 = m_model + m_act + p->mem_reserved[type_b[i]];
      if (m2 > p->mem_capacity[type_b[i]]) out->mask |= SO_BIT_OOM;
      if (m2 > peak) peak = m2;
    }
  }
  out->peak_mem = peak;

  /* stage times: compute plus activation / gradient transfers to the neighbours */
  const double p2p = (double)p->p2p_bytes[mb_idx];
  double sum_t = 0.0, max_t = 0.0, t_sync = 0.0, t_upd = 0.0;
  for (int i = 0; i < P; ++i) {
    int gt = type_of[i], z = zone_of[i];
    double f = layer_time_sum(p, p->t_fwd, gt, mb_idx, tpi_of[i], first_layer[i], nl[i]);
    double b = layer_time_sum(p, p->t_bwd, gt, mb_idx, tpi_of[i], first_layer[i], nl[i]);
    if (type_b[i] != gt) { /* the slower replica type sets the stage's pace (straggler, Sec. 4.3) */
      double f2 = layer_time_sum(p, p->t_fwd, type_b[i], mb_idx, tpi_of[i], first_layer[i], nl[i]);
      double b2 = layer_time_sum(p, p->t_bwd, type_b[i], mb_idx, tpi_of[i], first_layer[i], nl[i]);
      if (f2 + b2 > f + b) { f = f2; b = b2; }
    }
    double x = 0.0;
    if (i < P - 1) x += p2p / link_bandwidth(p, z, zone_of[i + 1], p2p);
    if (i > 0) x += p2p / link_bandwidth(p, z, zone_of[i - 1], p2p);
    double t = f + b + x;
    sum_t += t;
    if (t > max_t) max_t = t;
    /* gradient all-reduce of the stage's D replicas inside their zone: ring */
    double sync = 0.0;
    if (D > 1) {
      const double grad_bytes = (double)params_of[i] * (double)p->grad_bytes_per_param;
      sync = 2.0 * (double)(D - 1) / (double)D * grad_bytes / link_bandwidth(p, z, z, grad_bytes);
    }
    if (sync > t_sync) t_sync = sync;
    double u = upd_time_sum(p, gt, tpi_of[i], first_layer[i], nl[i]);
    if (u > t_upd) t_upd = u;
    if (type_b[i] != gt) {
      double u2 = upd_time_sum(p, type_b[i], tpi_of[i], first_layer[i], nl[i]);
      if (u2 > t_upd) t_upd = u2;
    }
  }
  /* 1F1B: warm-up + cool-down pass every stage once, the steady phase repeats the
   * straggler for the remaining microbatches */
  const double t_pp = sum_t + (double)(Nb - 1) * max_t;
  const double t_iter = t_pp + t_sync + t_upd;
  out->iter_time = t_iter;

  /* cost per iteration: rented GPUs for T_iter plus cross-zone traffic */
  double gpu_dollars_per_hour = 0.0, c_comm = 0.0;
  for (int i = 0; i < P; ++i)
    gpu_dollars_per_hour +=
        type_b[i] == type_of[i]
            ? (double)(D * tp_of[i]) * p->price_per_hour[type_of[i]]
            : (double)(D * tp_of[i]) * (0.5 * (p->price_per_hour[type_of[i]] + p->price_per_hour[type_b[i]]));
  if (p->egress_per_byte)
    for (int i = 0; i + 1 < P; ++i) {
      int z = zone_of[i], zn = zone_of[i + 1];
      if (z != zn)
        c_comm += (double)Nb * (double)D * p2p *
                  (p->egress_per_byte[(size_t)z * Z + zn] + p->egress_per_byte[(size_t)zn * Z + z]);
    }
  out->cost = gpu_dollars_per_hour / 3600.0 * t_iter + c_comm;

  if (has_bound) {
    if (objective == SO_MAX_THROUGHPUT) {
      if (out->cost > bound) out->mask |= SO_BIT_CONSTRAINT;
    } else {
      if (1.0 / t_iter < bound) out->mask |= SO_BIT_CONSTRAINT;
    }
  }
}

/* A plan of the flat space: every stage takes the pool and the TP degree of its segment. */
static void eval_config(const so_ctx *c, const so_config *g, uint64_t index, int objective,
                        int has_bound, double bound, so_eval *out) {
  int pool_of[SO_MAX_STAGES];
  int tp_of[SO_MAX_STAGES], tpi_of[SO_MAX_STAGES]; /* TP degree of the stage and its list index */
  for (int i = 0; i < g->pp; ++i) {
    int seg = (i < g->cut[0]) ? 0 : (i < g->cut[1]) ? 1 : 2;
    pool_of[i] = g->pool[seg];
    tp_of[i] = g->seg_tp[seg];
    tpi_of[i] = g->seg_tp_idx[seg];
  }
  eval_stages(c, g->pp, partition_row(c, g), pool_of, tp_of, tpi_of, g->dp, g->mb, g->mb_idx, index,
              objective, has_bound, bound, out);
}

/* A plan whose stages choose their pools freely (the plan tuple of Sec. 4.2 without the
 * contiguous-segment restriction of the flat space): pools[i] = zone * G' + extended type of
 * stage i, one TP degree for all stages.  Returns 0, -1 for a value out of range. */
int so_eval_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                          const int32_t *tp_idx, const int32_t *pools, int objective, int has_bound,
                          double bound, so_eval *out) {
  const so_problem *p = &c->p;
  if (pp_idx < 0 || pp_idx >= p->n_pp || dp_idx < 0 || dp_idx >= p->n_dp || mb_idx < 0 ||
      mb_idx >= p->n_mb || partition < 0 || partition >= p->n_partitions[pp_idx])
    return -1;
  const int P = p->pp_values[pp_idx];
  int pool_of[SO_MAX_STAGES], tp_of[SO_MAX_STAGES], tpi_of[SO_MAX_STAGES];
  for (int i = 0; i < P; ++i) {
    if (pools[i] < 0 || pools[i] >= c->ZG || tp_idx[i] < 0 || tp_idx[i] >= p->n_tp) return -1;
    pool_of[i] = pools[i];
    tp_of[i] = p->tp_values[tp_idx[i]];
    tpi_of[i] = tp_idx[i];
  }
  so_config g;
  memset(&g, 0, sizeof g);
  g.pp_idx = pp_idx;
  g.pp = P;
  g.partition = partition;
  eval_stages(c, P, partition_row(c, &g), pool_of, tp_of, tpi_of, p->dp_values[dp_idx],
              p->mb_values[mb_idx], mb_idx, 0, objective, has_bound, bound, out);
  return 0;
}

int so_eval_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx, int tp_idx,
                       const int32_t *pools, int objective, int has_bound, double bound,
                       so_eval *out) {
  int32_t tps[SO_MAX_STAGES];
  for (int i = 0; i < SO_MAX_STAGES; ++i) tps[i] = tp_idx;
  return so_eval_assignment_tp(c, pp_idx, partition, dp_idx, mb_idx, tps, pools, objective, has_bound,
                               bound, out);
}

/* A plan whose stages may split their D replicas over two pools, half on each -- pools of
 * different zones too (the D tuples (GPU, TP, zone) of a stage, Sec. 4.2).  Replicas 0 .. D/2-1
 * form the pipelines through the first pools, the others the pipelines through the second
 * pools; the two kinds of pipeline differ in stage times and transfers, and the iteration
 * waits for the slower kind: T_iter = max(T_pp) + T_sync + T_update (Sec. 4.3).  The gradient
 * all-reduce of a split stage is a ring through both pools and runs at the pace of its slowest
 * link (intra-zone links of both zones, the two links between them).  Cross-zone traffic is
 * paid for: the pipelines' transfers (each kind of pipeline carries half of the replicas) and
 * the two ring links between the zones of a split stage.
 * pools_a[i] / pools_b[i]: zone * n_types + type (plain pools only); equal = not split.
 * tp_idx[i]: index of stage i's TP degree (both halves of a stage use the same degree); the
 * stage's shard, activation bytes, profiled times, node-size check, quota and rent follow it.
 * Returns 0, -1 for a value out of range or a problem with extended types. */
int so_eval_split_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                const int32_t *tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                                int objective, int has_bound, double bound, so_eval *out) {
  const so_problem *p = &c->p;
  if (p->mixed_types || pp_idx < 0 || pp_idx >= p->n_pp || dp_idx < 0 || dp_idx >= p->n_dp ||
      mb_idx < 0 || mb_idx >= p->n_mb || partition < 0 || partition >= p->n_partitions[pp_idx])
    return -1;
  const int P = p->pp_values[pp_idx], G = p->n_types, Z = p->n_zones;
  for (int i = 0; i < P; ++i)
    if (pools_a[i] < 0 || pools_a[i] >= Z * G || pools_b[i] < 0 || pools_b[i] >= Z * G ||
        tp_idx[i] < 0 || tp_idx[i] >= p->n_tp)
      return -1;
  const int64_t replicas = p->dp_values[dp_idx], micro = p->mb_values[mb_idx];
  so_config g;
  memset(&g, 0, sizeof g);
  g.pp_idx = pp_idx; g.pp = P; g.partition = partition;
  const int32_t *nl = partition_row(c, &g);
  out->index = 0; out->mask = 0; out->peak_mem = 0;
  if (p->global_batch % (replicas * micro) != 0) {
    out->mask = SO_BIT_BATCH;
    out->iter_time = INFINITY;
    out->cost = INFINITY;
    return 0;
  }
  const int64_t n_micro = p->global_batch / (replicas * micro);
  const int32_t *side[2] = {pools_a, pools_b};

  /* quota, counted in half replicas; node size; an odd D cannot be halved */
  int64_t halves[SO_MAX_POOLS];
  memset(halves, 0, sizeof halves);
  for (int i = 0; i < P; ++i) {
    const int64_t width = p->tp_values[tp_idx[i]]; /* GPUs of one replica of this stage */
    halves[pools_a[i]] += width;
    halves[pools_b[i]] += width;
    if (pools_a[i] != pools_b[i] && replicas % 2 != 0) out->mask |= SO_BIT_QUOTA;
    for (int h = 0; h < 2; ++h)
      if (width > p->gpus_per_node[side[h][i] % G]) out->mask |= SO_BIT_TP_NODE;
  }
  for (int a = 0; a < Z * G; ++a)
    if (halves[a] * replicas > 2 * (int64_t)p->avail[a]) out->mask |= SO_BIT_QUOTA;

  /* memory of a worker of either half */
  uint64_t shard_of[SO_MAX_STAGES];
  int first_of[SO_MAX_STAGES];
  int layer = 0;
  uint64_t peak = 0;
  for (int i = 0; i < P; ++i) {
    uint64_t params = 0;
    first_of[i] = layer;
    for (int l = layer; l < layer + nl[i]; ++l) params += p->layer_params[l];
    layer += nl[i];
    if (i == 0) params += p->embed_params;
    if (i + 1 == P) params += p->head_params;
    const uint64_t width = (uint64_t)p->tp_values[tp_idx[i]];
    shard_of[i] = (params + width - 1) / width;
    const int64_t alive = (P - i) < n_micro ? (P - i) : n_micro;
    const uint64_t bytes = shard_of[i] * (uint64_t)p->bytes_per_param +
                           (uint64_t)alive * (uint64_t)nl[i] *
                               p->act_store_bytes[(size_t)mb_idx * p->n_tp + tp_idx[i]];
    for (int h = 0; h < 2; ++h) {
      const int gt = side[h][i] % G;
      const uint64_t m = bytes + p->mem_reserved[gt];
      if (m > p->mem_capacity[gt]) out->mask |= SO_BIT_OOM;
      if (m > peak) peak = m;
    }
  }
  out->peak_mem = peak;

  /* the two kinds of pipeline */
  const double msg = (double)p->p2p_bytes[mb_idx];
  const double *price_of_byte = p->egress_per_byte; /* $/byte between zones, or NULL */
  double t_pipe = 0.0, t_update = 0.0, traffic_cost = 0.0;
  for (int h = 0; h < 2; ++h) {
    double total = 0.0, slowest = 0.0;
    for (int i = 0; i < P; ++i) {
      const int gt = side[h][i] % G, z = side[h][i] / G;
      double t = layer_time_sum(p, p->t_fwd, gt, mb_idx, tp_idx[i], first_of[i], nl[i]) +
                 layer_time_sum(p, p->t_bwd, gt, mb_idx, tp_idx[i], first_of[i], nl[i]);
      double moves = 0.0;
      if (i < P - 1) {
        const int zn = side[h][i + 1] / G;
        moves += msg / link_bandwidth(p, z, zn, msg);
        if (price_of_byte && zn != z) /* this kind of pipeline carries half of the replicas */
          traffic_cost += (double)n_micro * (0.5 * (double)replicas) * msg *
                          (price_of_byte[(size_t)z * Z + zn] + price_of_byte[(size_t)zn * Z + z]);
      }
      if (i > 0) moves += msg / link_bandwidth(p, z, side[h][i - 1] / G, msg);
      t += moves;
      total += t;
      if (t > slowest) slowest = t;
      const double u = upd_time_sum(p, gt, tp_idx[i], first_of[i], nl[i]);
      if (u > t_update) t_update = u;
    }
    const double t_kind = total + (double)(n_micro - 1) * slowest;
    if (t_kind > t_pipe) t_pipe = t_kind;
  }

  /* gradient all-reduce per stage: a ring through both pools, as fast as its slowest link */
  double t_allreduce = 0.0;
  if (replicas > 1)
    for (int i = 0; i < P; ++i) {
      const int za = pools_a[i] / G, zb = pools_b[i] / G;
      const double buffer = (double)shard_of[i] * (double)p->grad_bytes_per_param;
      double link = link_bandwidth(p, za, za, buffer);
      if (zb != za) {
        const double others[3] = {link_bandwidth(p, zb, zb, buffer), link_bandwidth(p, za, zb, buffer),
                                  link_bandwidth(p, zb, za, buffer)};
        for (int k = 0; k < 3; ++k)
          if (others[k] < link) link = others[k];
      }
      const double ring_bytes = 2.0 * (double)(replicas - 1) / (double)replicas * buffer;
      const double t = ring_bytes / link;
      if (t > t_allreduce) t_allreduce = t;
      if (price_of_byte && zb != za) /* the ring crosses between the zones once each way */
        traffic_cost += ring_bytes * (price_of_byte[(size_t)za * Z + zb] + price_of_byte[(size_t)zb * Z + za]);
    }
  out->iter_time = t_pipe + t_allreduce + t_update;

  double rent = 0.0; /* $/h of all replicas: half of a stage's at each pool's price */
  for (int i = 0; i < P; ++i)
    rent += (double)(replicas * (int64_t)p->tp_values[tp_idx[i]]) *
            (0.5 * (p->price_per_hour[pools_a[i] % G] + p->price_per_hour[pools_b[i] % G]));
  out->cost = rent / 3600.0 * out->iter_time + traffic_cost;
  if (has_bound) {
    if (objective == SO_MAX_THROUGHPUT ? out->cost > bound : 1.0 / out->iter_time < bound)
      out->mask |= SO_BIT_CONSTRAINT;
  }
  return 0;
}

/* The same with one TP degree for all stages. */
int so_eval_split_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                             int tp_idx, const int32_t *pools_a, const int32_t *pools_b,
                             int objective, int has_bound, double bound, so_eval *out) {
  int32_t every_stage[SO_MAX_STAGES];
  for (int i = 0; i < SO_MAX_STAGES; ++i) every_stage[i] = tp_idx;
  return so_eval_split_assignment_tp(c, pp_idx, partition, dp_idx, mb_idx, every_stage, pools_a, pools_b,
                                     objective, has_bound, bound, out);
}

const so_problem *so_problem_of(const so_ctx *c) { return &c->p; }

int so_eval_one(const so_ctx *c, uint64_t index, int objective, int has_bound, double bound,
                so_eval *out) {
  so_config g;
  if (so_decode(c, index, &g) != 0) return -1;
  eval_config(c, &g, index, objective, has_bound, bound, out);
  return 0;
}

/* ---- discrete-event 1F1B schedule of one pipeline -------------------------------------- */

/* The op a stage runs at position pos of its 1F1B order (warm-up forwards, one forward /
 * one backward in turn, the remaining backwards): kind 0 = forward, 1 = backward. */
static void op_at(int P, int64_t M, int i, int64_t pos, int *kind, int64_t *m) {
  int64_t w = (P - 1 - i) < M ? (P - 1 - i) : M;
  if (pos < w) { *kind = 0; *m = pos; return; }
  int64_t q = pos - w;
  if (q < 2 * (M - w)) {
    if (q % 2 == 0) { *kind = 0; *m = w + q / 2; }
    else { *kind = 1; *m = q / 2; }
    return;
  }
  *kind = 1;
  *m = (M - w) + (q - 2 * (M - w));
}

/* Makespan of the 1F1B schedule of one pipeline of the plan, event by event (Sec. 4.3 names
 * the warm-up, steady and cool-down phases; the closed form of Sec. 4.2.2 summarises them).
 * A forward of stage i takes its layers' forward time plus the transfer of the activations
 * to stage i + 1, a backward its layers' backward time plus the transfer of the gradients to
 * stage i - 1 (transfers are not overlapped, as in the closed form).  A forward starts when
 * the stage is free and the previous stage's forward of that microbatch has ended, a backward
 * when the next stage's backward has ended (the last stage: its own forward).
 * t_closed receives sum_i t_i + (N_b - 1) max_i t_i of the same stage times.
 * Returns 0, -1 for a bad index, 1 when the batch does not divide (outputs +inf). */
int so_simulate_1f1b(const so_ctx *c, uint64_t index, double *t_event, double *t_closed) {
  const so_problem *p = &c->p;
  so_config g;
  if (so_decode(c, index, &g) != 0) return -1;
  const int P = g.pp;
  const int32_t *nl = partition_row(c, &g);
  if (p->global_batch % ((int64_t)g.dp * g.mb) != 0) {
    *t_event = INFINITY;
    *t_closed = INFINITY;
    return 1;
  }
  const int64_t M = p->global_batch / ((int64_t)g.dp * g.mb);
  const double p2p = (double)p->p2p_bytes[g.mb_idx];
  double fdur[SO_MAX_STAGES], bdur[SO_MAX_STAGES];
  int zone_of[SO_MAX_STAGES], type_of[SO_MAX_STAGES], type_b[SO_MAX_STAGES], tpi_of[SO_MAX_STAGES];
  for (int i = 0; i < P; ++i) {
    int seg = (i < g.cut[0]) ? 0 : (i < g.cut[1]) ? 1 : 2;
    type_of[i] = c->xa[g.pool[seg] % c->GX];
    type_b[i] = c->xb[g.pool[seg] % c->GX];
    zone_of[i] = g.pool[seg] / c->GX;
    tpi_of[i] = g.seg_tp_idx[seg];
  }
  int layer = 0;
  double sum_t = 0.0, max_t = 0.0;
  for (int i = 0; i < P; ++i) {
    double f = layer_time_sum(p, p->t_fwd, type_of[i], g.mb_idx, tpi_of[i], layer, nl[i]);
    double b = layer_time_sum(p, p->t_bwd, type_of[i], g.mb_idx, tpi_of[i], layer, nl[i]);
    if (type_b[i] != type_of[i]) { /* the pipeline through the slower replica type */
      double f2 = layer_time_sum(p, p->t_fwd, type_b[i], g.mb_idx, tpi_of[i], layer, nl[i]);
      double b2 = layer_time_sum(p, p->t_bwd, type_b[i], g.mb_idx, tpi_of[i], layer, nl[i]);
      if (f2 + b2 > f + b) { f = f2; b = b2; }
    }
    double send_f = (i < P - 1) ? p2p / link_bandwidth(p, zone_of[i], zone_of[i + 1], p2p) : 0.0;
    double send_b = (i > 0) ? p2p / link_bandwidth(p, zone_of[i], zone_of[i - 1], p2p) : 0.0;
    fdur[i] = f + send_f;
    bdur[i] = b + send_b;
    double t = f + b + (send_f + send_b);
    sum_t += t;
    if (t > max_t) max_t = t;
    layer += nl[i];
  }
  *t_closed = sum_t + (double)(M - 1) * max_t;

  double *fdone = (double *)malloc(sizeof(double) * (size_t)P * (size_t)M * 2);
  if (!fdone) return -1;
  double *bdone = fdone + (size_t)P * (size_t)M;
  for (size_t k = 0; k < (size_t)P * (size_t)M * 2; ++k) fdone[k] = -1.0; /* not yet run */
  int64_t pos[SO_MAX_STAGES];
  double free_at[SO_MAX_STAGES];
  for (int i = 0; i < P; ++i) { pos[i] = 0; free_at[i] = 0.0; }
  int progressed = 1;
  while (progressed) {
    progressed = 0;
    for (int i = 0; i < P; ++i) {
      while (pos[i] < 2 * M) {
        int kind;
        int64_t m;
        op_at(P, M, i, pos[i], &kind, &m);
        double dep;
        if (kind == 0) dep = (i == 0) ? 0.0 : fdone[(size_t)(i - 1) * M + m];
        else dep = (i == P - 1) ? fdone[(size_t)i * M + m] : bdone[(size_t)(i + 1) * M + m];
        if (dep < 0.0) break; /* the neighbour has not produced it yet */
        double start = free_at[i] > dep ? free_at[i] : dep;
        free_at[i] = start + (kind == 0 ? fdur[i] : bdur[i]);
        (kind == 0 ? fdone : bdone)[(size_t)i * M + m] = free_at[i];
        pos[i] += 1;
        progressed = 1;
      }
    }
  }
  double end = 0.0;
  for (int i = 0; i < P; ++i) {
    if (pos[i] != 2 * M) { free(fdone); return -1; } /* cannot happen: the order is deadlock-free */
    if (free_at[i] > end) end = free_at[i];
  }
  free(fdone);
  *t_event = end;
  return 0;
}

static double key_of(const so_eval *e, int objective) {
  return objective == SO_MAX_THROUGHPUT ? e->iter_time : e->cost;
}

/* ---- plain thread sharding by contiguous index range ---------------------------------- */

typedef struct {
  const so_ctx *c;
  uint64_t first, count;
  const uint64_t *indices;
  int objective, has_bound, k, mode; /* mode 0 batch, 1 min key, 2 first within tol, 3 top-k */
  double bound, limit;
  double *time, *cost;
  uint64_t *mem;
  uint32_t *mask;
  /* results */
  int found;
  so_eval best;
  so_eval *top;
  int n_top;
} so_job;

static int lex_less(double ka, uint64_t ia, double kb, uint64_t ib) {
  return ka < kb || (ka == kb && ia < ib);
}

static void *run_job(void *arg) {
  so_job *j = (so_job *)arg;
  j->found = 0;
  j->n_top = 0;
  for (uint64_t n = 0; n < j->count; ++n) {
    uint64_t idx = j->indices ? j->indices[j->first + n] : j->first + n;
    so_eval e;
    if (so_eval_one(j->c, idx, j->objective, j->has_bound, j->bound, &e) != 0) continue;
    if (j->mode == 0) {
      uint64_t o = j->first + n;
      if (j->time) j->time[o] = e.iter_time;
      if (j->cost) j->cost[o] = e.cost;
      if (j->mem) j->mem[o] = e.peak_mem;
      if (j->mask) j->mask[o] = e.mask;
      continue;
    }
    if (e.mask != 0) continue;
    double key = key_of(&e, j->objective);
    if (j->mode == 1) {
      if (!j->found || key < key_of(&j->best, j->objective)) { j->best = e; j->found = 1; }
    } else if (j->mode == 2) {
      if (key <= j->limit) { j->best = e; j->found = 1; break; } /* lowest index in range */
    } else {
      /* insertion into the sorted list of the k best so far */
      int pos = j->n_top;
      while (pos > 0 && lex_less(key, e.index, key_of(&j->top[pos - 1], j->objective),
                                 j->top[pos - 1].index))
        --pos;
      if (pos < j->k) {
        int last = j->n_top < j->k ? j->n_top : j->k - 1;
        for (int m = last; m > pos; --m) j->top[m] = j->top[m - 1];
        j->top[pos] = e;
        if (j->n_top < j->k) j->n_top += 1;
      }
    }
  }
  return NULL;
}

static void run_sharded(so_job *proto, int n_threads, so_job *jobs) {
  if (n_threads < 1) n_threads = 1;
  pthread_t th[256];
  if (n_threads > 256) n_threads = 256;
  uint64_t per = (proto->count + n_threads - 1) / n_threads;
  for (int t = 0; t < n_threads; ++t) {
    jobs[t] = *proto;
    uint64_t lo = per * t;
    if (lo > proto->count) lo = proto->count;
    uint64_t hi = lo + per < proto->count ? lo + per : proto->count;
    jobs[t].first = proto->first + lo;
    jobs[t].count = hi - lo;
    if (proto->mode == 3) jobs[t].top = (so_eval *)calloc((size_t)proto->k, sizeof(so_eval));
  }
  if (n_threads == 1) {
    run_job(&jobs[0]);
    return;
  }
  for (int t = 0; t < n_threads; ++t) pthread_create(&th[t], NULL, run_job, &jobs[t]);
  for (int t = 0; t < n_threads; ++t) pthread_join(th[t], NULL);
}

int so_eval_batch(const so_ctx *c, uint64_t first, uint64_t count, const uint64_t *indices,
                  int objective, int has_bound, double bound, double *time, double *cost,
                  uint64_t *mem, uint32_t *mask, int n_threads) {
  /* outputs are written at position first + n when a range is given, n when a list is */
  so_job proto;
  memset(&proto, 0, sizeof proto);
  proto.c = c; proto.count = count; proto.indices = indices;
  proto.objective = objective; proto.has_bound = has_bound; proto.bound = bound;
  proto.mode = 0;
  if (indices) {
    proto.first = 0;
    proto.time = time; proto.cost = cost; proto.mem = mem; proto.mask = mask;
  } else {
    if (first + count > c->n_candidates) return -1;
    proto.first = first;
    proto.time = time ? time - first : NULL;
    proto.cost = cost ? cost - first : NULL;
    proto.mem = mem ? mem - first : NULL;
    proto.mask = mask ? mask - first : NULL;
  }
  so_job jobs[256];
  run_sharded(&proto, n_threads, jobs);
  return 0;
}

int so_best(const so_ctx *c, uint64_t first, uint64_t count, int objective, int has_bound,
            double bound, int n_threads, so_eval *out) {
  if (first + count > c->n_candidates) return 0;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 256) n_threads = 256;
  so_job proto, jobs[256];
  memset(&proto, 0, sizeof proto);
  proto.c = c; proto.first = first; proto.count = count;
  proto.objective = objective; proto.has_bound = has_bound; proto.bound = bound;
  /* pass 1: the minimum key over feasible candidates */
  proto.mode = 1;
  run_sharded(&proto, n_threads, jobs);
  int found = 0;
  double vmin = 0.0;
  for (int t = 0; t < n_threads; ++t)
    if (jobs[t].found) {
      double k = key_of(&jobs[t].best, objective);
      if (!found || k < vmin) { vmin = k; found = 1; }
    }
  if (!found) return 0;
  /* pass 2: the lowest index whose key lies within the tie tolerance of the minimum */
  proto.mode = 2;
  proto.limit = vmin * (1.0 + SO_TIE_TOL);
  run_sharded(&proto, n_threads, jobs);
  for (int t = 0; t < n_threads; ++t)
    if (jobs[t].found) { *out = jobs[t].best; return 1; } /* shards are in index order */
  return 0;
}

int so_topk(const so_ctx *c, uint64_t first, uint64_t count, int objective, int has_bound,
            double bound, int k, int n_threads, so_eval *out) {
  if (first + count > c->n_candidates || k < 1) return 0;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 256) n_threads = 256;
  so_job proto, jobs[256];
  memset(&proto, 0, sizeof proto);
  proto.c = c; proto.first = first; proto.count = count;
  proto.objective = objective; proto.has_bound = has_bound; proto.bound = bound;
  proto.mode = 3; proto.k = k;
  run_sharded(&proto, n_threads, jobs);
  /* merge the per-shard lists: repeatedly take the lexicographically smallest head */
  int head[256];
  memset(head, 0, sizeof head);
  int n = 0;
  while (n < k) {
    int bt = -1;
    for (int t = 0; t < n_threads; ++t) {
      if (head[t] >= jobs[t].n_top) continue;
      so_eval *e = &jobs[t].top[head[t]];
      if (bt < 0 || lex_less(key_of(e, objective), e->index,
                             key_of(&jobs[bt].top[head[bt]], objective),
                             jobs[bt].top[head[bt]].index))
        bt = t;
    }
    if (bt < 0) break;
    out[n++] = jobs[bt].top[head[bt]++];
  }
  for (int t = 0; t < n_threads; ++t) free(jobs[t].top);
  return n;
}

int so_eval_replica_assignment_tp(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                                  const int32_t *tp_idx, const int32_t *pools, int objective,
                                  int has_bound, double bound, so_eval *out) {
  const so_problem *p = &c->p;
  if (p->mixed_types || pp_idx < 0 || pp_idx >= p->n_pp || dp_idx < 0 || dp_idx >= p->n_dp ||
      mb_idx < 0 || mb_idx >= p->n_mb || partition < 0 || partition >= p->n_partitions[pp_idx])
    return -1;
  const int P = p->pp_values[pp_idx], G = p->n_types, Z = p->n_zones;
  const int64_t D = p->dp_values[dp_idx], micro = p->mb_values[mb_idx];
  for (int64_t k = 0; k < (int64_t)P * D; ++k)
    if (pools[k] < 0 || pools[k] >= Z * G) return -1;
  for (int i = 0; i < P; ++i)
    if (tp_idx[i] < 0 || tp_idx[i] >= p->n_tp) return -1;
  so_config g;
  memset(&g, 0, sizeof g);
  g.pp_idx = pp_idx; g.pp = P; g.partition = partition;
  const int32_t *nl = partition_row(c, &g);
  out->index = 0; out->mask = 0; out->peak_mem = 0;
  if (p->global_batch % (D * micro) != 0) {
    out->mask = SO_BIT_BATCH;
    out->iter_time = INFINITY;
    out->cost = INFINITY;
    return 0;
  }
  const int64_t n_micro = p->global_batch / (D * micro);

  /* what every pool gives, node size, memory of every replica's worker */
  int64_t gpus[SO_MAX_POOLS];
  memset(gpus, 0, sizeof gpus);
  uint64_t shard_of[SO_MAX_STAGES], peak = 0;
  int first_of[SO_MAX_STAGES];
  int layer = 0;
  for (int i = 0; i < P; ++i) {
    uint64_t params = 0;
    first_of[i] = layer;
    for (int l = layer; l < layer + nl[i]; ++l) params += p->layer_params[l];
    layer += nl[i];
    if (i == 0) params += p->embed_params;
    if (i + 1 == P) params += p->head_params;
    const int64_t degree = p->tp_values[tp_idx[i]]; /* every replica of the stage runs at it */
    shard_of[i] = (params + (uint64_t)degree - 1) / (uint64_t)degree;
    const int64_t in_flight = (P - i) < n_micro ? (P - i) : n_micro;
    const uint64_t bytes = shard_of[i] * (uint64_t)p->bytes_per_param +
                           (uint64_t)in_flight * (uint64_t)nl[i] *
                               p->act_store_bytes[(size_t)mb_idx * p->n_tp + (size_t)tp_idx[i]]; /* at the stage's degree */
    for (int64_t r = 0; r < D; ++r) {
      const int a = pools[(int64_t)i * D + r], gt = a % G;
      gpus[a] += degree;
      if (degree > p->gpus_per_node[gt]) out->mask |= SO_BIT_TP_NODE;
      const uint64_t m = bytes + p->mem_reserved[gt];
      if (m > p->mem_capacity[gt]) out->mask |= SO_BIT_OOM;
      if (m > peak) peak = m;
    }
  }
  for (int a = 0; a < Z * G; ++a)
    if (gpus[a] > (int64_t)p->avail[a]) out->mask |= SO_BIT_QUOTA;
  out->peak_mem = peak;

  /* the D pipelines, each with its own stage times and transfers */
  const double msg = (double)p->p2p_bytes[mb_idx];
  const double *fee = p->egress_per_byte; /* $/byte between zones, or NULL */
  double t_pipe = 0.0, t_update = 0.0, traffic_cost = 0.0, rent = 0.0;
  for (int64_t r = 0; r < D; ++r) {
    double total = 0.0, slowest = 0.0;
    for (int i = 0; i < P; ++i) {
      const int a = pools[(int64_t)i * D + r], gt = a % G, z = a / G;
      double t = layer_time_sum(p, p->t_fwd, gt, mb_idx, tp_idx[i], first_of[i], nl[i]) +
                 layer_time_sum(p, p->t_bwd, gt, mb_idx, tp_idx[i], first_of[i], nl[i]);
      double moves = 0.0;
      if (i < P - 1) {
        const int zn = pools[(int64_t)(i + 1) * D + r] / G;
        moves += msg / link_bandwidth(p, z, zn, msg);
        if (fee && zn != z) /* one replica's microbatches, both directions */
          traffic_cost += (double)n_micro * msg * (fee[(size_t)z * Z + zn] + fee[(size_t)zn * Z + z]);
      }
      if (i > 0) moves += msg / link_bandwidth(p, z, pools[(int64_t)(i - 1) * D + r] / G, msg);
      t += moves;
      total += t;
      if (t > slowest) slowest = t;
      const double step = upd_time_sum(p, gt, tp_idx[i], first_of[i], nl[i]); /* optimizer step */
      if (step > t_update) t_update = step;
      rent += (double)p->tp_values[tp_idx[i]] * p->price_per_hour[gt];
    }
    const double t_this = total + (double)(n_micro - 1) * slowest;
    if (t_this > t_pipe) t_pipe = t_this;
  }

  /* gradient all-reduce per stage: a ring through the replicas in their order */
  double t_allreduce = 0.0;
  if (D > 1)
    for (int i = 0; i < P; ++i) {
      const double buffer = (double)shard_of[i] * (double)p->grad_bytes_per_param;
      const double ring_bytes = 2.0 * (double)(D - 1) / (double)D * buffer;
      double link = INFINITY;
      for (int64_t r = 0; r < D; ++r) {
        const int zr = pools[(int64_t)i * D + r] / G, zs = pools[(int64_t)i * D + (r + 1) % D] / G;
        const double w = link_bandwidth(p, zr, zs, buffer);
        if (w < link) link = w;
        if (fee && zr != zs) traffic_cost += ring_bytes * fee[(size_t)zr * Z + zs];
      }
      const double t = ring_bytes / link;
      if (t > t_allreduce) t_allreduce = t;
    }
  out->iter_time = t_pipe + t_allreduce + t_update;
  out->cost = rent / 3600.0 * out->iter_time + traffic_cost;
  if (has_bound) {
    if (objective == SO_MAX_THROUGHPUT ? out->cost > bound : 1.0 / out->iter_time < bound)
      out->mask |= SO_BIT_CONSTRAINT;
  }
  return 0;
}

/* The same with one TP degree for all stages. */
int so_eval_replica_assignment(const so_ctx *c, int pp_idx, int partition, int dp_idx, int mb_idx,
                               int tp_idx, const int32_t *pools, int objective, int has_bound,
                               double bound, so_eval *out) {
  int32_t all_stages[SO_MAX_STAGES];
  for (int i = 0; i < SO_MAX_STAGES; ++i) all_stages[i] = tp_idx;
  return so_eval_replica_assignment_tp(c, pp_idx, partition, dp_idx, mb_idx, all_stages, pools, objective,
                                       has_bound, bound, out);
}
