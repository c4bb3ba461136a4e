/* A plain C99 program that drives the planner through its C ABI (include/sailor.h): no
 * Python, no C++.  It builds a small planning problem by hand, evaluates every candidate
 * into device arrays, selects the best and the five best plans, replays them through the
 * event-by-event schedule and checks what must hold between those results.  Prints
 * "abi_example: OK" and exits 0 when everything does.
 *
 * Build (see tests/test_gpu_abi_example.py):
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude abi_example.c \
 *       -Lpaper_2504_17096_amd -lsailor -L/opt/rocm/lib -lamdhip64 -lm
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sailor.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "abi_example: line %d: %s\n", __LINE__, #cond);      \
      return 1;                                                            \
    }                                                                      \
  } while (0)

enum { L = 8, G = 2, Z = 2, MB = 2, TP = 2, DP = 3, PP = 3 };

int main(void) {
  /* job: 8 equal layers; type 1 is half as fast and half the price */
  static const int32_t mb_values[MB] = {1, 2}, tp_values[TP] = {1, 2}, dp_values[DP] = {1, 2, 4};
  static const int32_t pp_values[PP] = {1, 2, 4}, n_partitions[PP] = {1, 2, 1};
  static const int32_t partition_layers[] = {8, /* pp 1 */ 4, 4, 3, 5, /* pp 2: two splits */
                                             2, 2, 2, 2 /* pp 4 */};
  uint64_t layer_params[L];
  double t_fwd[G * MB * TP], t_bwd[G * MB * TP], t_upd[G * TP]; /* uniform_layers: one column */
  uint64_t act[MB * TP], p2p[MB];
  static const uint64_t cap[G] = {40ull << 30, 16ull << 30}, res[G] = {1ull << 30, 1ull << 30};
  static const int32_t node[G] = {8, 8};
  static const double price[G] = {3.0, 1.5};
  int32_t avail[Z * G] = {8, 16, 4, 8};
  static const double bw[Z * Z] = {1.0e10, 1.5e9, 1.0e9, 1.0e10};
  static const double egress[Z * Z] = {0.0, 2.0e-11, 3.0e-11, 0.0};
  for (int i = 0; i < L; ++i) layer_params[i] = 50u * 1000u * 1000u;
  for (int g = 0; g < G; ++g)
    for (int m = 0; m < MB; ++m)
      for (int k = 0; k < TP; ++k) {
        const double t = 2.0e-3 * (g + 1) * mb_values[m] / tp_values[k];
        t_fwd[(g * MB + m) * TP + k] = t;
        t_bwd[(g * MB + m) * TP + k] = 2.0 * t;
      }
  for (int g = 0; g < G; ++g)
    for (int k = 0; k < TP; ++k) t_upd[g * TP + k] = 1.0e-4 * (g + 1) / tp_values[k];
  for (int m = 0; m < MB; ++m) {
    p2p[m] = 4u * 1000u * 1000u * (uint64_t)mb_values[m];
    for (int k = 0; k < TP; ++k) act[m * TP + k] = 200u * 1000u * 1000u * (uint64_t)mb_values[m] / tp_values[k];
  }
  sailor_problem p;
  memset(&p, 0, sizeof p);
  p.n_layers = L; p.n_types = G; p.n_zones = Z; p.n_mb = MB; p.n_tp = TP; p.n_dp = DP; p.n_pp = PP;
  p.max_segments = 3; p.seg3_max_pp = 4; p.uniform_layers = 1; p.global_batch = 16;
  p.mb_values = mb_values; p.tp_values = tp_values; p.dp_values = dp_values; p.pp_values = pp_values;
  p.n_partitions = n_partitions; p.partition_layers = partition_layers;
  p.layer_params = layer_params; p.embed_params = 30u * 1000u * 1000u; p.head_params = 30u * 1000u * 1000u;
  p.bytes_per_param = 16; p.grad_bytes_per_param = 2;
  p.t_fwd = t_fwd; p.t_bwd = t_bwd; p.t_upd = t_upd;
  p.act_store_bytes = act; p.p2p_bytes = p2p; p.mem_capacity = cap; p.mem_reserved = res;
  p.gpus_per_node = node; p.price_per_hour = price; p.avail = avail; p.bandwidth = bw;
  p.egress_per_byte = egress;

  sailor_plan *plan = NULL;
  CHECK(sailor_plan_create(&p, &plan) == SAILOR_OK && plan != NULL);
  uint64_t n = 0;
  CHECK(sailor_plan_num_candidates(plan, &n) == SAILOR_OK && n > 1000 && n < 10000000);

  /* every candidate, into device arrays */
  float *d_time = NULL, *d_cost = NULL;
  uint64_t *d_mem = NULL;
  uint32_t *d_mask = NULL;
  CHECK(hipMalloc((void **)&d_time, n * sizeof(float)) == hipSuccess);
  CHECK(hipMalloc((void **)&d_cost, n * sizeof(float)) == hipSuccess);
  CHECK(hipMalloc((void **)&d_mem, n * sizeof(uint64_t)) == hipSuccess);
  CHECK(hipMalloc((void **)&d_mask, n * sizeof(uint32_t)) == hipSuccess);
  CHECK(sailor_eval_batch(plan, 0, n, NULL, SAILOR_MAX_THROUGHPUT, NULL, d_time, d_cost, d_mem,
                          d_mask, NULL) == SAILOR_OK);
  CHECK(hipDeviceSynchronize() == hipSuccess);
  float *h_time = (float *)malloc(n * sizeof(float)), *h_cost = (float *)malloc(n * sizeof(float));
  uint32_t *h_mask = (uint32_t *)malloc(n * sizeof(uint32_t));
  CHECK(h_time && h_cost && h_mask);
  CHECK(hipMemcpy(h_time, d_time, n * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(hipMemcpy(h_cost, d_cost, n * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(hipMemcpy(h_mask, d_mask, n * sizeof(uint32_t), hipMemcpyDeviceToHost) == hipSuccess);
  uint64_t n_valid = 0;
  double t_min = HUGE_VAL, c_min = HUGE_VAL;
  for (uint64_t i = 0; i < n; ++i)
    if (h_mask[i] == 0) {
      ++n_valid;
      if (h_time[i] < t_min) t_min = h_time[i];
      if (h_cost[i] < c_min) c_min = h_cost[i];
    }
  CHECK(n_valid > 10 && n_valid < n);

  /* the best plan agrees with the minimum over the evaluated space, and decodes to itself */
  sailor_result best, dec;
  CHECK(sailor_best_plan(plan, SAILOR_MAX_THROUGHPUT, NULL, &best, NULL) == SAILOR_OK);
  CHECK(best.mask == 0 && best.index < n && h_mask[best.index] == 0);
  CHECK(fabs(best.iter_time_s - t_min) <= 2e-5 * t_min);
  CHECK(fabs(best.iter_time_s - h_time[best.index]) <= 1e-5 * best.iter_time_s);
  CHECK(sailor_plan_decode(plan, best.index, &dec) == SAILOR_OK);
  CHECK(dec.pp == best.pp && dec.tp == best.tp && dec.dp == best.dp && dec.mb == best.mb &&
        dec.n_segments == best.n_segments && dec.pool[0] == best.pool[0] &&
        dec.zone[0] == best.zone[0] && dec.type_a[0] == best.type_a[0]);
  CHECK(best.pp * best.tp * best.dp >= 1 && best.dp * best.mb <= 16);

  /* the five cheapest plans that reach half of the best throughput, in ascending order */
  sailor_constraint floor_;
  floor_.bound = 0.5 / best.iter_time_s;
  floor_.has_bound = 1;
  sailor_result top[5];
  int32_t found = 0;
  CHECK(sailor_topk(plan, SAILOR_MIN_COST, &floor_, 5, top, &found, NULL) == SAILOR_OK && found == 5);
  for (int i = 0; i < 5; ++i) {
    CHECK(top[i].mask == 0 && 1.0 / top[i].iter_time_s >= floor_.bound);
    CHECK(fabs(top[i].cost_per_iter - h_cost[top[i].index]) <= 1e-5 * top[i].cost_per_iter);
    if (i) CHECK(top[i].cost_per_iter >= top[i - 1].cost_per_iter);
  }
  CHECK(top[0].cost_per_iter >= c_min * (1.0 - 1e-5));

  /* their 1F1B schedules, op by op, against the closed form the evaluator uses */
  uint64_t h_idx[5], *d_idx = NULL;
  double h_ev[5], h_cl[5], *d_ev = NULL, *d_cl = NULL;
  for (int i = 0; i < 5; ++i) h_idx[i] = top[i].index;
  CHECK(hipMalloc((void **)&d_idx, sizeof h_idx) == hipSuccess);
  CHECK(hipMalloc((void **)&d_ev, sizeof h_ev) == hipSuccess);
  CHECK(hipMalloc((void **)&d_cl, sizeof h_cl) == hipSuccess);
  CHECK(hipMemcpy(d_idx, h_idx, sizeof h_idx, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(sailor_simulate_1f1b(plan, 5, d_idx, d_ev, d_cl, NULL) == SAILOR_OK);
  CHECK(hipDeviceSynchronize() == hipSuccess);
  CHECK(hipMemcpy(h_ev, d_ev, sizeof h_ev, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(hipMemcpy(h_cl, d_cl, sizeof h_cl, hipMemcpyDeviceToHost) == hipSuccess);
  for (int i = 0; i < 5; ++i) {
    CHECK(h_ev[i] > 0.0 && h_cl[i] > 0.0 && h_cl[i] < top[i].iter_time_s * (1.0 + 1e-9));
    CHECK(h_cl[i] / h_ev[i] > 0.5 && h_cl[i] / h_ev[i] < 1.5);
  }

  /* a pool per stage: the search, with the enumerated space's best plan as the incumbent, finds a
   * plan that is no worse; the simulator for listed plans gives the same plan the same values,
   * also when every replica names its pool */
  sailor_search_options so;
  memset(&so, 0, sizeof so);
  so.beam_width = 32;
  so.use_incumbent = 2;
  static sailor_stage_plan sp;
  CHECK(sailor_search(plan, SAILOR_MAX_THROUGHPUT, NULL, &so, &sp, NULL) == SAILOR_OK);
  CHECK(sp.found == 1 && sp.mask == 0 && sp.incumbent_used == 1);
  CHECK(sp.iter_time_s <= best.iter_time_s * (1.0 + 2e-9) && sp.eval_time_s == sp.iter_time_s);
  {
    int32_t h_desc[5] = {sp.pp_index, sp.partition, sp.tp_index, sp.dp_index, sp.mb_index};
    int32_t *h_rep = (int32_t *)malloc(sizeof(int32_t) * (size_t)sp.pp * (size_t)sp.dp);
    CHECK(h_rep != NULL);
    for (int i = 0; i < sp.pp; ++i)
      for (int r = 0; r < sp.dp; ++r) h_rep[i * sp.dp + r] = sp.pool[i];
    int32_t *d_desc = NULL, *d_pool = NULL, *d_rep = NULL;
    double *d_two = NULL, h_two[2];
    CHECK(hipMalloc((void **)&d_desc, sizeof h_desc) == hipSuccess);
    CHECK(hipMalloc((void **)&d_pool, sizeof(int32_t) * (size_t)sp.pp) == hipSuccess);
    CHECK(hipMalloc((void **)&d_rep, sizeof(int32_t) * (size_t)sp.pp * (size_t)sp.dp) == hipSuccess);
    CHECK(hipMalloc((void **)&d_two, sizeof h_two) == hipSuccess);
    CHECK(hipMemcpy(d_desc, h_desc, sizeof h_desc, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_pool, sp.pool, sizeof(int32_t) * (size_t)sp.pp, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(d_rep, h_rep, sizeof(int32_t) * (size_t)sp.pp * (size_t)sp.dp, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(sailor_eval_placements(plan, 1, d_desc, d_pool, NULL, NULL, (uint32_t)sp.pp, SAILOR_MAX_THROUGHPUT, NULL,
                                 d_two, NULL, NULL, NULL, NULL) == SAILOR_OK);
    CHECK(sailor_eval_replica_placements(plan, 1, d_desc, d_rep, (uint64_t)sp.pp * (uint64_t)sp.dp, NULL, 0,
                                         SAILOR_MAX_THROUGHPUT, NULL, d_two + 1, NULL, NULL, NULL, NULL) == SAILOR_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(hipMemcpy(h_two, d_two, sizeof h_two, hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(h_two[0] == sp.iter_time_s && h_two[1] == sp.iter_time_s);
    hipFree(d_desc); hipFree(d_pool); hipFree(d_rep); hipFree(d_two);
    free(h_rep);
  }

  /* a re-plan with the minima of the last pass kept: the same answer as before for the same table */
  {
    sailor_result again;
    uint32_t evaluated = 0, units = 0;
    CHECK(sailor_plan_set_incremental(plan, 1) == SAILOR_OK);
    CHECK(sailor_best_plan(plan, SAILOR_MAX_THROUGHPUT, NULL, &again, NULL) == SAILOR_OK);
    CHECK(sailor_best_plan(plan, SAILOR_MAX_THROUGHPUT, NULL, &again, NULL) == SAILOR_OK);
    CHECK(again.index == best.index && again.iter_time_s == best.iter_time_s);
    CHECK(sailor_plan_last_scan(plan, &evaluated, &units) == SAILOR_OK && evaluated == 0 && units > 0);
    CHECK(sailor_plan_set_incremental(plan, 0) == SAILOR_OK);
  }

  /* no GPUs, no plan; errors are statuses, not crashes */
  memset(avail, 0, sizeof avail);
  CHECK(sailor_plan_set_avail(plan, avail) == SAILOR_OK);
  CHECK(sailor_best_plan(plan, SAILOR_MAX_THROUGHPUT, NULL, &best, NULL) == SAILOR_ENOFEASIBLE);
  CHECK(sailor_plan_decode(plan, n, &dec) == SAILOR_ERANGE);
  CHECK(sailor_topk(plan, SAILOR_MIN_COST, NULL, 0, top, &found, NULL) == SAILOR_EINVAL);

  CHECK(sailor_plan_destroy(plan) == SAILOR_OK);
  hipFree(d_time); hipFree(d_cost); hipFree(d_mem); hipFree(d_mask);
  hipFree(d_idx); hipFree(d_ev); hipFree(d_cl);
  free(h_time); free(h_cost); free(h_mask);
  printf("abi_example: OK (%llu candidates, %llu valid)\n", (unsigned long long)n,
         (unsigned long long)n_valid);
  return 0;
}
