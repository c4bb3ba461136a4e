// Host side of the C ABI declared in include/sailor.h: validation, upload, launches,
// decoding of winning indices.  No simulator arithmetic runs here.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/sailor.h"
#include "sailor_kernels.hip.h"
#include "sailor_search.hip.h"

using namespace sailor;

// Rings of sailor_simulate_1f1b_static: device memory that exists without any allocation call.
// Every GPU the library runs on holds its own copy at its own address until the process ends;
// in host code the array's name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[SAILOR_STATIC_SCRATCH_BYTES];

namespace {

constexpr uint32_t kDefaultSurvCap = 1u << 22;  // 96 MiB of survivors
constexpr uint32_t kDefaultRefCap = 1u << 18;
// candidates per scan workgroup: large enough to amortise the staging of a unit, small
// enough to leave about ten workgroups per compute unit
constexpr uint64_t kUnitTargetMin = 4096, kUnitTargetMax = 65536, kUnitsWanted = 2560;
constexpr uint32_t kCollectSub = 4;      // workgroups that share one unit in the collect pass
constexpr uint32_t kListSub = 8;         // the same when the pass walks a list of units,
constexpr uint32_t kListUnits = 256;     // and the units it visits per round
// A query whose constraint leaves at most this many units alive skips the scan: one pass
// keeps every valid candidate of those units (see run_selection_impl)
constexpr uint32_t kDirectUnits = 128;
constexpr uint32_t kDirectSub = 16;             // workgroups that share one of them
constexpr uint32_t kDirectManySurvivors = 8192;  // more than the select kernel holds in registers
                                                // (or than half the survivor buffer): the query
                                                // goes back to the scan from then on
// a scan unit that takes more than kSplitAbove x the average load of a workgroup slot (and
// kSplitAboveMean x the mean unit) is cut into parts of about kSplitTo x that load
constexpr double kSplitAbove = 0.9, kSplitAboveMean = 1.5, kSplitTo = 0.7, kSplitToMean = 1.1;
constexpr uint32_t kRankOneWorkgroup = 128;  // largest k whose final ranking runs as one workgroup
constexpr uint32_t kEvalUnitTarget = 16384;  // candidates per workgroup of the range evaluation
constexpr unsigned kEvalRowsThreads = 512;
constexpr size_t kEvalRowsMaxLds = 64 * 1024;  // above this the range form evaluates lane by lane
constexpr size_t kScanMaxLds = 160 * 1024;     // a scan workgroup stages its records within the LDS of a compute unit
constexpr size_t kSimMaxLds = 56 * 1024;       // rings of the event-by-event schedule beyond this
constexpr uint64_t kSimBatch = 64;             // live in device memory, for so many candidates at once

constexpr int kMaxDevices = 64;                // devices whose static scratch address is kept

#define HIP_TRY(expr)                                                              \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      std::fprintf(stderr, "sailor: %s failed: %s\n", #expr, hipGetErrorString(e_)); \
      return SAILOR_EDEVICE;                                                       \
    }                                                                              \
  } while (0)

std::atomic<void *> g_scratch_ptr[kMaxDevices];  // per device, looked up once
std::atomic<int> g_forced_unit_parts{0};         // sailor_set_scan_unit_parts

// The current device's copy of `scratch` (the device must be current).
sailor_status static_scratch(int device, double **out) {
  if (device < 0 || device >= kMaxDevices) return SAILOR_EINVAL;
  void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
  if (!p) {
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SAILOR_EDEVICE;
    g_scratch_ptr[device].store(p, std::memory_order_release);  // (racing threads store the same)
  }
  *out = static_cast<double *>(p);
  return SAILOR_OK;
}

struct DeviceArena {  // every device allocation of a plan, freed together
  std::vector<void *> ptrs;
  template <typename T>
  hipError_t alloc(T **out, size_t n) {
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, std::max<size_t>(n, 1) * sizeof(T));
    if (e == hipSuccess) ptrs.push_back(p);
    *out = static_cast<T *>(p);
    return e;
  }
  template <typename T>
  hipError_t upload(const T **out, const T *src, size_t n) {
    T *p = nullptr;
    hipError_t e = alloc(&p, n);
    if (e != hipSuccess) return e;
    *out = p;
    return n ? hipMemcpy(p, src, n * sizeof(T), hipMemcpyHostToDevice) : hipSuccess;
  }
  void free_one(void *p) {
    for (size_t i = 0; i < ptrs.size(); ++i)
      if (ptrs[i] == p) {
        (void)hipFree(p);
        ptrs.erase(ptrs.begin() + (long)i);
        return;
      }
  }
  void release() {
    for (void *p : ptrs) (void)hipFree(p);
    ptrs.clear();
  }
};

}  // namespace

struct sailor_plan {
  DevPlan dev{};
  DeviceArena arena;
  std::vector<ShapeRec> shapes;
  std::vector<BlockRec> blocks;
  std::vector<UnitRec> units;
  std::vector<EvalUnit> eunits;  // range evaluation, ascending idx_lo
  const EvalUnit *d_eunits = nullptr;
  size_t eval_lds_bytes = 0;
  std::vector<int32_t> mbv, tpv, dpv, ppv;
  std::vector<uint16_t> xt;        // real types a | b << 8 of every extended type
  int device = 0;
  size_t lds_bytes = 0;
  unsigned unit_threads = 256;
  uint32_t seq = 0;                // sequence number of the last selection's final kernel
  ResultHeader last_hdr{};         // of the last successful selection
  bool have_hdr = false;
  int32_t *d_avail = nullptr;
  int32_t *h_avail = nullptr;      // pinned staging of the availability table
  const int32_t *h_avail_dev = nullptr;  // the same memory as the device addresses it
  bool avail_dirty = false;        // h_avail is newer than the device copy
  bool upload_pending = false;     // an asynchronous upload from h_avail was enqueued
  hipEvent_t ev_upload = nullptr;
  // scratch of the selection pipeline
  float *umin_s = nullptr, *umin_l = nullptr;
  float *lb_time = nullptr, *lb_cost = nullptr;  // per unit: smallest time / cost with availability ignored
  // the units in ascending order of either bound (device), and the sorted bounds (host)
  uint32_t *order_time = nullptr, *order_cost = nullptr;
  std::vector<float> lb_time_sorted, lb_cost_sorted;
  // the last query whose direct pass kept too many candidates (it is not tried again)
  bool direct_declined = false;
  int declined_obj = 0;
  float declined_lim = 0.f;
  bool last_direct = false;       // the last successful selection took the direct pass
  uint32_t last_direct_units = 0; // over this many units
  uint32_t *counters = nullptr;
  uint32_t *ulist = nullptr;   // units the collect pass has to visit
  SurvRec *surv = nullptr;
  RefRec *ref = nullptr;
  uint32_t surv_cap = kDefaultSurvCap, ref_cap = kDefaultRefCap;
  // host-mapped result area: header + SAILOR_MAX_K records
  void *h_result = nullptr;
  ResultHeader *d_hdr = nullptr;
  RefRec *d_out = nullptr;
  RefRec *staged = nullptr;    // device-side copy of the top-k records before they go to the host
  // re-planning: per-unit minima of the last scan are kept while the query stays the same
  uint32_t *unit_gen = nullptr;   // device, per unit: availability generation of its minima
  uint32_t *unit_seq = nullptr;   // device, per unit: the call that evaluated it last
  uint32_t *ubits = nullptr;      // device, per unit: validity words as last staged
  uint32_t last_scan_seq = 0;     // call_seq of the last successful selection's scan
  uint32_t ubits_stride = 0;
  uint32_t avail_gen = 1;         // bumped whenever a new availability table reaches the device
  bool incremental = false;       // sailor_plan_set_incremental
  bool cache_ok = false;          // the minima on the device belong to the query below
  int cache_obj = 0, cache_hasb = 0;
  float cache_lim_s = 0.f, cache_lim_l = 0.f;
  bool last_incremental = false;  // the last successful selection reused minima
  // search over per-stage placements: tables and scratch, created by the first call
  std::vector<SearchPP> search_pps;
  const SearchPP *d_search_pps = nullptr;
  uint32_t n_sub = 0, n_sub_t = 0;  // sub-problems with TP in them / with a TP degree per stage
  uint8_t *search_states = nullptr;
  uint32_t search_wgs = 0, search_state_stride = 0, search_path_stride = 0;
  int search_beam_cap = 0;  // beam width the frontier buffers hold
  SubResult *search_results = nullptr, *search_final = nullptr;
  double *search_eval = nullptr;  // T, C, then (as 64-bit words) mem and mask of the winner
  uint32_t cnt_phase = 0;      // which of the two counter sets the next call uses
  bool counters_dirty = false; // a failed call may have left either set in any state
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};  // start, scan end, end, scan start
  int timing_mode = 0;         // 0 none, 1 dominant kernel, 2 dominant kernel + whole call
  bool total_timed = false, scan_timed = false;
};

namespace {

bool ascending_positive(const int32_t *v, int n) {
  if (!v || n < 1) return false;
  for (int i = 0; i < n; ++i) {
    if (v[i] < 1) return false;
    if (i && v[i] <= v[i - 1]) return false;
  }
  return true;
}

bool finite_nonneg(const double *v, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!(v[i] >= 0.0) || !std::isfinite(v[i])) return false;
  return true;
}

// types a segment can choose: the plain ones and, with mixed replicas, every pair of them
int extended_types(const sailor_problem *p) {
  return p->mixed_types ? p->n_types + p->n_types * (p->n_types - 1) / 2 : p->n_types;
}

uint64_t n_cut_choices(int P, int s);

sailor_status validate(const sailor_problem *p) {
  if (!p) return SAILOR_EINVAL;
  if (p->n_layers < 1 || p->n_types < 1 || p->n_zones < 1) return SAILOR_EINVAL;
  if (p->n_types > SAILOR_MAX_TYPES || p->n_zones > SAILOR_MAX_ZONES) return SAILOR_EINVAL;
  if (p->n_types * p->n_zones > SAILOR_MAX_POOLS) return SAILOR_EINVAL;
  if (p->n_mb < 1 || p->n_mb > SAILOR_MAX_MB || p->n_tp < 1 || p->n_tp > SAILOR_MAX_TP ||
      p->n_dp < 1 || p->n_dp > SAILOR_MAX_DP || p->n_pp < 1)
    return SAILOR_EINVAL;
  if (p->max_segments < 1 || p->max_segments > 3 || p->global_batch < 1) return SAILOR_EINVAL;
  if (p->per_segment_tp != 0 && p->per_segment_tp != 1) return SAILOR_EINVAL;
  if (p->mixed_types != 0 && p->mixed_types != 1) return SAILOR_EINVAL;
  if (p->n_zones * extended_types(p) > SAILOR_MAX_POOLS) return SAILOR_EINVAL;
  if (p->n_bw_coef < 0 || p->n_bw_coef > SAILOR_MAX_BW_COEF || (p->n_bw_coef > 0 && !p->bw_poly))
    return SAILOR_EINVAL;
  if (!ascending_positive(p->mb_values, p->n_mb) || !ascending_positive(p->tp_values, p->n_tp) ||
      !ascending_positive(p->dp_values, p->n_dp) || !ascending_positive(p->pp_values, p->n_pp))
    return SAILOR_EINVAL;
  if (!p->n_partitions || !p->partition_layers || !p->layer_params || !p->t_fwd || !p->t_bwd ||
      !p->t_upd || !p->act_store_bytes || !p->p2p_bytes || !p->mem_capacity || !p->mem_reserved ||
      !p->gpus_per_node || !p->price_per_hour || !p->avail || !p->bandwidth)
    return SAILOR_EINVAL;
  const int G = p->n_types, Z = p->n_zones, L = p->n_layers;
  size_t row = 0;
  for (int ip = 0; ip < p->n_pp; ++ip) {
    const int P = p->pp_values[ip];
    if (P > L || P > SAILOR_MAX_STAGES || p->n_partitions[ip] < 1) return SAILOR_EINVAL;
    for (int q = 0; q < p->n_partitions[ip]; ++q) {
      int64_t sum = 0;
      for (int i = 0; i < P; ++i) {
        const int32_t n = p->partition_layers[row++];
        if (n < 1) return SAILOR_EINVAL;
        sum += n;
      }
      if (sum != L) return SAILOR_EINVAL;
    }
  }
  {  // shapes (layer split x cut points) carry per-shape tables: keep their number bounded
    uint64_t n_shapes = 0;
    for (int ip = 0; ip < p->n_pp; ++ip)
      for (int s = 1; s <= p->max_segments; ++s) {
        const int P = p->pp_values[ip];
        if (s > P || (s == 3 && P > p->seg3_max_pp)) continue;
        n_shapes += n_cut_choices(P, s) * (uint64_t)p->n_partitions[ip];
        if (n_shapes > (uint64_t)SAILOR_MAX_SHAPES) return SAILOR_EINVAL;
      }
  }
  // the quota table has one row per GPU count a replica can take from a pool
  if ((int64_t)p->pp_values[p->n_pp - 1] * p->tp_values[p->n_tp - 1] > (1 << 20)) return SAILOR_EINVAL;
  const size_t Lc = p->uniform_layers ? 1 : (size_t)L;
  if (!finite_nonneg(p->t_fwd, (size_t)G * p->n_mb * p->n_tp * Lc) ||
      !finite_nonneg(p->t_bwd, (size_t)G * p->n_mb * p->n_tp * Lc) ||
      !finite_nonneg(p->t_upd, (size_t)G * p->n_tp * Lc) ||
      !finite_nonneg(p->price_per_hour, G))
    return SAILOR_EINVAL;
  for (int i = 0; i < Z * Z; ++i)
    if (!(p->bandwidth[i] > 0.0) || !std::isfinite(p->bandwidth[i])) return SAILOR_EINVAL;
  if (p->egress_per_byte && !finite_nonneg(p->egress_per_byte, (size_t)Z * Z)) return SAILOR_EINVAL;
  for (size_t i = 0; i < (size_t)Z * Z * p->n_bw_coef; ++i)
    if (!std::isfinite(p->bw_poly[i])) return SAILOR_EINVAL;
  for (int i = 0; i < Z * G; ++i)
    if (p->avail[i] < 0) return SAILOR_EINVAL;
  for (int g = 0; g < G; ++g)
    if (p->gpus_per_node[g] < 1) return SAILOR_EINVAL;
  // byte counts must stay far below 2^64: total parameters * bytes + the largest
  // activation term + reserved
  unsigned __int128 params = (unsigned __int128)p->embed_params + p->head_params;
  for (int l = 0; l < L; ++l) params += p->layer_params[l];
  uint64_t act_max = 0, res_max = 0;
  for (int i = 0; i < p->n_mb * p->n_tp; ++i) act_max = std::max(act_max, p->act_store_bytes[i]);
  for (int g = 0; g < G; ++g) res_max = std::max(res_max, p->mem_reserved[g]);
  unsigned __int128 worst = params * p->bytes_per_param +
                            (unsigned __int128)act_max * (unsigned)L * (unsigned)SAILOR_MAX_STAGES +
                            res_max;
  if (worst >> 62) return SAILOR_EINVAL;
  for (int g = 0; g < G; ++g)
    if (p->mem_capacity[g] >> 62) return SAILOR_EINVAL;
  for (int m = 0; m < p->n_mb; ++m)
    if (p->p2p_bytes[m] >> 53) return SAILOR_EINVAL;
  return SAILOR_OK;
}

uint64_t n_cut_choices(int P, int s) {
  if (s == 1) return 1;
  if (s == 2) return (uint64_t)(P - 1);
  return (uint64_t)(P - 1) * (uint64_t)(P - 2) / 2;
}

// Lays the candidate space out as blocks -> shapes -> scan units (host bookkeeping only).
sailor_status build_space(const sailor_problem *p, sailor_plan *pl, std::vector<int32_t> &st_n,
                          std::vector<int32_t> &st_first, std::vector<uint8_t> &st_flags) {
  const int ZG = extended_types(p) * p->n_zones;
  const uint64_t inner = (uint64_t)p->n_mb * p->n_tp * p->n_dp * ZG;
  const int pst = p->per_segment_tp ? 1 : 0;
  const uint64_t otp = pst ? (uint64_t)p->n_tp : 1u;  // radix of the tp digits of segments 2, 3
  uint64_t off = 0;
  uint32_t row_stage = 0;
  size_t row = 0;
  for (int ip = 0; ip < p->n_pp; ++ip) {
    const int P = p->pp_values[ip];
    const uint32_t row_stage0 = row_stage;
    for (int q = 0; q < p->n_partitions[ip]; ++q) {
      int first = 0;
      for (int i = 0; i < P; ++i) {
        const int32_t n = p->partition_layers[row++];
        st_n.push_back(n);
        st_first.push_back(first);
        st_flags.push_back((uint8_t)((i == 0 ? 1 : 0) | (i == P - 1 ? 2 : 0)));
        first += n;
      }
      row_stage += P;
    }
    for (int s = 1; s <= 3; ++s) {
      if (s > p->max_segments || s > P || (s == 3 && P > p->seg3_max_pp)) continue;
      uint64_t shape_size = inner;
      for (int j = 1; j < s; ++j) shape_size *= (uint64_t)(ZG - 1) * otp;
      if (shape_size == 0) continue;
      BlockRec b{};
      b.off = off;
      b.first_shape = (uint32_t)pl->shapes.size();
      b.shape_size = shape_size;
      b.pp_idx = ip;
      b.s = s;
      b.P = P;
      for (int q = 0; q < p->n_partitions[ip]; ++q)
        for (int k1 = (s >= 2 ? 1 : P); k1 <= (s >= 2 ? P - (s - 1) : P); ++k1)
          for (int k2 = (s == 3 ? k1 + 1 : P); k2 <= (s == 3 ? P - 1 : P); ++k2) {
            ShapeRec sh{};
            sh.base = off;
            sh.row_stage = row_stage0 + (uint32_t)q * P;
            sh.pp_idx = ip;
            sh.q = q;
            sh.P = (uint16_t)P;
            sh.s = (uint16_t)s;
            sh.k1 = (uint16_t)k1;
            sh.k2 = (uint16_t)k2;
            const int edges[4] = {0, k1, k2, P};
            for (int j = 0; j < 3; ++j) {
              sh.lo[j] = (uint16_t)(j < s ? edges[j] : 0);
              sh.n[j] = (uint16_t)(j < s ? edges[j + 1] - edges[j] : 0);
            }
            if (s == 1) sh.n[0] = (uint16_t)P;
            if (s == 2) sh.n[1] = (uint16_t)(P - k1);
            pl->shapes.push_back(sh);
            off += shape_size;
          }
      b.n_shapes = (uint32_t)pl->shapes.size() - b.first_shape;
      b.size = off - b.off;
      if (b.n_shapes != n_cut_choices(P, s) * (uint64_t)p->n_partitions[ip]) return SAILOR_EINVAL;
      pl->blocks.push_back(b);
    }
  }
  pl->dev.N = off;
  pl->dev.inner = (uint32_t)inner;
  pl->dev.n_row_stages = (int)row_stage;
  pl->dev.pst = pst;
  pl->dev.otp = (int)otp;
  pl->dev.stride3 = inner * (uint64_t)(ZG - 1) * otp;

  // scan units: (shape, tp of every segment, range of segment 2's pool)
  const uint64_t unit_target =
      std::min(kUnitTargetMax, std::max(kUnitTargetMin, pl->dev.N / kUnitsWanted));
  const uint64_t innerp = (uint64_t)p->n_mb * p->n_dp * ZG;
  for (uint32_t si = 0; si < pl->shapes.size(); ++si) {
    const ShapeRec &sh = pl->shapes[si];
    const int n_o = sh.s >= 2 ? ZG : 1;
    const uint64_t per_o = sh.s == 3 ? innerp * (uint64_t)(ZG - 1) : innerp;
    int chunk = (int)std::min<uint64_t>((uint64_t)n_o, std::max<uint64_t>(1, unit_target / per_o));
    const int n_chunks = (n_o + chunk - 1) / chunk;
    const int n_t1 = (pst && sh.s >= 2) ? p->n_tp : 1, n_t2 = (pst && sh.s == 3) ? p->n_tp : 1;
    for (int t2 = 0; t2 < n_t2; ++t2)
      for (int t1 = 0; t1 < n_t1; ++t1)
        for (int t = 0; t < p->n_tp; ++t)
          for (int c = 0; c < n_chunks; ++c) {
            const int lo = (int)((int64_t)n_o * c / n_chunks),
                      hi = (int)((int64_t)n_o * (c + 1) / n_chunks);
            UnitRec u{};
            u.shape = si;
            u.tp[0] = (uint8_t)t;
            u.tp[1] = (uint8_t)(pst ? t1 : t);
            u.tp[2] = (uint8_t)(pst ? t2 : t);
            u.s = (uint8_t)sh.s;
            u.o_lo = (uint16_t)lo;
            u.o_cnt = (uint16_t)(hi - lo);
            for (int j = 0; j < 3; ++j) u.n[j] = sh.n[j];
            u.part = 0;
            u.n_parts = 1;
            u.base = sh.base + (pst ? inner * (uint64_t)(ZG - 1) * (uint64_t)t1 +
                                          pl->dev.stride3 * (uint64_t)(ZG - 1) * (uint64_t)t2
                                    : 0u);
            pl->units.push_back(u);
          }
  }
  if (pl->units.size() > (size_t)0x7fffffff / kCollectSub) return SAILOR_EINVAL;
  // units of the range evaluation: (shape, range of the outer digits), about 16 Ki
  // candidates each, in index order
  for (uint32_t si = 0; si < pl->shapes.size(); ++si) {
    const ShapeRec &sh = pl->shapes[si];
    uint64_t o_total = 1;
    for (int j = 1; j < sh.s; ++j) o_total *= (uint64_t)(ZG - 1) * otp;
    const uint64_t chunk = std::min<uint64_t>(
        std::min<uint64_t>(o_total, kEvalUnitMaxOuter), std::max<uint64_t>(1, kEvalUnitTarget / inner));
    for (uint64_t lo = 0; lo < o_total; lo += chunk) {
      EvalUnit e{};
      e.shape = si;
      e.o_lo = (uint32_t)lo;
      e.o_cnt = (uint32_t)std::min<uint64_t>(chunk, o_total - lo);
      e.idx_lo = sh.base + lo * inner;
      pl->eunits.push_back(e);
    }
  }
  // Largest units first, so that the small ones fill the tail of the launch (the order is
  // refined by a timed pass once the tables are on the device).
  auto unit_cost = [&](const UnitRec &u) {  // candidates of the unit
    return innerp * (uint64_t)u.o_cnt * (u.s == 3 ? (uint64_t)(ZG - 1) : 1u);
  };
  std::stable_sort(pl->units.begin(), pl->units.end(),
                   [&](const UnitRec &a, const UnitRec &b) { return unit_cost(a) > unit_cost(b); });
  // Waves per workgroup: the lanes of a unit cover MB*DP*ZG triples in chunks of 64; pick
  // the wave count (2..8) that leaves the fewest idle wave slots in the last round.
  const uint64_t chunks = (innerp + 63) / 64;
  unsigned best_w = 4;
  double best_eff = 0.0;
  for (unsigned w = 2; w <= kMaxUnitThreads / 64; ++w) {
    const uint64_t rounds = (chunks + w - 1) / w;
    const double eff = (double)chunks / (double)(rounds * w);
    if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && w == 4)) { best_eff = eff; best_w = w; }
  }
  pl->unit_threads = best_w * 64;
  return SAILOR_OK;
}

sailor_status constraint_limits(sailor_objective obj, const sailor_constraint *c, int *has_bound,
                                double *bound, float *lim_s, float *lim_l) {
  *has_bound = (c && c->has_bound) ? 1 : 0;
  *bound = 0.0;
  *lim_s = *lim_l = kPosInf;
  if (!*has_bound) return SAILOR_OK;
  if (std::isnan(c->bound)) return SAILOR_EINVAL;
  *bound = c->bound;
  // the fp32 scan compares cost <= bound, or time <= 1 / bound (throughput floor)
  double lim = obj == SAILOR_MAX_THROUGHPUT ? c->bound : 1.0 / c->bound;
  if (obj == SAILOR_MIN_COST && c->bound <= 0.0) lim = HUGE_VAL;
  if (lim < 0.0) {
    *lim_s = *lim_l = -1.0f;  // nothing satisfies a negative cost bound
    return SAILOR_OK;
  }
  *lim_s = std::nextafterf((float)(lim * (1.0 - (double)kEvalEps)), 0.0f);
  *lim_l = std::nextafterf((float)(lim * (1.0 + (double)kEvalEps)), kPosInf);
  return SAILOR_OK;
}

void fill_config(const sailor_plan *pl, const ShapeRec &sh, uint64_t index, sailor_result *out) {
  const DevPlan &d = pl->dev;
  std::memset(out, 0, sizeof *out);
  out->index = index;
  const BlockRec *blk = &pl->blocks[0];
  for (const BlockRec &b : pl->blocks)
    if (index >= b.off) blk = &b;
  uint64_t rem = (index - blk->off) % blk->shape_size;
  const uint32_t in = (uint32_t)(rem % d.inner);
  uint32_t o = (uint32_t)(rem / d.inner);
  out->mb_index = in % d.MB;
  out->tp_index = (in / d.MB) % d.TP;
  out->dp_index = (in / (d.MB * d.TP)) % d.DP;
  out->pool[0] = in / (d.MB * d.TP * d.DP);
  out->pool[1] = out->pool[2] = -1;
  out->seg_tp_index[0] = out->tp_index;
  out->seg_tp_index[1] = out->seg_tp_index[2] = -1;
  if (sh.s >= 2) {
    out->pool[1] = (out->pool[0] + 1 + (int)(o % (d.ZG - 1))) % d.ZG;
    o /= (d.ZG - 1);
    out->seg_tp_index[1] = d.pst ? (int32_t)(o % d.TP) : out->tp_index;
    if (d.pst) o /= d.TP;
  }
  if (sh.s == 3) {
    out->pool[2] = (out->pool[1] + 1 + (int)(o % (d.ZG - 1))) % d.ZG;
    o /= (d.ZG - 1);
    out->seg_tp_index[2] = d.pst ? (int32_t)o : out->tp_index;
  }
  for (int j = 0; j < 3; ++j) {
    out->seg_tp[j] = out->seg_tp_index[j] >= 0 ? pl->tpv[out->seg_tp_index[j]] : 0;
    const bool used = out->pool[j] >= 0;
    out->zone[j] = used ? out->pool[j] / d.GX : -1;
    out->type_a[j] = used ? (pl->xt[out->pool[j] % d.GX] & 255) : -1;
    out->type_b[j] = used ? (pl->xt[out->pool[j] % d.GX] >> 8) : -1;
  }
  out->pp_index = sh.pp_idx;
  out->pp = sh.P;
  out->mb = pl->mbv[out->mb_index];
  out->tp = pl->tpv[out->tp_index];
  out->dp = pl->dpv[out->dp_index];
  out->partition = sh.q;
  out->n_segments = sh.s;
  out->cut[0] = sh.k1;
  out->cut[1] = sh.k2;
}

const ShapeRec &shape_of(const sailor_plan *pl, uint64_t index) {
  const BlockRec *blk = &pl->blocks[0];
  for (const BlockRec &b : pl->blocks)
    if (index >= b.off) blk = &b;
  return pl->shapes[blk->first_shape + (index - blk->off) / blk->shape_size];
}

unsigned quota_grid(const DevPlan &d) {
  const size_t n = std::max((size_t)(d.W_max + 1) * d.ZG, d.mixed ? (size_t)(2 * d.W_max + 1) * d.ZGr : 0);
  return (unsigned)std::min<size_t>(1024, (n + 255) / 256);
}

// Brings a changed availability table to the device on the caller's stream and rebuilds
// the quota table from it.
sailor_status refresh_avail(sailor_plan *pl, hipStream_t st) {
  if (!pl->avail_dirty) return SAILOR_OK;
  // the kernel reads the new table from the pinned staging buffer and leaves a copy on the
  // device (no separate upload in front of it)
  pl->avail_gen += 1;
  k_quota_table<<<quota_grid(pl->dev), 256, 0, st>>>(pl->dev, pl->h_avail_dev, pl->d_avail,
                                                      pl->avail_gen);
  HIP_TRY(hipEventRecord(pl->ev_upload, st));
  pl->upload_pending = true;
  pl->avail_dirty = false;
  return SAILOR_OK;
}

// Plain launch, or a launch whose own start / stop timestamps are recorded in two events.
template <typename K, typename... A>
void launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t e0,
            hipEvent_t e1, A... args) {
  if (e0) hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, e0, e1, 0, args...);
  else kernel<<<grid, block, lds, st>>>(args...);
}

template <int MODE, bool MIXED>
void launch_units_m(sailor_plan *pl, sailor_objective obj, int has_bound, const ScanArgs &a,
                    dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  if (obj == SAILOR_MAX_THROUGHPUT) {
    if (has_bound) launch(k_units<MODE, 0, true, MIXED>, grid, block, lds, st, e0, e1, pl->dev, a);
    else launch(k_units<MODE, 0, false, MIXED>, grid, block, lds, st, e0, e1, pl->dev, a);
  } else {
    if (has_bound) launch(k_units<MODE, 1, true, MIXED>, grid, block, lds, st, e0, e1, pl->dev, a);
    else launch(k_units<MODE, 1, false, MIXED>, grid, block, lds, st, e0, e1, pl->dev, a);
  }
}

template <int MODE>
void launch_units(sailor_plan *pl, sailor_objective obj, int has_bound, const ScanArgs &a,
                  hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  const unsigned n_units = (unsigned)pl->units.size();
  const dim3 grid(MODE == MODE_SCAN ? n_units
                  : a.direct        ? a.n_list_host * a.n_sub
                  : a.ulist         ? std::min(n_units, kListUnits) * a.n_sub
                                    : n_units * a.n_sub),
      block(pl->unit_threads);
  const size_t lds = pl->lds_bytes;
  if (pl->dev.mixed) launch_units_m<MODE, true>(pl, obj, has_bound, a, grid, block, lds, st, e0, e1);
  else launch_units_m<MODE, false>(pl, obj, has_bound, a, grid, block, lds, st, e0, e1);
}

// Shared by best_plan (k = 0: tolerance rule) and topk.
sailor_status run_selection_impl(sailor_plan *pl, sailor_objective obj,
                                 const sailor_constraint *con, uint32_t k, hipStream_t st,
                                 ResultHeader *hdr_out, bool allow_direct, bool *again) {
  int has_bound;
  double bound;
  ScanArgs sa{};
  sailor_status rc = constraint_limits(obj, con, &has_bound, &bound, &sa.lim_s, &sa.lim_l);
  if (rc != SAILOR_OK) return rc;
  HIP_TRY(hipSetDevice(pl->device));
  rc = refresh_avail(pl, st);
  if (rc != SAILOR_OK) return rc;
  if (pl->counters_dirty) {
    k_init_counters<<<1, 64, 0, st>>>(pl->counters, 2 * CNT_COUNT);
    pl->counters_dirty = false;
  }
  // two counter sets: this call's set was reset by the final kernel of the previous call
  uint32_t *cnt = pl->counters + pl->cnt_phase * CNT_COUNT;
  uint32_t *cnt_next = pl->counters + (pl->cnt_phase ^ 1u) * CNT_COUNT;
  pl->cnt_phase ^= 1u;
  sa.umin_s = pl->umin_s;
  sa.umin_l = pl->umin_l;
  sa.counters = cnt;
  sa.surv = pl->surv;
  sa.surv_cap = pl->surv_cap;
  sa.n_sub = kCollectSub;
  // a unit's minima of the last scan are reused when the query is the same and no quota row
  // the unit reads has changed since (the kernels compare generations per unit)
  sa.unit_gen = pl->unit_gen;
  sa.cur_gen = pl->avail_gen;
  sa.unit_seq = pl->unit_seq;
  sa.call_seq = pl->seq + 1;  // the sequence number this call's final kernel will publish
  sa.ubits = pl->incremental ? pl->ubits : nullptr;
  sa.ubits_stride = pl->ubits_stride;
  sa.incremental = (pl->incremental && pl->cache_ok && pl->cache_obj == (int)obj &&
                    pl->cache_hasb == has_bound && pl->cache_lim_s == sa.lim_s &&
                    pl->cache_lim_l == sa.lim_l) ? 1 : 0;
  const bool was_incremental = sa.incremental != 0;
  // (the constrained quantity is the cost when throughput is the objective, and the time otherwise)
  if (has_bound) sa.ulb_con = obj == SAILOR_MAX_THROUGHPUT ? pl->lb_cost : pl->lb_time;
  pl->cache_ok = false;  // until this call has succeeded
  pl->cache_obj = (int)obj;
  pl->cache_hasb = has_bound;
  pl->cache_lim_s = sa.lim_s;
  pl->cache_lim_l = sa.lim_l;
  const bool best = (k == 0);
  const uint32_t n_units = (uint32_t)pl->units.size();
  const bool t_scan = pl->timing_mode >= 1, t_all = pl->timing_mode >= 2;

  // collect -> [k-th smallest survivor key] -> fp64 refine -> final selection -> sync
  auto run_tail = [&](ResultHeader *hdr) -> sailor_status {
    // (a direct pass is the call's pass over the space: the scan's timing events ride on it)
    launch_units<MODE_COLLECT>(pl, obj, has_bound, sa, st, sa.direct && t_scan ? pl->ev[3] : nullptr,
                               sa.direct && t_scan ? pl->ev[1] : nullptr);
    RefineArgs ra{};
    ra.surv = pl->surv;
    ra.surv_cap = pl->surv_cap;
    ra.counters = cnt;
    ra.ref = pl->ref;
    ra.ref_cap = pl->ref_cap;
    ra.objective = (int)obj;
    ra.has_bound = has_bound;
    ra.bound = bound;
    ra.band = 1.0f + 3.0f * kEvalEps;
    if (!best || sa.direct) {
      // the exact k-th smallest fp32 key among the survivors, then only its neighbourhood
      // (best plan after a direct pass: the smallest key and its tie band -- what the collect
      // pass behind a scan gathers in the first place)
      k_select_kth<256><<<1, 256, 0, st>>>(&pl->surv[0].key, (int)(sizeof(SurvRec) / 4),
                                       cnt + CNT_SURV, pl->surv_cap, best ? 1u : k, cnt + CNT_TAU1,
                                       nullptr, 0u, 0.f, nullptr, nullptr);
      ra.tau_src = cnt + CNT_TAU1;
      if (best) ra.band = (float)(1.0 + kTieTol) + 3.0f * kEvalEps;
    }
    k_refine<<<256, kRefineWaves * 64, 0, st>>>(pl->dev, ra);
    if (best) {
      k_pick_best<<<1, 1024, 0, st>>>(pl->ref, pl->ref_cap, cnt, cnt_next, (int)obj, pl->d_hdr,
                                      pl->d_out, ++pl->seq);
    } else {
      // few records expected (about k, plus ties): one workgroup ranks them from LDS
      const bool one = k <= kRankOneWorkgroup;
      k_rank_topk<<<one ? 1 : 64, one ? kRankLds : 256, 0, st>>>(
          pl->ref, pl->ref_cap, cnt, cnt_next, (int)obj, k, pl->d_hdr, pl->d_out, pl->staged,
          cnt + CNT_DONE, ++pl->seq);
    }
    if (t_all) HIP_TRY(hipEventRecord(pl->ev[2], st));
    HIP_TRY(hipGetLastError());
    // Wait for the sequence number in host-mapped memory rather than for the dispatch to
    // retire; the stream is asked now and then, so that a failed launch cannot hang the wait.
    const volatile uint32_t *flag = &static_cast<ResultHeader *>(pl->h_result)->seq;
    for (uint32_t spins = 1; *flag != pl->seq; ++spins) {
      if ((spins & 0x3FFu) != 0) continue;
      const hipError_t q = hipStreamQuery(st);
      if (q == hipErrorNotReady) continue;
      HIP_TRY(q);
      if (*flag != pl->seq) return SAILOR_EDEVICE;  // the stream drained without a result
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    *hdr = *static_cast<ResultHeader *>(pl->h_result);
    return SAILOR_OK;
  };

  if (t_all) HIP_TRY(hipEventRecord(pl->ev[0], st));
  // A query whose constraint leaves only a few units alive (their bounds are sorted on the
  // host) needs no scan and no threshold: one pass over those units keeps every valid
  // candidate within the loose limit, and the usual tail -- the k-th smallest key among them
  // (the smallest, for the best plan), fp64 re-evaluation, ranking -- follows.  Not when minima are kept for later calls (this
  // pass produces none), and not for a query that kept too many candidates the last time.
  pl->last_direct = false;
  if (allow_direct && has_bound && !pl->incremental &&
      !(pl->direct_declined && pl->declined_obj == (int)obj && pl->declined_lim == sa.lim_l)) {
    const bool on_cost = obj == SAILOR_MAX_THROUGHPUT;
    const std::vector<float> &sorted_lb = on_cost ? pl->lb_cost_sorted : pl->lb_time_sorted;
    const size_t n_live = (size_t)(std::upper_bound(sorted_lb.begin(), sorted_lb.end(), sa.lim_l) -
                                   sorted_lb.begin());
    if (n_live > 0 && n_live <= kDirectUnits) {
      sa.direct = 1;
      sa.n_list_host = (uint32_t)n_live;
      sa.ulist = on_cost ? pl->order_cost : pl->order_time;
      sa.n_sub = kDirectSub;
      sa.use_tau_host = 1;
      sa.tau_host = kPosInf;
      rc = run_tail(hdr_out);
      if (rc != SAILOR_OK) return rc;
      pl->total_timed = t_all;
      pl->scan_timed = t_scan;
      if (hdr_out->surv_count > std::min(kDirectManySurvivors, pl->surv_cap / 2)) {
        pl->direct_declined = true;
        pl->declined_obj = (int)obj;
        pl->declined_lim = sa.lim_l;
      }
      if (hdr_out->surv_count > pl->surv_cap || hdr_out->ref_count > pl->ref_cap) {
        *again = true;  // more candidates than the buffers hold: the scan and its threshold decide
        return SAILOR_OK;
      }
      pl->last_direct = true;
      pl->last_direct_units = (uint32_t)n_live;
      pl->last_incremental = false;
      return SAILOR_OK;
    }
  }
  if (best) {
    // the scan itself lists the units that can hold a plan within the tie band of the
    // minimum (a superset: see ScanArgs), so the collect pass visits a handful of units
    // instead of asking every unit's workgroups
    sa.band = (float)(1.0 + kTieTol) + 3.0f * kEvalEps;
    // (not when minima are reused: units that are not evaluated again report at once, before
    // any running minimum exists, and nearly all of them would be listed)
    if (!sa.incremental) {
      sa.near_list = pl->ulist;
      sa.near_band = sa.band;
      // (minima kept for later calls must not depend on this call's running minimum)
      if (!pl->incremental) sa.ulb_key = obj == SAILOR_MAX_THROUGHPUT ? pl->lb_time : pl->lb_cost;
    }
  }
  launch_units<MODE_SCAN>(pl, obj, has_bound, sa, st, t_scan ? pl->ev[3] : nullptr,
                          t_scan ? pl->ev[1] : nullptr);
  const bool listed_by_scan = sa.near_list != nullptr;
  sa.near_list = nullptr;
  sa.ulb_key = nullptr;
  if (best && listed_by_scan) {
    sa.tau_src = cnt + CNT_GMIN;
    sa.ulist = pl->ulist;
    sa.n_sub = kListSub;
  } else if (best) {
    // the smallest strict unit minimum is the scan's minimum; the same kernel lists the units
    // whose loose minimum lies within the tie band of it
    k_select_kth<1024><<<1, 1024, 0, st>>>(pl->umin_s, 1, nullptr, n_units, 1u, cnt + CNT_TAU0,
                                     pl->umin_l, n_units, sa.band, pl->ulist, cnt + CNT_NLIST);
    sa.tau_src = cnt + CNT_TAU0;
    sa.ulist = pl->ulist;
    sa.n_sub = kListSub;
  } else {
    // an upper bound of the k-th smallest key: the k-th smallest unit minimum
    // (the same kernel lists the units whose loose minimum lies under it)
    sa.band = 1.0f + 3.0f * kEvalEps;
    k_select_kth<1024><<<1, 1024, 0, st>>>(pl->umin_s, 1, nullptr, n_units, k, cnt + CNT_TAU0,
                                     pl->umin_l, n_units, sa.band, pl->ulist, cnt + CNT_NLIST);
    sa.tau_src = cnt + CNT_TAU0;
    sa.ulist = pl->ulist;
    sa.n_sub = kListSub;
  }
  rc = run_tail(hdr_out);
  if (rc != SAILOR_OK) return rc;
  pl->total_timed = t_all;
  pl->scan_timed = t_scan;
  if (!best && hdr_out->surv_count > pl->surv_cap) {
    // The unit minima gave too loose a bound (few units hold valid plans, or none of them
    // strictly inside the constraint).  Search for a threshold that keeps at least k strict
    // candidates and fits the survivor buffer, with count-only collect passes: first
    // doubling up from the smallest key, then bisecting.
    const float gmin = __builtin_bit_cast(float, hdr_out->gmin_bits);
    if (!(gmin < kPosInf)) return SAILOR_ENOMEM;  // nothing strictly valid to anchor on
    sa.use_tau_host = 1;
    sa.count_only = 1;
    sa.ulist = nullptr;  // the list belongs to the first threshold
    sa.n_sub = kCollectSub;
    auto count_at = [&](float tau, uint32_t *n_loose, uint32_t *n_strict) -> sailor_status {
      k_zero_counters<<<1, 64, 0, st>>>(cnt, (1u << CNT_NLOOSE) | (1u << CNT_NSTRICT));
      sa.tau_host = tau;
      launch_units<MODE_COLLECT>(pl, obj, has_bound, sa, st, nullptr, nullptr);
      uint32_t two[2];
      HIP_TRY(hipMemcpyAsync(two, cnt + CNT_NLOOSE, sizeof two, hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      *n_loose = two[0];
      *n_strict = two[1];
      return SAILOR_OK;
    };
    double lo = (double)gmin, hi = 0.0;  // strict count < k at lo (or unknown), too many at hi
    float tau = 0.f;
    bool found = false;
    uint32_t nl = 0, ns = 0;
    for (int it = 0; it < 200 && !found; ++it) {
      double t;
      // doubling (from the smallest normal float when the minimum key is zero)
      if (hi == 0.0) t = (it == 0) ? lo * (1.0 + 1e-6) : std::max(lo * 2.0, 1.17549435e-38);
      else t = std::sqrt(lo * hi);                                            // bisecting
      if (!(t < 3.0e38)) break;
      tau = (float)t;
      rc = count_at(tau, &nl, &ns);
      if (rc != SAILOR_OK) return rc;
      if (nl > pl->surv_cap) hi = t;
      else if (ns >= k) found = true;
      else lo = t;
      if (hi != 0.0 && hi <= lo * (1.0 + 1e-7)) break;  // a wall of ties: give up
    }
    if (!found) return SAILOR_ENOMEM;
    k_zero_counters<<<1, 64, 0, st>>>(
        cnt, (1u << CNT_SURV) | (1u << CNT_REF) | (1u << CNT_FEAS) | (1u << CNT_DONE));
    sa.count_only = 0;
    sa.tau_host = tau;
    rc = run_tail(hdr_out);
    if (rc != SAILOR_OK) return rc;
  }
  pl->cache_ok = true;  // the scan completed: every unit's minima and stamp are in place
  pl->last_incremental = was_incremental;
  pl->last_scan_seq = sa.call_seq;
  if (hdr_out->surv_count > pl->surv_cap || hdr_out->ref_count > pl->ref_cap) return SAILOR_ENOMEM;
  return SAILOR_OK;
}

sailor_status run_selection(sailor_plan *pl, sailor_objective obj, const sailor_constraint *con,
                            uint32_t k, hipStream_t st, ResultHeader *hdr_out) {
  bool again = false;
  sailor_status rc = run_selection_impl(pl, obj, con, k, st, hdr_out, true, &again);
  if (rc == SAILOR_OK && again) rc = run_selection_impl(pl, obj, con, k, st, hdr_out, false, &again);
  if (rc == SAILOR_EDEVICE) pl->counters_dirty = true;
  if (rc == SAILOR_OK) { pl->last_hdr = *hdr_out; pl->have_hdr = true; }
  return rc;
}

void to_result(const sailor_plan *pl, const RefRec &r, sailor_result *out) {
  fill_config(pl, shape_of(pl, r.idx), r.idx, out);
  out->peak_mem_bytes = r.mem;
  out->iter_time_s = r.T;
  out->cost_per_iter = r.C;
  out->mask = r.mask;
}

}  // namespace

extern "C" {

sailor_status sailor_plan_destroy(sailor_plan *pl) {
  if (!pl) return SAILOR_OK;
  (void)hipSetDevice(pl->device);
  pl->arena.release();
  if (pl->h_result) (void)hipHostFree(pl->h_result);
  if (pl->h_avail) (void)hipHostFree(pl->h_avail);
  if (pl->ev_upload) (void)hipEventDestroy(pl->ev_upload);
  for (hipEvent_t e : pl->ev)
    if (e) (void)hipEventDestroy(e);
  delete pl;
  return SAILOR_OK;
}

// The body of sailor_plan_create.  *track holds the plan while this function owns it, so that
// the caller can release it when a container throws half-way.
static sailor_status create_impl(const sailor_problem *p, sailor_plan **out, sailor_plan **track) {
  if (!out) return SAILOR_EINVAL;
  sailor_status rc = validate(p);
  if (rc != SAILOR_OK) return rc;
  sailor_plan *pl = new (std::nothrow) sailor_plan();
  if (!pl) return SAILOR_ENOMEM;
  *track = pl;
  std::vector<int32_t> st_n, st_first;
  std::vector<uint8_t> st_flags;
  rc = build_space(p, pl, st_n, st_first, st_flags);
  if (rc != SAILOR_OK || pl->dev.N == 0) {
    *track = nullptr;
    delete pl;
    return rc != SAILOR_OK ? rc : SAILOR_EINVAL;
  }
  DevPlan &d = pl->dev;
  d.G = p->n_types; d.Z = p->n_zones;
  d.mixed = p->mixed_types ? 1 : 0;
  d.GX = extended_types(p);
  d.ZG = d.GX * d.Z;
  d.ZGr = d.G * d.Z;
  d.MB = p->n_mb; d.TP = p->n_tp; d.DP = p->n_dp;
  d.bpp = p->bytes_per_param; d.gb = p->grad_bytes_per_param; d.B = p->global_batch;
  d.n_blocks = (int)pl->blocks.size();
  d.n_shapes = (int)pl->shapes.size();
  d.n_units = (int)pl->units.size();
  for (int i = 0; i < d.MB; ++i) d.mbv[i] = p->mb_values[i];
  for (int i = 0; i < d.TP; ++i) d.tpv[i] = p->tp_values[i];
  for (int i = 0; i < d.DP; ++i) d.dpv[i] = p->dp_values[i];
  pl->mbv.assign(p->mb_values, p->mb_values + d.MB);
  pl->tpv.assign(p->tp_values, p->tp_values + d.TP);
  pl->dpv.assign(p->dp_values, p->dp_values + d.DP);
  pl->ppv.assign(p->pp_values, p->pp_values + p->n_pp);
  auto magic = [](uint32_t dv) { return dv == 1 ? 0u : (uint32_t)(((1ull << 32) + dv - 1) / dv); };
  d.mg_mb = magic((uint32_t)d.MB);
  d.mg_mbzg = magic((uint32_t)(d.MB * d.ZG));
  d.mg_mbzg1 = d.ZG > 1 ? magic((uint32_t)(d.MB * (d.ZG - 1))) : 0u;
  d.mg_g = magic((uint32_t)d.GX);
  d.mg_mbtp = magic((uint32_t)(d.MB * d.TP));
  d.mg_mbtpdp = magic((uint32_t)(d.MB * d.TP * d.DP));
  pl->eval_lds_bytes = (size_t)3 * d.TP * ((size_t)d.ZG * d.MB + 1) * sizeof(Rec) +
                       (size_t)d.MB * d.Z * d.Z * sizeof(float4) +
                       (size_t)3 * d.TP * d.MB * d.DP * sizeof(uint64_t) +
                       (size_t)3 * d.TP * d.ZG * sizeof(uint32_t) +
                       (size_t)d.ZG * (sizeof(PoolInfo) + 2 * sizeof(uint64_t)) +
                       (size_t)(kEvalUnitMaxOuter + d.DP + d.TP) * sizeof(uint32_t);
  pl->lds_bytes = unit_lds_records(d.ZG, d.MB) * (2 * sizeof(float4) + sizeof(uint32_t)) +
                  (size_t)d.MB * d.Z * d.Z * sizeof(float4) +
                  (size_t)d.ZG * (2 * sizeof(uint64_t) + sizeof(uint32_t));
  if (pl->lds_bytes > kScanMaxLds) {  // pools x microbatch sizes beyond what a workgroup can stage
    delete pl;
    *track = nullptr;
    return SAILOR_EINVAL;
  }

#define CREATE_TRY(expr)                                                           \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      std::fprintf(stderr, "sailor: %s failed: %s\n", #expr, hipGetErrorString(e_)); \
      *track = nullptr;                                                            \
      sailor_plan_destroy(pl);                                                     \
      return e_ == hipErrorOutOfMemory ? SAILOR_ENOMEM : SAILOR_EDEVICE;           \
    }                                                                              \
  } while (0)

  CREATE_TRY(hipGetDevice(&pl->device));
  DeviceArena &ar = pl->arena;
  const int G = d.G, GX = d.GX, Z = d.Z, ZG = d.ZG, ZGr = d.ZGr, MB = d.MB, TP = d.TP, DP = d.DP,
            L = p->n_layers;
  const size_t Lc = p->uniform_layers ? 1 : (size_t)L;
  const size_t RS = (size_t)d.n_row_stages, NS = pl->shapes.size();

  // inputs, copied as they are
  CREATE_TRY(ar.alloc(&pl->d_avail, ZGr));
  CREATE_TRY(hipMemcpy(pl->d_avail, p->avail, ZGr * sizeof(int32_t), hipMemcpyHostToDevice));
  d.avail = pl->d_avail;
  CREATE_TRY(hipHostMalloc(reinterpret_cast<void **>(&pl->h_avail), ZGr * sizeof(int32_t), 0));
  {
    void *dev_view = nullptr;
    CREATE_TRY(hipHostGetDevicePointer(&dev_view, pl->h_avail, 0));
    pl->h_avail_dev = static_cast<const int32_t *>(dev_view);
  }
  CREATE_TRY(hipEventCreateWithFlags(&pl->ev_upload, hipEventDisableTiming));
  d.P_max = 0;
  for (int ip = 0; ip < p->n_pp; ++ip) d.P_max = std::max(d.P_max, (int)p->pp_values[ip]);
  d.W_max = d.P_max * p->tp_values[TP - 1];
  CREATE_TRY(ar.alloc(&d.qw, (size_t)(d.W_max + 1) * ZG));
  if (d.mixed) CREATE_TRY(ar.alloc(&d.qh, (size_t)(2 * d.W_max + 1) * ZGr));
  CREATE_TRY(ar.alloc(&d.row_gen, 1));
  CREATE_TRY(hipMemset(d.row_gen, 0, sizeof(uint32_t)));
  CREATE_TRY(ar.alloc(&d.h1m, ZG));
  CREATE_TRY(ar.alloc(&d.isect, (size_t)2 * ZG));
  {
    std::vector<uint16_t> xt;
    for (int a = 0; a < G; ++a) xt.push_back((uint16_t)(a | (a << 8)));
    if (d.mixed)
      for (int a = 0; a < G; ++a)
        for (int b = a + 1; b < G; ++b) xt.push_back((uint16_t)(a | (b << 8)));
    pl->xt = xt;
    CREATE_TRY(ar.upload(&d.xt, xt.data(), xt.size()));
  }
  {
    std::vector<int32_t> vals(p->dp_values, p->dp_values + DP);
    vals.insert(vals.end(), p->tp_values, p->tp_values + TP);
    CREATE_TRY(ar.upload(&d.vals, vals.data(), vals.size()));
  }
  CREATE_TRY(ar.upload(&d.cap, p->mem_capacity, G));
  CREATE_TRY(ar.upload(&d.res, p->mem_reserved, G));
  CREATE_TRY(ar.upload(&d.node, p->gpus_per_node, G));
  CREATE_TRY(ar.upload(&d.price, p->price_per_hour, G));
  CREATE_TRY(ar.upload(&d.bw, p->bandwidth, (size_t)Z * Z));
  if (p->egress_per_byte) CREATE_TRY(ar.upload(&d.egress, p->egress_per_byte, (size_t)Z * Z));
  CREATE_TRY(ar.upload(&d.act, p->act_store_bytes, (size_t)MB * TP));
  CREATE_TRY(ar.upload(&d.p2p, p->p2p_bytes, MB));
  StageArgs sa{};
  CREATE_TRY(ar.upload(&sa.layer_params, p->layer_params, L));
  CREATE_TRY(ar.upload(&sa.t_fwd, p->t_fwd, (size_t)G * MB * TP * Lc));
  CREATE_TRY(ar.upload(&sa.t_bwd, p->t_bwd, (size_t)G * MB * TP * Lc));
  CREATE_TRY(ar.upload(&sa.t_upd, p->t_upd, (size_t)G * TP * Lc));
  CREATE_TRY(ar.upload(&sa.st_flags, st_flags.data(), RS));
  sa.embed = p->embed_params; sa.head = p->head_params; sa.L = L; sa.uniform = p->uniform_layers ? 1 : 0;
  CREATE_TRY(ar.upload(&d.st_n, st_n.data(), RS));
  CREATE_TRY(ar.upload(&d.st_first, st_first.data(), RS));
  CREATE_TRY(ar.upload(&d.shapes, pl->shapes.data(), NS));
  CREATE_TRY(ar.upload(&d.blocks, pl->blocks.data(), pl->blocks.size()));
  // per-unit tables: one entry per unit as laid out (units dropped later leave room for the
  // parts of units that are cut); sailor_set_scan_unit_parts(n) cuts every unit into n parts
  // whatever the timing says and needs n times the room
  const long forced_parts = g_forced_unit_parts.load(std::memory_order_relaxed);
  const size_t unit_cap = pl->units.size() * (size_t)std::max(1L, forced_parts);
  {
    UnitRec *d_units_new = nullptr;
    CREATE_TRY(ar.alloc(&d_units_new, unit_cap));
    CREATE_TRY(hipMemcpy(d_units_new, pl->units.data(), pl->units.size() * sizeof(UnitRec),
                         hipMemcpyHostToDevice));
    d.units = d_units_new;
  }
  CREATE_TRY(ar.upload(&pl->d_eunits, pl->eunits.data(), pl->eunits.size()));
  // derived tables, filled by the set-up kernels
  d.n_bw_coef = p->n_bw_coef;
  if (p->n_bw_coef > 0) CREATE_TRY(ar.upload(&d.bw_poly, p->bw_poly, (size_t)Z * Z * p->n_bw_coef));
  CREATE_TRY(ar.alloc(&d.bwp, (size_t)MB * Z * Z));
  CREATE_TRY(ar.alloc(&d.tsec_f, (size_t)MB * Z * Z));
  CREATE_TRY(ar.alloc(&d.egs_f, (size_t)Z * Z));
  CREATE_TRY(ar.alloc(&d.price_f, GX));
  CREATE_TRY(ar.alloc(&d.xb_f, MB));
  CREATE_TRY(ar.alloc(&d.cd_f, DP));
  CREATE_TRY(ar.alloc(&d.nbm1_f, (size_t)MB * DP));
  CREATE_TRY(ar.alloc(&d.dph_f, DP));
  CREATE_TRY(ar.alloc(&d.nb, (size_t)MB * DP));
  CREATE_TRY(ar.alloc(&d.divis, MB));
  CREATE_TRY(ar.alloc(&d.st_params, RS));
  CREATE_TRY(ar.alloc(&d.st_c, RS * G * MB * TP));
  CREATE_TRY(ar.alloc(&d.st_f, RS * G * MB * TP));
  CREATE_TRY(ar.alloc(&d.st_b, RS * G * MB * TP));
  CREATE_TRY(ar.alloc(&d.st_u, RS * G * TP));
  const size_t slots = NS * TP * 3;
  CREATE_TRY(ar.alloc(&d.ta, slots * GX * MB));
  CREATE_TRY(ar.alloc(&d.memok, slots * GX * MB));
  CREATE_TRY(ar.alloc(&d.need, slots * MB * DP));
  CREATE_TRY(ar.alloc(&d.syncz, slots * Z));
  CREATE_TRY(ar.alloc(&d.upd, slots * GX));
  // selection scratch
  CREATE_TRY(ar.alloc(&pl->umin_s, unit_cap));
  CREATE_TRY(ar.alloc(&pl->umin_l, unit_cap));
  CREATE_TRY(ar.alloc(&pl->lb_time, unit_cap));
  CREATE_TRY(ar.alloc(&pl->lb_cost, unit_cap));
  CREATE_TRY(ar.alloc(&pl->order_time, unit_cap));
  CREATE_TRY(ar.alloc(&pl->order_cost, unit_cap));
  CREATE_TRY(ar.alloc(&pl->counters, (size_t)2 * CNT_COUNT));
  CREATE_TRY(ar.alloc(&pl->ulist, unit_cap));
  CREATE_TRY(ar.alloc(&pl->unit_gen, unit_cap));
  CREATE_TRY(hipMemset(pl->unit_gen, 0, unit_cap * sizeof(uint32_t)));
  CREATE_TRY(ar.alloc(&pl->unit_seq, unit_cap));
  CREATE_TRY(hipMemset(pl->unit_seq, 0, unit_cap * sizeof(uint32_t)));
  pl->ubits_stride = (uint32_t)(unit_lds_records(ZG, MB) + (size_t)ZG);
  CREATE_TRY(ar.alloc(&pl->ubits, unit_cap * (size_t)pl->ubits_stride));
  CREATE_TRY(ar.alloc(&pl->surv, (size_t)pl->surv_cap));
  CREATE_TRY(ar.alloc(&pl->ref, (size_t)pl->ref_cap));
  CREATE_TRY(ar.alloc(&pl->staged, (size_t)SAILOR_MAX_K));
  const size_t res_bytes = sizeof(ResultHeader) + 8 + (size_t)SAILOR_MAX_K * sizeof(RefRec);
  CREATE_TRY(hipHostMalloc(&pl->h_result, res_bytes, hipHostMallocMapped));
  std::memset(pl->h_result, 0, res_bytes);
  void *d_res = nullptr;
  CREATE_TRY(hipHostGetDevicePointer(&d_res, pl->h_result, 0));
  pl->d_hdr = static_cast<ResultHeader *>(d_res);
  pl->d_out = reinterpret_cast<RefRec *>(static_cast<char *>(d_res) + sizeof(ResultHeader));
  for (hipEvent_t &e : pl->ev) CREATE_TRY(hipEventCreate(&e));

  k_init_counters<<<1, 64>>>(pl->counters, 2 * CNT_COUNT);
  k_quota_table<<<quota_grid(d), 256>>>(d, d.avail, nullptr, 0u);
  k_small_tables<<<1, 256>>>(d);
  k_stage_tables<<<(unsigned)RS, 128>>>(d, sa);
  k_shape_agg<<<(unsigned)NS, 256>>>(d);
  CREATE_TRY(hipGetLastError());
  CREATE_TRY(hipDeviceSynchronize());
  {
    // Two passes over the space order the scan.  With availability ignored, a unit whose
    // minimum is +inf holds no plan that memory, node size and batch divisibility allow,
    // whatever the availability becomes: it is dropped for good.  Units of equal size still
    // differ widely in cost, because invalid plans are pruned early, so a second pass
    // records how long each remaining unit takes; they are then launched longest first,
    // which also deals them evenly to the hardware's dispatch queues.
    size_t NU = pl->units.size();
    const size_t n_units_alloc = unit_cap;  // entries of the per-unit tables on the device
    float *d_cost = nullptr;
    CREATE_TRY(ar.alloc(&d_cost, unit_cap));
    ScanArgs ca{};
    ca.umin_s = pl->umin_s;
    ca.umin_l = pl->umin_l;
    ca.counters = pl->counters;
    ca.lim_s = ca.lim_l = kPosInf;
    ca.ignore_quota = 1;
    launch_units<MODE_SCAN>(pl, SAILOR_MAX_THROUGHPUT, 0, ca, nullptr, nullptr, nullptr);
    CREATE_TRY(hipGetLastError());
    std::vector<float> val(NU);
    CREATE_TRY(hipMemcpy(val.data(), pl->umin_s, NU * sizeof(float), hipMemcpyDeviceToHost));
    std::vector<UnitRec> kept;
    for (size_t i = 0; i < NU; ++i)
      if (val[i] < kPosInf) kept.push_back(pl->units[i]);
    if (kept.empty()) kept.push_back(pl->units[0]);  // launches need a non-empty grid
    pl->units.swap(kept);
    NU = pl->units.size();
    d.n_units = (int)NU;
    UnitRec *d_units = const_cast<UnitRec *>(d.units);
    CREATE_TRY(hipMemcpy(d_units, pl->units.data(), NU * sizeof(UnitRec), hipMemcpyHostToDevice));
    ca.ignore_quota = 0;
    ca.ucost = d_cost;
    launch_units<MODE_SCAN>(pl, SAILOR_MAX_THROUGHPUT, 0, ca, nullptr, nullptr, nullptr);
    CREATE_TRY(hipGetLastError());
    CREATE_TRY(hipMemcpy(val.data(), d_cost, NU * sizeof(float), hipMemcpyDeviceToHost));
    // With the longest units first the launch ends about when the average load of a
    // workgroup slot is done, unless a unit on its own takes longer than that: such a unit is
    // cut into parts -- every part keeps the unit's records and takes a share of its lane
    // space -- within the room the dropped units left in the tables, and the pass is timed
    // again.  (Cutting units that are merely above the mean costs more in staging than it
    // gains: spaces with far more units than slots ran 4 % slower that way.)
    {
      double total = 0.0;
      for (size_t i = 0; i < NU; ++i) total += val[i];
      const double mean = total / (double)NU;
      int per_cu = 0, cus = 0;
      const void *scan_kernel = d.mixed ? (const void *)k_units<MODE_SCAN, 0, true, true>
                                        : (const void *)k_units<MODE_SCAN, 0, true, false>;
      CREATE_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_kernel,
                                                              (int)pl->unit_threads, pl->lds_bytes));
      CREATE_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, pl->device));
      const double slots = (double)std::max(1, per_cu) * (double)std::max(1, cus);
      const double load = total / std::min((double)NU, slots);  // average load of a slot
      const double above = std::max(kSplitAbove * load, kSplitAboveMean * mean);
      const double target = std::max(kSplitTo * load, kSplitToMean * mean);
      const size_t waves = pl->unit_threads / 64;
      // 64-lane chunks of a unit's lane space (three segments: pool 1 skips segment 2's pool)
      const size_t chunks_of_unit = ((size_t)d.MB * d.DP * (size_t)std::max(1, d.ZG - 1) + 63) / 64;
      const size_t most = std::max<size_t>(1, std::min<size_t>(255, chunks_of_unit / waves));
      size_t room = n_units_alloc - NU;
      std::vector<UnitRec> cut;
      cut.reserve(n_units_alloc);
      for (size_t i = 0; i < NU; ++i) {
        UnitRec u = pl->units[i];
        size_t parts = 1;
        if (forced_parts > 0) parts = std::min<size_t>((size_t)forced_parts, room + 1);
        else if (val[i] > above)
          parts = std::min<size_t>({most, (size_t)std::ceil(val[i] / target), room + 1});
        u.n_parts = (uint8_t)parts;
        for (size_t c = 0; c < parts; ++c) {
          u.part = (uint8_t)c;
          cut.push_back(u);
        }
        room -= parts - 1;
      }
      if (cut.size() != NU) {
        pl->units.swap(cut);
        NU = pl->units.size();
        d.n_units = (int)NU;
        val.resize(NU);
        CREATE_TRY(hipMemcpy(d_units, pl->units.data(), NU * sizeof(UnitRec), hipMemcpyHostToDevice));
        launch_units<MODE_SCAN>(pl, SAILOR_MAX_THROUGHPUT, 0, ca, nullptr, nullptr, nullptr);
        CREATE_TRY(hipGetLastError());
        CREATE_TRY(hipMemcpy(val.data(), d_cost, NU * sizeof(float), hipMemcpyDeviceToHost));
      }
    }
    std::vector<uint32_t> order(NU);
    for (size_t i = 0; i < NU; ++i) order[i] = (uint32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t x, uint32_t y) { return val[x] > val[y]; });
    std::vector<UnitRec> sorted(NU);
    for (size_t i = 0; i < NU; ++i) sorted[i] = pl->units[order[i]];
    pl->units.swap(sorted);
    CREATE_TRY(hipMemcpy(d_units, pl->units.data(), NU * sizeof(UnitRec), hipMemcpyHostToDevice));
    // Per unit (in its final order), the smallest iteration time and the smallest cost over the
    // plans that do not depend on the availability: bounds that let a query pass over a unit.
    ca.ignore_quota = 1;
    ca.ucost = nullptr;
    launch_units<MODE_SCAN>(pl, SAILOR_MAX_THROUGHPUT, 0, ca, nullptr, nullptr, nullptr);
    CREATE_TRY(hipMemcpy(pl->lb_time, pl->umin_s, NU * sizeof(float), hipMemcpyDeviceToDevice));
    launch_units<MODE_SCAN>(pl, SAILOR_MIN_COST, 0, ca, nullptr, nullptr, nullptr);
    CREATE_TRY(hipMemcpy(pl->lb_cost, pl->umin_s, NU * sizeof(float), hipMemcpyDeviceToDevice));
    CREATE_TRY(hipGetLastError());
    // ... and the units sorted by either bound: the host then knows how many units a limit
    // leaves alive, and the device which
    for (int which = 0; which < 2; ++which) {
      CREATE_TRY(hipMemcpy(val.data(), which ? pl->lb_cost : pl->lb_time, NU * sizeof(float), hipMemcpyDeviceToHost));
      std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return val[x] < val[y]; });
      std::vector<float> &sorted_lb = which ? pl->lb_cost_sorted : pl->lb_time_sorted;
      sorted_lb.resize(NU);
      for (size_t i = 0; i < NU; ++i) sorted_lb[i] = val[order[i]];
      CREATE_TRY(hipMemcpy(which ? pl->order_cost : pl->order_time, order.data(), NU * sizeof(uint32_t),
                           hipMemcpyHostToDevice));
    }
    k_init_counters<<<1, 64>>>(pl->counters, 2 * CNT_COUNT);
    CREATE_TRY(hipDeviceSynchronize());
    ar.free_one(d_cost);
  }
#undef CREATE_TRY
  *track = nullptr;
  *out = pl;
  return SAILOR_OK;
}

sailor_status sailor_plan_create(const sailor_problem *p, sailor_plan **out) {
  sailor_plan *half_built = nullptr;
  try {  // no C++ exception crosses the C boundary
    return create_impl(p, out, &half_built);
  } catch (const std::bad_alloc &) {
    if (half_built) sailor_plan_destroy(half_built);
    return SAILOR_ENOMEM;
  } catch (...) {
    if (half_built) sailor_plan_destroy(half_built);
    return SAILOR_EINVAL;
  }
}

sailor_status sailor_plan_set_avail(sailor_plan *pl, const int32_t *avail) {
  if (!pl || !avail) return SAILOR_EINVAL;
  for (int i = 0; i < pl->dev.ZGr; ++i)
    if (avail[i] < 0) return SAILOR_EINVAL;
  HIP_TRY(hipSetDevice(pl->device));
  if (pl->upload_pending) {  // the staging buffer may still be read by an earlier upload
    HIP_TRY(hipEventSynchronize(pl->ev_upload));
    pl->upload_pending = false;
  }
  std::memcpy(pl->h_avail, avail, pl->dev.ZGr * sizeof(int32_t));
  pl->avail_dirty = true;  // uploaded, with the quota table, by the next call on its stream
  return SAILOR_OK;
}

sailor_status sailor_plan_num_candidates(const sailor_plan *pl, uint64_t *out) {
  if (!pl || !out) return SAILOR_EINVAL;
  *out = pl->dev.N;
  return SAILOR_OK;
}

sailor_status sailor_plan_decode(const sailor_plan *pl, uint64_t index, sailor_result *out) {
  if (!pl || !out) return SAILOR_EINVAL;
  if (index >= pl->dev.N) return SAILOR_ERANGE;
  fill_config(pl, shape_of(pl, index), index, out);
  return SAILOR_OK;
}

sailor_status sailor_eval_batch(sailor_plan *pl, uint64_t first, uint64_t count,
                                const uint64_t *d_indices, sailor_objective objective,
                                const sailor_constraint *constraint, float *d_time, float *d_cost,
                                uint64_t *d_mem, uint32_t *d_mask, void *hip_stream) {
  if (!pl || (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST))
    return SAILOR_EINVAL;
  if (!d_indices && (first > pl->dev.N || count > pl->dev.N - first)) return SAILOR_ERANGE;
  if (count > (uint64_t)0x7fffffff * 256) return SAILOR_ERANGE;
  if (constraint && constraint->has_bound && std::isnan(constraint->bound)) return SAILOR_EINVAL;
  if (count == 0) return SAILOR_OK;
  HIP_TRY(hipSetDevice(pl->device));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  {
    const sailor_status rc = refresh_avail(pl, st);
    if (rc != SAILOR_OK) return rc;
  }
  EvalArgs a{};
  a.first = first; a.count = count; a.indices = d_indices;
  a.time = d_time; a.cost = d_cost; a.mem = d_mem; a.mask = d_mask;
  a.objective = (int)objective;
  a.has_bound = (constraint && constraint->has_bound) ? 1 : 0;
  a.bound = a.has_bound ? (float)constraint->bound : 0.f;
  const bool timed = pl->timing_mode >= 1;
  if (!d_indices && pl->eval_lds_bytes <= kEvalRowsMaxLds) {
    // the units that intersect [first, first + count)
    auto end_of = [&](const EvalUnit &e) { return e.idx_lo + (uint64_t)e.o_cnt * pl->dev.inner; };
    size_t lo = 0, hi = pl->eunits.size();
    while (lo < hi) {  // first unit that ends after `first`
      const size_t mid = (lo + hi) / 2;
      if (end_of(pl->eunits[mid]) <= first) lo = mid + 1; else hi = mid;
    }
    const size_t u0 = lo;
    hi = pl->eunits.size();
    while (lo < hi) {  // first unit that starts at or after the end of the range
      const size_t mid = (lo + hi) / 2;
      if (pl->eunits[mid].idx_lo < first + count) lo = mid + 1; else hi = mid;
    }
    if (pl->dev.mixed)
      launch(k_eval_rows<true>, dim3((unsigned)(lo - u0)), dim3(kEvalRowsThreads), pl->eval_lds_bytes,
             st, timed ? pl->ev[3] : nullptr, timed ? pl->ev[1] : nullptr, pl->dev, a, pl->d_eunits,
             (uint32_t)u0);
    else
      launch(k_eval_rows<false>, dim3((unsigned)(lo - u0)), dim3(kEvalRowsThreads), pl->eval_lds_bytes,
             st, timed ? pl->ev[3] : nullptr, timed ? pl->ev[1] : nullptr, pl->dev, a, pl->d_eunits,
             (uint32_t)u0);
    HIP_TRY(hipGetLastError());
    pl->total_timed = false;
    pl->scan_timed = timed;
    return SAILOR_OK;
  }
  launch(k_eval_direct, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
         timed ? pl->ev[3] : nullptr, timed ? pl->ev[1] : nullptr, pl->dev, a);
  HIP_TRY(hipGetLastError());
  pl->total_timed = false;
  pl->scan_timed = timed;
  return SAILOR_OK;
}

sailor_status sailor_best_plan(sailor_plan *pl, sailor_objective objective,
                               const sailor_constraint *constraint, sailor_result *out,
                               void *hip_stream) {
  if (!pl || !out || (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST))
    return SAILOR_EINVAL;
  ResultHeader hdr;
  sailor_status rc = run_selection(pl, objective, constraint, 0,
                                   static_cast<hipStream_t>(hip_stream), &hdr);
  if (rc != SAILOR_OK) return rc;
  if (hdr.n_found == 0) return SAILOR_ENOFEASIBLE;
  const RefRec *rec = reinterpret_cast<const RefRec *>(static_cast<char *>(pl->h_result) +
                                                       sizeof(ResultHeader));
  to_result(pl, rec[0], out);
  return SAILOR_OK;
}

sailor_status sailor_topk(sailor_plan *pl, sailor_objective objective,
                          const sailor_constraint *constraint, int32_t k, sailor_result *out,
                          int32_t *n_found, void *hip_stream) {
  if (!pl || !out || !n_found || k < 1 || k > SAILOR_MAX_K ||
      (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST))
    return SAILOR_EINVAL;
  ResultHeader hdr;
  sailor_status rc = run_selection(pl, objective, constraint, (uint32_t)k,
                                   static_cast<hipStream_t>(hip_stream), &hdr);
  if (rc != SAILOR_OK) return rc;
  *n_found = (int32_t)hdr.n_found;
  if (hdr.n_found == 0) return SAILOR_ENOFEASIBLE;
  const RefRec *rec = reinterpret_cast<const RefRec *>(static_cast<char *>(pl->h_result) +
                                                       sizeof(ResultHeader));
  for (uint32_t i = 0; i < hdr.n_found; ++i) to_result(pl, rec[i], &out[i]);
  return SAILOR_OK;
}

sailor_status sailor_plan_set_scratch(sailor_plan *pl, uint32_t max_survivors,
                                      uint32_t max_refined) {
  if (!pl || max_survivors < 1 || max_refined < 1) return SAILOR_EINVAL;
  HIP_TRY(hipSetDevice(pl->device));
  HIP_TRY(hipDeviceSynchronize());
  SurvRec *surv = nullptr;
  RefRec *ref = nullptr;
  if (pl->arena.alloc(&surv, (size_t)max_survivors) != hipSuccess) return SAILOR_ENOMEM;
  if (pl->arena.alloc(&ref, (size_t)max_refined) != hipSuccess) {
    pl->arena.free_one(surv);
    return SAILOR_ENOMEM;
  }
  pl->arena.free_one(pl->surv);
  pl->arena.free_one(pl->ref);
  pl->surv = surv;
  pl->ref = ref;
  pl->surv_cap = max_survivors;
  pl->ref_cap = max_refined;
  return SAILOR_OK;
}

sailor_status sailor_plan_set_timing(sailor_plan *pl, int32_t mode) {
  if (!pl || mode < 0 || mode > 2) return SAILOR_EINVAL;
  pl->timing_mode = mode;
  pl->total_timed = pl->scan_timed = false;
  return SAILOR_OK;
}

sailor_status sailor_plan_last_timing(sailor_plan *pl, float *total_ms, float *kernel_ms) {
  if (!pl || (!pl->total_timed && !pl->scan_timed)) return SAILOR_EINVAL;
  float t = 0.f, s = 0.f;
  if (pl->scan_timed) {
    HIP_TRY(hipEventSynchronize(pl->ev[1]));
    HIP_TRY(hipEventElapsedTime(&s, pl->ev[3], pl->ev[1]));
  }
  if (pl->total_timed) {
    HIP_TRY(hipEventSynchronize(pl->ev[2]));
    HIP_TRY(hipEventElapsedTime(&t, pl->ev[0], pl->ev[2]));
  }
  if (total_ms) *total_ms = t;
  if (kernel_ms) *kernel_ms = s;
  return SAILOR_OK;
}

sailor_status sailor_simulate_1f1b(sailor_plan *pl, uint64_t count, const uint64_t *d_indices,
                                   double *d_event, double *d_closed, void *hip_stream) {
  if (!pl) return SAILOR_EINVAL;
  if (count == 0) return SAILOR_OK;
  if (!d_indices || (!d_event && !d_closed)) return SAILOR_EINVAL;
  if (count > 0x7fffffffu) return SAILOR_ERANGE;
  // microbatches per pipeline are counted in 32-bit integers
  if (pl->dev.B / ((int64_t)pl->dpv[0] * pl->mbv[0]) > (1 << 24)) return SAILOR_ERANGE;
  HIP_TRY(hipSetDevice(pl->device));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int p_max = pl->dev.P_max;
  int ring = 2;
  while (ring <= p_max) ring *= 2;
  const size_t ring_bytes = (size_t)2 * p_max * ring * sizeof(double);  // per candidate
  const unsigned threads = 64u * (unsigned)((p_max + 63) / 64);
  SimArgs a{};
  a.ring = ring;
  a.p_max = p_max;
  if (ring_bytes <= kSimMaxLds) {
    a.count = count;
    a.indices = d_indices;
    a.t_event = d_event;
    a.t_closed = d_closed;
    k_sim_1f1b<<<(unsigned)count, threads, ring_bytes, st>>>(pl->dev, a);
    HIP_TRY(hipGetLastError());
    return SAILOR_OK;
  }
  // deep pipelines: the rings do not fit LDS and live in device memory, a batch at a time
  const uint64_t batch = std::min<uint64_t>(count, kSimBatch);
  double *rings = nullptr;
  if (hipMalloc(reinterpret_cast<void **>(&rings), batch * ring_bytes) != hipSuccess)
    return SAILOR_ENOMEM;
  a.rings = rings;
  hipError_t err = hipSuccess;
  for (uint64_t off = 0; off < count && err == hipSuccess; off += batch) {
    a.count = std::min<uint64_t>(batch, count - off);
    a.indices = d_indices + off;
    a.t_event = d_event ? d_event + off : nullptr;
    a.t_closed = d_closed ? d_closed + off : nullptr;
    k_sim_1f1b<<<(unsigned)a.count, threads, 0, st>>>(pl->dev, a);
    err = hipGetLastError();
  }
  if (err == hipSuccess) err = hipStreamSynchronize(st);  // the rings are freed below
  (void)hipFree(rings);
  if (err != hipSuccess) {
    std::fprintf(stderr, "sailor: event schedule failed: %s\n", hipGetErrorString(err));
    return SAILOR_EDEVICE;
  }
  return SAILOR_OK;
}

sailor_status sailor_simulate_1f1b_static(sailor_plan *pl, uint64_t count, const uint64_t *d_indices,
                                          double *d_event, double *d_closed, void *hip_stream) {
  if (!pl) return SAILOR_EINVAL;
  if (count == 0) return SAILOR_OK;
  if (!d_indices || (!d_event && !d_closed)) return SAILOR_EINVAL;
  if (count > SAILOR_STATIC_MAX_PLANS) {
    std::fprintf(stderr, "sailor: sailor_simulate_1f1b_static takes at most %d plans per call (%llu given)\n",
                 (int)SAILOR_STATIC_MAX_PLANS, (unsigned long long)count);
    return SAILOR_ERANGE;
  }
  if (pl->dev.B / ((int64_t)pl->dpv[0] * pl->mbv[0]) > (1 << 24)) return SAILOR_ERANGE;
  const int p_max = pl->dev.P_max;
  int ring = 2;
  while (ring <= p_max) ring *= 2;
  const size_t ring_bytes = (size_t)2 * p_max * ring * sizeof(double);  // per plan
  if (ring_bytes > (size_t)SAILOR_STATIC_SCRATCH_BYTES) {
    std::fprintf(stderr, "sailor: the rings of one %d-stage pipeline (%zu bytes) exceed the static scratch\n",
                 p_max, ring_bytes);
    return SAILOR_ERANGE;
  }
  HIP_TRY(hipSetDevice(pl->device));
  double *rings = nullptr;
  const sailor_status rc = static_scratch(pl->device, &rings);
  if (rc != SAILOR_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const unsigned threads = 64u * (unsigned)((p_max + 63) / 64);
  const uint64_t batch = std::min<uint64_t>(count, (uint64_t)SAILOR_STATIC_SCRATCH_BYTES / ring_bytes);
  SimArgs a{};
  a.ring = ring;
  a.p_max = p_max;
  a.rings = rings;  // the batches follow one another on the stream and reuse the rings
  for (uint64_t off = 0; off < count; off += batch) {
    a.count = std::min<uint64_t>(batch, count - off);
    a.indices = d_indices + off;
    a.t_event = d_event ? d_event + off : nullptr;
    a.t_closed = d_closed ? d_closed + off : nullptr;
    k_sim_1f1b<<<(unsigned)a.count, threads, 0, st>>>(pl->dev, a);
    HIP_TRY(hipGetLastError());
  }
  return SAILOR_OK;
}

// tables of the search and of the placement evaluation (once per plan)
// (beam = 0: the tables only; beam > 0: also the search's buffers, its frontiers sized for the
// widest beam asked for so far)
static sailor_status search_setup(sailor_plan *pl, int beam) {
  if (!pl->d_search_pps) {
    pl->search_pps.clear();
    uint32_t sub = 0, sub_t = 0;
    for (size_t ip = 0; ip < pl->ppv.size(); ++ip) {
      SearchPP e{};
      e.P = pl->ppv[ip];
      e.n_part = 0;
      e.rs0 = 0;
      bool seen = false;
      for (const ShapeRec &sh : pl->shapes)
        if (sh.pp_idx == ip) {
          if (!seen || sh.row_stage < e.rs0) e.rs0 = sh.row_stage;
          seen = true;
          e.n_part = std::max(e.n_part, (int32_t)sh.q + 1);
        }
      if (!seen) return SAILOR_EINVAL;  // (every depth has a one-segment block)
      e.sub_off = sub;
      e.sub_off_t = sub_t;
      sub += (uint32_t)e.n_part * (uint32_t)(pl->dev.TP * pl->dev.DP * pl->dev.MB);
      sub_t += (uint32_t)e.n_part * (uint32_t)(pl->dev.DP * pl->dev.MB);
      pl->search_pps.push_back(e);
    }
    pl->n_sub = sub;
    pl->n_sub_t = sub_t;
    if (pl->arena.upload(&pl->d_search_pps, pl->search_pps.data(), pl->search_pps.size()) != hipSuccess)
      return SAILOR_ENOMEM;
  }
  if (beam > 0 && !pl->search_results) {
    SubResult *res = nullptr, *fin = nullptr;
    double *ev = nullptr;
    if (pl->arena.alloc(&res, (size_t)pl->n_sub) != hipSuccess || pl->arena.alloc(&fin, 1) != hipSuccess ||
        pl->arena.alloc(&ev, 4) != hipSuccess) {
      pl->arena.free_one(res);
      pl->arena.free_one(fin);
      pl->arena.free_one(ev);
      return SAILOR_ENOMEM;
    }
    if (hipMemset(fin, 0, sizeof(SubResult)) != hipSuccess) {  // (read by the winner's re-evaluation
      pl->arena.free_one(res);                                 // also when nothing was found)
      pl->arena.free_one(fin);
      pl->arena.free_one(ev);
      return SAILOR_EDEVICE;
    }
    pl->search_results = res;
    pl->search_final = fin;
    pl->search_eval = ev;
  }
  if (beam > pl->search_beam_cap) {
    // (no search is in flight on these buffers: every call waits for its own kernels)
    pl->arena.free_one(pl->search_states);
    pl->search_states = nullptr;
    pl->search_beam_cap = 0;
    pl->search_wgs = std::min<uint32_t>(pl->n_sub, 2048u);
    pl->search_path_stride = ((uint32_t)pl->dev.P_max + 7u) & ~7u;
    pl->search_state_stride = kStateBytes + 3 * pl->search_path_stride;  // pools, second pools, TP indices
    const size_t bytes = (size_t)pl->search_wgs * 2 * (size_t)beam * pl->search_state_stride;
    if (pl->arena.alloc(&pl->search_states, bytes) != hipSuccess) {
      pl->search_states = nullptr;
      return SAILOR_ENOMEM;
    }
    pl->search_beam_cap = beam;
  }
  return SAILOR_OK;
}

sailor_status sailor_eval_placements(sailor_plan *pl, uint64_t count, const int32_t *d_desc,
                                     const int32_t *d_pools, const int32_t *d_pools_b,
                                     const int32_t *d_tps, uint32_t pool_stride,
                                     sailor_objective objective, const sailor_constraint *constraint,
                                     double *d_time, double *d_cost, uint64_t *d_mem, uint32_t *d_mask,
                                     void *hip_stream) {
  if (!pl || (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST)) return SAILOR_EINVAL;
  if (count == 0) return SAILOR_OK;
  if (!d_desc || !d_pools || pool_stride < 1) return SAILOR_EINVAL;
  if (pl->dev.mixed || pl->dev.ZGr > kSearchMaxPools) return SAILOR_EINVAL;
  if (count > (uint64_t)0x7fffffff) return SAILOR_ERANGE;
  if (constraint && constraint->has_bound && std::isnan(constraint->bound)) return SAILOR_EINVAL;
  HIP_TRY(hipSetDevice(pl->device));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  sailor_status rc;
  try { rc = search_setup(pl, 0); } catch (...) { rc = SAILOR_ENOMEM; }
  if (rc != SAILOR_OK) return rc;
  rc = refresh_avail(pl, st);
  if (rc != SAILOR_OK) return rc;
  PlaceArgs a{};
  a.count = count; a.desc = d_desc; a.pools = d_pools; a.pools_b = d_pools_b; a.tps = d_tps;
  a.pool_stride = pool_stride;
  a.pps = pl->d_search_pps; a.n_pp = (int)pl->search_pps.size();
  a.objective = (int)objective;
  a.has_bound = (constraint && constraint->has_bound) ? 1 : 0;
  a.bound = a.has_bound ? constraint->bound : 0.0;
  a.T = d_time; a.C = d_cost; a.mem = d_mem; a.mask = d_mask;
  k_eval_placements<<<(unsigned)((count + kPlaceWaves - 1) / kPlaceWaves), kPlaceWaves * 64, 0, st>>>(pl->dev, a);
  HIP_TRY(hipGetLastError());
  return SAILOR_OK;
}

sailor_status sailor_eval_replica_placements(sailor_plan *pl, uint64_t count, const int32_t *d_desc,
                                             const int32_t *d_pools, uint64_t stride,
                                             const int32_t *d_tps, uint32_t tps_stride,
                                             sailor_objective objective,
                                             const sailor_constraint *constraint, double *d_time,
                                             double *d_cost, uint64_t *d_mem, uint32_t *d_mask,
                                             void *hip_stream) {
  if (!pl || (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST)) return SAILOR_EINVAL;
  if (count == 0) return SAILOR_OK;
  if (!d_desc || !d_pools || stride < 1 || (d_tps && tps_stride < 1)) return SAILOR_EINVAL;
  if (pl->dev.mixed || pl->dev.ZGr > kSearchMaxPools) return SAILOR_EINVAL;
  if (count > (uint64_t)0x7fffffff) return SAILOR_ERANGE;
  if (constraint && constraint->has_bound && std::isnan(constraint->bound)) return SAILOR_EINVAL;
  HIP_TRY(hipSetDevice(pl->device));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  sailor_status rc;
  try { rc = search_setup(pl, 0); } catch (...) { rc = SAILOR_ENOMEM; }
  if (rc != SAILOR_OK) return rc;
  rc = refresh_avail(pl, st);
  if (rc != SAILOR_OK) return rc;
  ReplicaArgs a{};
  a.count = count; a.desc = d_desc; a.pools = d_pools; a.stride = stride;
  a.tps = d_tps; a.tps_stride = tps_stride;
  a.pps = pl->d_search_pps; a.n_pp = (int)pl->search_pps.size();
  a.objective = (int)objective;
  a.has_bound = (constraint && constraint->has_bound) ? 1 : 0;
  a.bound = a.has_bound ? constraint->bound : 0.0;
  a.T = d_time; a.C = d_cost; a.mem = d_mem; a.mask = d_mask;
  k_eval_replicas<<<(unsigned)((count + kPlaceWaves - 1) / kPlaceWaves), kPlaceWaves * 64, 0, st>>>(pl->dev, a);
  HIP_TRY(hipGetLastError());
  return SAILOR_OK;
}

sailor_status sailor_search(sailor_plan *pl, sailor_objective objective,
                            const sailor_constraint *constraint, const sailor_search_options *opt,
                            sailor_stage_plan *out, void *hip_stream) {
  if (!pl || !opt || !out || (objective != SAILOR_MAX_THROUGHPUT && objective != SAILOR_MIN_COST))
    return SAILOR_EINVAL;
  if (opt->beam_width < 1 || opt->beam_width > kSearchMaxBeam || opt->max_runs < 0 ||
      opt->use_incumbent < 0 || opt->use_incumbent > 2)
    return SAILOR_EINVAL;
  if (opt->use_incumbent == 1 && std::isnan(opt->incumbent)) return SAILOR_EINVAL;
  if (opt->allow_split != 0 && opt->allow_split != 1) return SAILOR_EINVAL;
  if (opt->stage_tp != 0 && opt->stage_tp != 1) return SAILOR_EINVAL;
  // plain pools, constant link bandwidths, a pipeline's stages numbered in a byte
  if (pl->dev.mixed || pl->dev.n_bw_coef > 0 || pl->dev.ZGr > kSearchMaxPools ||
      pl->dev.P_max > kSearchMaxStages)
    return SAILOR_EINVAL;
  int has_bound;
  double bound;
  float lim_s, lim_l;
  sailor_status rc = constraint_limits(objective, constraint, &has_bound, &bound, &lim_s, &lim_l);
  if (rc != SAILOR_OK) return rc;
  HIP_TRY(hipSetDevice(pl->device));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  try { rc = search_setup(pl, opt->beam_width); } catch (...) { rc = SAILOR_ENOMEM; }
  if (rc != SAILOR_OK) return rc;
  SearchArgs a{};
  a.objective = (int)objective;
  a.has_bound = has_bound;
  a.bound = bound;
  a.W = opt->beam_width;
  a.max_runs = opt->max_runs;
  if (opt->use_incumbent == 1) {
    a.has_inc = 1;
    a.inc = opt->incumbent;
  } else if (opt->use_incumbent == 2) {
    // the best plan of the flat space (at most three contiguous runs) through the evaluator:
    // every placement whose bound exceeds its key can be dropped
    ResultHeader hdr;
    rc = run_selection(pl, objective, constraint, 0, st, &hdr);
    if (rc != SAILOR_OK) return rc;
    if (hdr.n_found) {
      const RefRec *rec = reinterpret_cast<const RefRec *>(static_cast<char *>(pl->h_result) + sizeof(ResultHeader));
      a.has_inc = 1;
      a.inc = (objective == SAILOR_MAX_THROUGHPUT ? rec[0].T : rec[0].C) * (1.0 + 1e-9);
    }
  }
  rc = refresh_avail(pl, st);
  if (rc != SAILOR_OK) return rc;
  a.pps = pl->d_search_pps;
  a.n_pp = (int)pl->search_pps.size();
  a.n_sub = opt->stage_tp ? pl->n_sub_t : pl->n_sub;
  a.states = pl->search_states;
  a.state_stride = pl->search_state_stride;
  a.path_stride = pl->search_path_stride;
  a.results = pl->search_results;
  const unsigned wgs = std::min<uint32_t>(pl->search_wgs, a.n_sub);
  if (opt->allow_split && opt->stage_tp) k_search_beam<SEARCH_SPLIT_TP><<<wgs, kSearchThreads, 0, st>>>(pl->dev, a);
  else if (opt->allow_split) k_search_beam<SEARCH_SPLIT><<<wgs, kSearchThreads, 0, st>>>(pl->dev, a);
  else if (opt->stage_tp) k_search_beam<SEARCH_STAGE_TP><<<wgs, kSearchThreads, 0, st>>>(pl->dev, a);
  else k_search_beam<SEARCH_PLAIN><<<wgs, kSearchThreads, 0, st>>>(pl->dev, a);
  k_search_pick<<<1, 256, 0, st>>>(pl->search_results, a.n_sub, pl->search_final);
  // the winner once more through the simulator, for its memory footprint and its mask
  PlaceArgs pa{};
  pa.count = 1;
  pa.one = pl->search_final;
  pa.pps = pl->d_search_pps;
  pa.n_pp = a.n_pp;
  pa.objective = (int)objective;
  pa.has_bound = has_bound;
  pa.bound = bound;
  pa.T = pl->search_eval;
  pa.C = pl->search_eval + 1;
  pa.mem = reinterpret_cast<uint64_t *>(pl->search_eval + 2);
  pa.mask = reinterpret_cast<uint32_t *>(pl->search_eval + 3);
  k_eval_placements<<<1, kPlaceWaves * 64, 0, st>>>(pl->dev, pa);
  HIP_TRY(hipGetLastError());
  SubResult fin;
  double ev[4];
  HIP_TRY(hipMemcpyAsync(&fin, pl->search_final, sizeof fin, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipMemcpyAsync(ev, pl->search_eval, sizeof ev, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  std::memset(out, 0, sizeof *out);
  for (int i = 0; i < SAILOR_MAX_STAGES; ++i) out->pool[i] = out->pool_b[i] = out->stage_tp_index[i] = -1;
  out->exact = fin.truncated ? 0 : 1;
  out->expanded = fin.expanded;
  out->incumbent_used = a.has_inc;
  out->incumbent = a.has_inc ? a.inc : 0.0;
  if (!fin.found) return SAILOR_ENOFEASIBLE;
  out->found = 1;
  out->pp_index = fin.desc[0];
  out->partition = fin.desc[1];
  out->tp_index = fin.desc[2];
  out->dp_index = fin.desc[3];
  out->mb_index = fin.desc[4];
  out->pp = pl->ppv[fin.desc[0]];
  out->tp = pl->tpv[fin.desc[2]];
  out->dp = pl->dpv[fin.desc[3]];
  out->mb = pl->mbv[fin.desc[4]];
  out->iter_time_s = fin.T;
  out->cost_per_iter = fin.C;
  out->eval_time_s = ev[0];
  out->eval_cost = ev[1];
  std::memcpy(&out->peak_mem_bytes, &ev[2], sizeof(uint64_t));
  std::memcpy(&out->mask, &ev[3], sizeof(uint32_t));
  for (int i = 0; i < out->pp; ++i) {
    out->pool[i] = fin.pools[i];
    out->pool_b[i] = fin.pools_b[i];
    out->stage_tp_index[i] = fin.tps[i];
  }
  return SAILOR_OK;
}

sailor_status sailor_set_scan_unit_parts(int32_t n) {
  if (n < 0 || n > 255) return SAILOR_EINVAL;
  g_forced_unit_parts.store(n, std::memory_order_relaxed);
  return SAILOR_OK;
}

sailor_status sailor_plan_set_incremental(sailor_plan *pl, int32_t on) {
  if (!pl || (on != 0 && on != 1)) return SAILOR_EINVAL;
  if (pl->incremental != (on != 0)) pl->cache_ok = false;  // what a scan keeps depends on it
  pl->incremental = on != 0;
  return SAILOR_OK;
}

sailor_status sailor_plan_last_scan(sailor_plan *pl, uint32_t *units_evaluated,
                                    uint32_t *units_total) {
  if (!pl || !pl->have_hdr) return SAILOR_EINVAL;
  const uint32_t total = (uint32_t)pl->units.size();
  if (units_evaluated) {
    if (pl->last_direct) {
      *units_evaluated = pl->last_direct_units;
    } else {
      // every unit carries the number of the call that evaluated it last; they are counted
      // here, off the selection's own path
      HIP_TRY(hipSetDevice(pl->device));
      uint32_t *seq = new (std::nothrow) uint32_t[total];
      if (!seq) return SAILOR_ENOMEM;
      const hipError_t e = hipMemcpy(seq, pl->unit_seq, total * sizeof(uint32_t), hipMemcpyDeviceToHost);
      uint32_t n = 0;
      for (uint32_t i = 0; i < total; ++i) n += seq[i] == pl->last_scan_seq ? 1u : 0u;
      delete[] seq;
      HIP_TRY(e);
      *units_evaluated = n;
    }
  }
  if (units_total) *units_total = total;
  return SAILOR_OK;
}

sailor_status sailor_plan_last_counts(const sailor_plan *pl, uint32_t *survivors,
                                      uint32_t *refined, uint32_t *feasible) {
  if (!pl || !pl->have_hdr) return SAILOR_EINVAL;
  if (survivors) *survivors = pl->last_hdr.surv_count;
  if (refined) *refined = pl->last_hdr.ref_count;
  if (feasible) *feasible = pl->last_hdr.feasible_count;
  return SAILOR_OK;
}

}  // extern "C"
