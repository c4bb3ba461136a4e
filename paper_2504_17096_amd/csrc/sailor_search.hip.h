// Search over per-stage placements (gfx950, wave64), on top of the tables of the evaluator.
//
// The planner assigns resources stage by stage (Sailor, Sec. 4.2.2, Eq. (1): stage i gets r,
// the stages behind it R - r, times composed by T_total); the heuristics H3 / H4 (Sec. 4.2.1)
// stop early when nothing better can follow.  Here every stage of a pipeline chooses its pool
// (zone, GPU type) freely -- all D replicas of a stage on that pool (H5), one TP degree per
// plan -- and one workgroup works through one sub-problem (pipeline depth, layer split, TP,
// D, microbatch size) level by level: the frontier of placements of stages 0 .. j-1 is
// extended by every pool for stage j, each extension gets a lower bound on T_iter and C_iter
// (Sec. 4.3) of all its completions, extensions whose bound breaks the constraint or exceeds
// an incumbent are dropped, and a frontier longer than the beam width keeps the smallest
// bounds.  At the last level the bound is the plan's own T_iter / C_iter.
//
// Two wider forms of a stage's choice: half of its replicas on a second pool (a, b), or its own
// TP degree (a, t) -- tp_ij of Sec. 4.2.2 taken per stage; TP then leaves the sub-problem and a
// pool's quota is counted in GPUs of one replica.
//
//   k_search_beam        the level-by-level expansion, one workgroup per sub-problem
//   k_search_pick        smallest (key, sub-problem) over the sub-problems' winners
//   k_eval_placements    the simulator of Sec. 4.3 for listed placements, one wave each, fp64
//   k_eval_replicas      the same for plans in which every replica of every stage names its pool
//
// All arithmetic is fp64 in a fixed order (sums in stage order), so that which extension is
// dropped or kept does not depend on how the work is spread over lanes.
#pragma once

#include <hip/hip_runtime.h>

#include "sailor_kernels.hip.h"

namespace sailor {

constexpr int kSearchThreads = 256;
constexpr int kSearchMaxBeam = 1024;   // longest frontier a sub-problem keeps (half of kSearchBuf at most)
constexpr int kSearchBuf = 2048;       // extensions buffered between two sorts
constexpr int kSearchMaxStages = 255;  // placements count stages per pool in a byte
constexpr int kSearchMaxPools = 64;

struct SearchPP {      // one pipeline depth
  int32_t P;
  uint32_t rs0;        // first entry of its first partition row in the stage tables
  uint32_t sub_off;    // first sub-problem of this depth
  int32_t n_part;
  uint32_t sub_off_t;  // the same when TP is not part of the sub-problem
  uint32_t pad[3];
};

enum : int { SEARCH_PLAIN = 0, SEARCH_SPLIT = 1, SEARCH_STAGE_TP = 2, SEARCH_SPLIT_TP = 3 };

struct SState {        // placement of stages 0 .. j; kStateBytes, followed by the paths (a byte per stage)
  double sum;          // times of the closed stages 0 .. j-1
  double maxt;         // slowest closed stage
  double c_open;       // compute time of stage j (its forward transfer is not known yet)
  double xb_open;      // its backward transfer to stage j-1
  double sum_b, maxt_b, c_open_b, xb_open_b;  // with split stages: the pipelines through the second pools
  double msync, mupd, dol, comm;
  uint16_t cnt[kSearchMaxPools];  // stages placed on each pool (split stages: halves of stages; a
                                  // TP degree per stage: GPUs of one replica)
  uint8_t pool, pool_b, runs, tpi, pad[4];  // tpi: the open stage's TP index (TP per stage)
};
constexpr uint32_t kStateBytes = sizeof(SState);
static_assert(kStateBytes == 232, "twelve doubles, the pool counts, pools, runs and TP index");

struct SubResult {     // winner of one sub-problem (or of the whole search)
  double key, T, C;
  uint32_t found, truncated;
  unsigned long long expanded;
  uint32_t sid, P;
  int32_t desc[6];     // pp index, partition, tp index, dp index, mb index, the search's mode
  int32_t pools[256];  // pool of every stage
  int32_t pools_b[256];  // pool of the other half of its replicas (= pools[i] when not split)
  int32_t tps[256];      // TP index of every stage (= desc[2] unless the stages choose their own)
};

struct SearchArgs {
  int objective, has_bound, has_inc, W, max_runs;
  double bound, inc;
  const SearchPP *pps;
  int n_pp;
  uint32_t n_sub;
  uint8_t *states;        // [workgroups][2][W] states of state_stride bytes
  uint32_t state_stride;  // kStateBytes + three paths of path_stride bytes (pools, second pools, TP indices)
  uint32_t path_stride;   // the deepest pipeline, rounded up to 8
  SubResult *results;     // [n_sub]
};

struct SBound { double T, C; };

// Lower bounds of T_iter and C_iter over the completions of a placement whose stage j is open;
// the plan's own values when j = P - 1 (then every S term is zero).
__device__ __forceinline__ SBound search_bounds(double sum, double maxt, double c_open, double xb_open,
                                                double msync, double mupd, double dol, double comm,
                                                double Ssum, double Smax, double Ssync, double Supd,
                                                double Sdol, double nbm1) {
  const double t_open = c_open + xb_open;
  const double tsum = (sum + t_open) + Ssum;
  const double tmax = fmax(fmax(maxt, t_open), Smax);
  SBound b;
  b.T = ((tsum + nbm1 * tmax) + fmax(msync, Ssync)) + fmax(mupd, Supd);
  b.C = (dol + Sdol) / 3600.0 * b.T + comm;
  return b;
}

__device__ __forceinline__ bool key_id_less(unsigned long long ka, uint32_t ia, unsigned long long kb,
                                            uint32_t ib) {
  return ka < kb || (ka == kb && ia < ib);
}

// Ascending bitonic sort of (key, id) pairs in LDS; m = the power of two >= n, entries
// n .. m-1 are filled with the largest pair first.
__device__ __forceinline__ void search_sort(unsigned long long *key, uint32_t *id, int n) {
  int m = 1;
  while (m < n) m <<= 1;
  for (int i = n + (int)threadIdx.x; i < m; i += blockDim.x) { key[i] = ~0ull; id[i] = ~0u; }
  __syncthreads();
  for (int k = 2; k <= m; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < m; i += blockDim.x) {
        const int x = i ^ j;
        if (x > i) {
          const bool up = (i & k) == 0;
          const unsigned long long ki = key[i], kx = key[x];
          const uint32_t ii = id[i], ix = id[x];
          const bool swap = up ? key_id_less(kx, ix, ki, ii) : key_id_less(ki, ii, kx, ix);
          if (swap) { key[i] = kx; key[x] = ki; id[i] = ix; id[x] = ii; }
        }
      }
      __syncthreads();
    }
}

struct SearchTables {  // LDS of a search workgroup: the sub-problem's and the level's tables
  double S[5][kSearchMaxStages + 1];   // what lies behind stage i: sum, max, sync, upd, $
  double xfer[kMaxZones][kMaxZones], comm[kMaxZones][kMaxZones];
  double comm_half[kMaxZones][kMaxZones];  // traffic of one kind of pipeline (half of the replicas)
  double bw[kMaxZones][kMaxZones], ring_price[kMaxZones][kMaxZones];
  double l_c[kMaxTypes], l_upd[kMaxTypes], l_dol[kMaxTypes], l_price[kMaxTypes], l_sync[kMaxZones];
  double l_ring;                       // bytes the level's stage's ring all-reduce moves over every link
  double smin[4][kSearchMaxStages + 1];  // cheapest admissible choice of every stage
  int cap[kSearchMaxPools];            // stages a pool can host
  int cap_half[kSearchMaxPools];       // halves of stages
  uint32_t l_fit;                      // bit g: the level's stage fits type g
  int dp_even;
  double dtp;                          // D * tp
  // a TP degree per stage: the level's stage on every type / zone at every degree
  double l_c3[kMaxTypes][kMaxTP], l_upd3[kMaxTypes][kMaxTP], l_dol3[kMaxTypes][kMaxTP];
  double l_sync3[kMaxZones][kMaxTP];
  uint32_t l_fit3[kMaxTP];             // bit g: the level's stage fits type g at this degree
  int tpv[kMaxTP];
  int cap_gpus[kSearchMaxPools];       // GPUs one replica can take from a pool
  // ... and two pools per stage as well
  double l_ring3[kMaxTP];              // the level's stage's ring bytes at every degree
  int cap_half_gpus[kSearchMaxPools];  // GPUs of one replica, counted once per half of a stage
  long long dp;                        // D
};

struct SAcc {          // what a placement carries besides its pool counts
  double sum, maxt, c_open, xb_open, sum_b, maxt_b, c_open_b, xb_open_b, msync, mupd, dol, comm;
};

// Stage j on pool a (split stages: half of its replicas on pool b, else b = a) at TP index k (a
// TP degree per stage; else the sub-problem's) behind the placement par (none for j = 0): may
// it be placed, and what the placement then carries.  The order of the operations is part of
// the definition: sums in stage order, a closed stage's transfers forward then backward.
template <int MODE>
__device__ __forceinline__ bool search_step(const SearchTables &T, const SState *par, int j, int a, int b,
                                            int k, int G, int max_runs, SAcc &o, int &runs) {
  constexpr bool SPLIT = MODE == SEARCH_SPLIT;
  if (MODE == SEARCH_SPLIT_TP) {
    const int ga = a % G, za = a / G, gb = b % G, zb = b / G, width = T.tpv[k];
    bool ok = ((T.l_fit3[k] >> ga) & 1u) != 0 && ((T.l_fit3[k] >> gb) & 1u) != 0;
    const int ca = par ? (int)par->cnt[a] : 0, cb = par ? (int)par->cnt[b] : 0;
    if (a == b) ok = ok && ca + 2 * width <= T.cap_half_gpus[a];
    else ok = ok && T.dp_even && ca + width <= T.cap_half_gpus[a] && cb + width <= T.cap_half_gpus[b];
    runs = par ? par->runs + ((a != par->pool || b != par->pool_b || k != par->tpi) ? 1 : 0) : 1;
    if (max_runs != 0 && runs > max_runs) ok = false;
    if (!ok) return false;
    double link = T.bw[za][za];
    if (zb != za) link = fmin(fmin(link, T.bw[zb][zb]), fmin(T.bw[za][zb], T.bw[zb][za]));
    const double sync = T.l_ring3[k] / link;
    const double upd = fmax(T.l_upd3[ga][k], T.l_upd3[gb][k]);
    const double dol = (double)(T.dp * (long long)width) * (0.5 * (T.l_price[ga] + T.l_price[gb]));
    const double ring = zb != za ? T.l_ring3[k] * T.ring_price[za][zb] : 0.0;
    o.c_open = T.l_c3[ga][k];
    o.c_open_b = T.l_c3[gb][k];
    if (!par) {
      o.sum = o.maxt = o.xb_open = o.sum_b = o.maxt_b = o.xb_open_b = 0.0;
      o.msync = sync; o.mupd = upd; o.dol = dol; o.comm = ring;
    } else {
      const int pza = par->pool / G, pzb = par->pool_b / G;
      const double ta = par->c_open + (T.xfer[pza][za] + par->xb_open);  // forward, then backward
      const double tb = par->c_open_b + (T.xfer[pzb][zb] + par->xb_open_b);
      o.sum = par->sum + ta;
      o.maxt = fmax(par->maxt, ta);
      o.sum_b = par->sum_b + tb;
      o.maxt_b = fmax(par->maxt_b, tb);
      o.xb_open = T.xfer[za][pza];
      o.xb_open_b = T.xfer[zb][pzb];
      o.msync = fmax(par->msync, sync);
      o.mupd = fmax(par->mupd, upd);
      o.dol = par->dol + dol;
      double comm = par->comm;
      if (pza != za) comm += T.comm_half[pza][za];
      if (pzb != zb) comm += T.comm_half[pzb][zb];
      o.comm = comm + ring;
    }
    return true;
  }
  if (MODE == SEARCH_STAGE_TP) {
    const int g = a % G, z = a / G, t = k;
    bool ok = ((T.l_fit3[t] >> g) & 1u) != 0;
    const int used = par ? (int)par->cnt[a] : 0;
    ok = ok && used + T.tpv[t] <= T.cap_gpus[a];
    runs = par ? par->runs + ((a != par->pool || t != par->tpi) ? 1 : 0) : 1;
    if (max_runs != 0 && runs > max_runs) ok = false;
    if (!ok) return false;
    o.c_open = T.l_c3[g][t];
    if (!par) {
      o.sum = 0.0; o.maxt = 0.0; o.xb_open = 0.0; o.msync = T.l_sync3[z][t]; o.mupd = T.l_upd3[g][t];
      o.dol = T.l_dol3[g][t]; o.comm = 0.0;
    } else {
      const int pz = par->pool / G;
      const double t_closed = par->c_open + (T.xfer[pz][z] + par->xb_open);  // forward, then backward
      o.sum = par->sum + t_closed;
      o.maxt = fmax(par->maxt, t_closed);
      o.xb_open = T.xfer[z][pz];
      o.msync = fmax(par->msync, T.l_sync3[z][t]);
      o.mupd = fmax(par->mupd, T.l_upd3[g][t]);
      o.dol = par->dol + T.l_dol3[g][t];
      o.comm = pz != z ? par->comm + T.comm[pz][z] : par->comm;
    }
    o.sum_b = o.maxt_b = o.c_open_b = o.xb_open_b = 0.0;
    return true;
  }
  const int ga = a % G, za = a / G, gb = b % G, zb = b / G;
  bool ok = ((T.l_fit >> ga) & 1u) != 0 && ((T.l_fit >> gb) & 1u) != 0;
  const int ca = par ? (int)par->cnt[a] : 0, cb = par ? (int)par->cnt[b] : 0;
  if (!SPLIT) ok = ok && ca + 1 <= T.cap[a];
  else if (a == b) ok = ok && ca + 2 <= T.cap_half[a];
  else ok = ok && T.dp_even && ca + 1 <= T.cap_half[a] && cb + 1 <= T.cap_half[b];
  runs = par ? par->runs + ((a != par->pool || (SPLIT && b != par->pool_b)) ? 1 : 0) : 1;
  if (max_runs != 0 && runs > max_runs) ok = false;
  if (!ok) return false;
  if (!SPLIT) {
    o.c_open = T.l_c[ga];
    if (!par) {
      o.sum = 0.0; o.maxt = 0.0; o.xb_open = 0.0; o.msync = T.l_sync[za]; o.mupd = T.l_upd[ga];
      o.dol = T.l_dol[ga]; o.comm = 0.0;
    } else {
      const int pz = par->pool / G;
      const double t_closed = par->c_open + (T.xfer[pz][za] + par->xb_open);  // forward, then backward
      o.sum = par->sum + t_closed;
      o.maxt = fmax(par->maxt, t_closed);
      o.xb_open = T.xfer[za][pz];
      o.msync = fmax(par->msync, T.l_sync[za]);
      o.mupd = fmax(par->mupd, T.l_upd[ga]);
      o.dol = par->dol + T.l_dol[ga];
      o.comm = pz != za ? par->comm + T.comm[pz][za] : par->comm;
    }
    o.sum_b = o.maxt_b = o.c_open_b = o.xb_open_b = 0.0;
    return true;
  }
  // the stage by itself: all-reduce over the slowest link of a ring through both pools, the
  // slower update, the mean rent, the ring's traffic between the zones
  double link = T.bw[za][za];
  if (zb != za) link = fmin(fmin(link, T.bw[zb][zb]), fmin(T.bw[za][zb], T.bw[zb][za]));
  const double sync = T.l_ring / link;
  const double upd = fmax(T.l_upd[ga], T.l_upd[gb]);
  const double dol = T.dtp * (0.5 * (T.l_price[ga] + T.l_price[gb]));
  const double ring = zb != za ? T.l_ring * T.ring_price[za][zb] : 0.0;
  o.c_open = T.l_c[ga];
  o.c_open_b = T.l_c[gb];
  if (!par) {
    o.sum = o.maxt = o.xb_open = o.sum_b = o.maxt_b = o.xb_open_b = 0.0;
    o.msync = sync; o.mupd = upd; o.dol = dol; o.comm = ring;
  } else {
    const int pza = par->pool / G, pzb = par->pool_b / G;
    const double ta = par->c_open + (T.xfer[pza][za] + par->xb_open);
    const double tb = par->c_open_b + (T.xfer[pzb][zb] + par->xb_open_b);
    o.sum = par->sum + ta;
    o.maxt = fmax(par->maxt, ta);
    o.sum_b = par->sum_b + tb;
    o.maxt_b = fmax(par->maxt_b, tb);
    o.xb_open = T.xfer[za][pza];
    o.xb_open_b = T.xfer[zb][pzb];
    o.msync = fmax(par->msync, sync);
    o.mupd = fmax(par->mupd, upd);
    o.dol = par->dol + dol;
    double comm = par->comm;
    if (pza != za) comm += T.comm_half[pza][za];
    if (pzb != zb) comm += T.comm_half[pzb][zb];
    o.comm = comm + ring;
  }
  return true;
}

// Bounds of a placement whose stage j is open; with split stages the slower of the two kinds
// of pipeline counts (Sec. 4.3).
template <int MODE>
__device__ __forceinline__ SBound search_bound_of(const SearchTables &T, const SAcc &o, int j, double nbm1) {
  if (MODE != SEARCH_SPLIT && MODE != SEARCH_SPLIT_TP)
    return search_bounds(o.sum, o.maxt, o.c_open, o.xb_open, o.msync, o.mupd, o.dol, o.comm, T.S[0][j],
                         T.S[1][j], T.S[2][j], T.S[3][j], T.S[4][j], nbm1);
  const double ta = o.c_open + o.xb_open, tb = o.c_open_b + o.xb_open_b;
  const double pa = ((o.sum + ta) + T.S[0][j]) + nbm1 * fmax(fmax(o.maxt, ta), T.S[1][j]);
  const double pb = ((o.sum_b + tb) + T.S[0][j]) + nbm1 * fmax(fmax(o.maxt_b, tb), T.S[1][j]);
  SBound b;
  b.T = (fmax(pa, pb) + fmax(o.msync, T.S[2][j])) + fmax(o.mupd, T.S[3][j]);
  b.C = (o.dol + T.S[4][j]) / 3600.0 * b.T + o.comm;
  return b;
}

template <int MODE>
__global__ __launch_bounds__(kSearchThreads) void k_search_beam(DevPlan pl, SearchArgs a) {
  constexpr bool BOTH = MODE == SEARCH_SPLIT_TP;
  constexpr bool SPLIT = MODE == SEARCH_SPLIT || BOTH;     // two pools per stage
  constexpr bool STP = MODE == SEARCH_STAGE_TP || BOTH;    // a TP degree per stage
  __shared__ SearchTables T;
  __shared__ unsigned long long b_key[kSearchBuf];
  __shared__ uint32_t b_id[kSearchBuf];
  __shared__ uint32_t s_wave[kSearchThreads / 64];
  __shared__ int s_nbuf, s_bad;
  __shared__ unsigned long long s_bk[kSearchThreads / 64];
  __shared__ uint32_t s_bi[kSearchThreads / 64];
  __shared__ unsigned long long s_expanded;
  __shared__ unsigned char s_fit3[kMaxTypes][kMaxTP];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const int G = pl.G, Z = pl.Z, ZG = pl.ZGr, MB = pl.MB, TP = pl.TP, DP = pl.DP;
  // choices per stage: a pool; a pair (a, b) = a * ZG + b; a pool and a TP index (a, t) = a * TP + t;
  // a pair and a TP index ((a * ZG + b) * TP + t)
  const int NCH = BOTH ? ZG * ZG * TP : (SPLIT ? ZG * ZG : (STP ? ZG * TP : ZG));
  // a choice c -> first pool, second pool (= the first without split stages), TP index
  auto choice = [&](int c, int it0, int &ca, int &cb, int &ck) {
    ck = STP ? c % TP : it0;
    const int pools = STP ? c / TP : c;
    ca = SPLIT ? pools / ZG : pools;
    cb = SPLIT ? pools - ca * ZG : ca;
  };
  uint8_t *const buf0 = a.states + (size_t)blockIdx.x * 2 * a.W * a.state_stride;
  uint8_t *const buf1 = buf0 + (size_t)a.W * a.state_stride;

  for (uint32_t sid = blockIdx.x; sid < a.n_sub; sid += gridDim.x) {  // uniform
    __syncthreads();  // the shared tables are reused
    int ip = 0;
    for (int i = 1; i < a.n_pp; ++i)
      if (sid >= (STP ? a.pps[i].sub_off_t : a.pps[i].sub_off)) ip = i;
    const SearchPP pp = a.pps[ip];
    uint32_t rem = sid - (STP ? pp.sub_off_t : pp.sub_off);
    const int im = (int)(rem % (uint32_t)MB); rem /= (uint32_t)MB;
    const int id = (int)(rem % (uint32_t)DP); rem /= (uint32_t)DP;
    const int it = STP ? 0 : (int)(rem % (uint32_t)TP);  // (TP per stage: not part of the sub-problem)
    const int q = STP ? (int)rem : (int)(rem / (uint32_t)TP);
    const int P = pp.P;
    const uint32_t rs = pp.rs0 + (uint32_t)q * (uint32_t)P;
    SubResult *res = a.results + sid;
    const int64_t nb = pl.nb[im * DP + id];
    const int64_t D = pl.dpv[id];
    const int tp = pl.tpv[it];
    if (t == 0) {
      res->found = 0; res->truncated = 0; res->expanded = 0; res->sid = sid; res->P = (uint32_t)P;
      res->desc[0] = ip; res->desc[1] = q; res->desc[2] = it; res->desc[3] = id; res->desc[4] = im;
      res->desc[5] = MODE;
      s_bad = 0;
      s_expanded = 0;
      T.dp_even = (D % 2 == 0) ? 1 : 0;
      T.dtp = (double)(D * tp);
      T.dp = (long long)D;
    }
    __syncthreads();
    if (nb == 0) continue;              // the batch does not divide (uniform)
    const double p2p = (double)pl.p2p[im];
    const double nbm1 = (double)(nb - 1);
    // tables of the sub-problem
    for (int i = t; i < Z * Z; i += blockDim.x) {
      const int z = i / Z, y = i - z * Z;
      T.xfer[z][y] = p2p / pl.bw[z * Z + y];
      T.bw[z][y] = pl.bw[z * Z + y];
      double cm = 0.0, ch = 0.0, rp = 0.0;
      if (pl.egress && z != y) {
        const double both = pl.egress[z * Z + y] + pl.egress[y * Z + z];
        cm = (double)nb * (double)D * p2p * both;
        ch = (double)nb * (0.5 * (double)D) * p2p * both;
        rp = both;
      }
      T.comm[z][y] = cm;
      T.comm_half[z][y] = ch;
      T.ring_price[z][y] = rp;
    }
    for (int p = t; p < ZG; p += blockDim.x) {
      T.cap[p] = (int)((int64_t)pl.avail[p] / ((int64_t)tp * D));
      T.cap_half[p] = (int)(2 * (int64_t)pl.avail[p] / ((int64_t)tp * D));
      T.cap_gpus[p] = (int)((int64_t)pl.avail[p] / D);
      T.cap_half_gpus[p] = (int)(2 * (int64_t)pl.avail[p] / D);
    }
    if (t < TP) T.tpv[t] = pl.tpv[t];
    if (STP) {
      for (int i = t; i < P; i += blockDim.x) {  // the cheapest admissible (type, TP) of stage i
        const uint64_t params = pl.st_params[rs + i];
        double cmin = __builtin_huge_val(), umin = cmin, dmin = cmin, smin = cmin;
        bool any = false;
        for (int k = 0; k < TP; ++k) {
          const int tpk = pl.tpv[k];
          const uint64_t bytes = stage_bytes_of(params, pl.st_n[rs + i], pl.bpp, i, P, tpk, nb, pl.act[im * TP + k]);
          const uint64_t shard = (params + (uint64_t)tpk - 1) / (uint64_t)tpk;
          bool fits_some = false;
          for (int g = 0; g < G; ++g) {
            if (!(bytes + pl.res[g] <= pl.cap[g] && tpk <= pl.node[g])) continue;
            fits_some = true;
            cmin = fmin(cmin, pl.st_c[(((size_t)(rs + i) * G + g) * MB + im) * TP + k]);
            umin = fmin(umin, pl.st_u[((size_t)(rs + i) * G + g) * TP + k]);
            dmin = fmin(dmin, (double)(D * tpk) * pl.price[g]);
          }
          if (!fits_some) continue;
          any = true;
          for (int z = 0; z < Z; ++z) {
            double sync = 0.0;
            if (D > 1) {
              const double grad = (double)shard * (double)pl.gb;
              sync = 2.0 * (double)(D - 1) / (double)D * grad / pl.bw[z * Z + z];
            }
            smin = fmin(smin, sync);
          }
        }
        T.smin[0][i] = cmin; T.smin[1][i] = smin; T.smin[2][i] = umin; T.smin[3][i] = dmin;
        if (!any) s_bad = 1;  // (benign race: every writer stores 1)
      }
    } else
    for (int i = t; i < P; i += blockDim.x) {  // the cheapest admissible choice of stage i
      const uint64_t params = pl.st_params[rs + i];
      const uint64_t bytes = stage_bytes_of(params, pl.st_n[rs + i], pl.bpp, i, P, tp, nb, pl.act[im * TP + it]);
      const uint64_t shard = (params + (uint64_t)tp - 1) / (uint64_t)tp;
      double cmin = __builtin_huge_val(), umin = cmin, dmin = cmin, smin = cmin;
      bool any = false;
      for (int g = 0; g < G; ++g) {
        if (!(bytes + pl.res[g] <= pl.cap[g] && tp <= pl.node[g])) continue;
        any = true;
        cmin = fmin(cmin, pl.st_c[(((size_t)(rs + i) * G + g) * MB + im) * TP + it]);
        umin = fmin(umin, pl.st_u[((size_t)(rs + i) * G + g) * TP + it]);
        dmin = fmin(dmin, (double)(D * tp) * pl.price[g]);
      }
      for (int z = 0; z < Z; ++z) {
        double sync = 0.0;
        if (D > 1) {
          const double grad = (double)shard * (double)pl.gb;
          sync = 2.0 * (double)(D - 1) / (double)D * grad / pl.bw[z * Z + z];
        }
        smin = fmin(smin, sync);
      }
      T.smin[0][i] = cmin; T.smin[1][i] = smin; T.smin[2][i] = umin; T.smin[3][i] = dmin;
      if (!any) s_bad = 1;  // (benign race: every writer stores 1)
    }
    __syncthreads();
    if (s_bad) continue;  // some stage fits no pool (uniform)
    if (t == 0) {  // what lies behind stage i, accumulated from the last stage backwards
      T.S[0][P - 1] = T.S[1][P - 1] = T.S[2][P - 1] = T.S[3][P - 1] = T.S[4][P - 1] = 0.0;
      for (int i = P - 2; i >= 0; --i) {
        T.S[0][i] = T.S[0][i + 1] + T.smin[0][i + 1];
        T.S[1][i] = fmax(T.S[1][i + 1], T.smin[0][i + 1]);
        T.S[2][i] = fmax(T.S[2][i + 1], T.smin[1][i + 1]);
        T.S[3][i] = fmax(T.S[3][i + 1], T.smin[2][i + 1]);
        T.S[4][i] = T.S[4][i + 1] + T.smin[3][i + 1];
      }
    }
    int n_cur = 1;  // frontier length; level 0 extends one empty placement
    bool truncated = false;
    for (int j = 0; j < P; ++j) {  // place stage j (uniform loop)
      uint8_t *const cur = (j & 1) ? buf1 : buf0, *const nxt = (j & 1) ? buf0 : buf1;
      __syncthreads();
      // the level's tables: stage j on every type / zone
      if (STP) {
        if (t < G * TP) {  // (type g, TP index k)
          const int g = t / TP, k = t - g * TP, tpk = pl.tpv[k];
          const uint64_t params = pl.st_params[rs + j];
          const uint64_t bytes = stage_bytes_of(params, pl.st_n[rs + j], pl.bpp, j, P, tpk, nb, pl.act[im * TP + k]);
          T.l_c3[g][k] = pl.st_c[(((size_t)(rs + j) * G + g) * MB + im) * TP + k];
          T.l_upd3[g][k] = pl.st_u[((size_t)(rs + j) * G + g) * TP + k];
          T.l_dol3[g][k] = (double)(D * tpk) * pl.price[g];
          if (k == 0) T.l_price[g] = pl.price[g];
          s_fit3[g][k] = (bytes + pl.res[g] <= pl.cap[g] && tpk <= pl.node[g]) ? 1 : 0;
        } else if (t >= 128 && t < 128 + Z * TP) {  // (zone z, TP index k)
          const int z = (t - 128) / TP, k = (t - 128) - z * TP, tpk = pl.tpv[k];
          const uint64_t params = pl.st_params[rs + j];
          const uint64_t shard = (params + (uint64_t)tpk - 1) / (uint64_t)tpk;
          double sync = 0.0, ring = 0.0;
          if (D > 1) {
            const double grad = (double)shard * (double)pl.gb;
            sync = 2.0 * (double)(D - 1) / (double)D * grad / pl.bw[z * Z + z];
            ring = 2.0 * (double)(D - 1) / (double)D * grad;
          }
          T.l_sync3[z][k] = sync;
          if (z == 0) T.l_ring3[k] = ring;
        }
        __syncthreads();
        if (t < TP) {
          uint32_t m = 0;
          for (int g = 0; g < G; ++g) m |= (uint32_t)s_fit3[g][t] << g;
          T.l_fit3[t] = m;
        }
      } else if (t < G) {
        const uint64_t params = pl.st_params[rs + j];
        const uint64_t bytes = stage_bytes_of(params, pl.st_n[rs + j], pl.bpp, j, P, tp, nb, pl.act[im * TP + it]);
        T.l_c[t] = pl.st_c[(((size_t)(rs + j) * G + t) * MB + im) * TP + it];
        T.l_upd[t] = pl.st_u[((size_t)(rs + j) * G + t) * TP + it];
        T.l_dol[t] = (double)(D * tp) * pl.price[t];
        T.l_price[t] = pl.price[t];
        const bool fits = bytes + pl.res[t] <= pl.cap[t] && tp <= pl.node[t];
        const unsigned long long m = __builtin_amdgcn_ballot_w64(fits);
        if (t == 0) T.l_fit = (uint32_t)m;
      } else if (t >= 64 && t < 64 + Z) {
        const int z = t - 64;
        const uint64_t params = pl.st_params[rs + j];
        const uint64_t shard = (params + (uint64_t)tp - 1) / (uint64_t)tp;
        double sync = 0.0, ring = 0.0;
        if (D > 1) {
          const double grad = (double)shard * (double)pl.gb;
          sync = 2.0 * (double)(D - 1) / (double)D * grad / pl.bw[z * Z + z];
          ring = 2.0 * (double)(D - 1) / (double)D * grad;
        }
        T.l_sync[z] = sync;
        if (z == 0) T.l_ring = ring;
      }
      if (t == 0) s_nbuf = 0;
      __syncthreads();
      const bool last = j == P - 1;
      const int n_total = n_cur * NCH;
      unsigned long long best_k = ~0ull;  // last level: this thread's smallest (key, id)
      uint32_t best_i = ~0u;
      uint32_t my_expanded = 0;
      for (int row = 0; row * kSearchThreads < n_total; ++row) {  // uniform
        const int cand = row * kSearchThreads + t;
        bool keep = false;
        unsigned long long kbits = 0;
        if (cand < n_total) {
          const int r = cand / NCH, c = cand - r * NCH;
          int pa, pb, pk;
          choice(c, it, pa, pb, pk);
          const SState *par = j == 0 ? nullptr : reinterpret_cast<const SState *>(cur + (size_t)r * a.state_stride);
          SAcc o;
          int runs;
          if (search_step<MODE>(T, par, j, pa, pb, pk, G, a.max_runs, o, runs)) {
            my_expanded += 1;
            const SBound b = search_bound_of<MODE>(T, o, j, nbm1);
            const double key = a.objective == 0 ? b.T : b.C;
            bool drop = false;
            if (a.has_bound) drop = a.objective == 0 ? b.C > a.bound : 1.0 / b.T < a.bound;
            if (a.has_inc && key > a.inc) drop = true;
            keep = !drop;
            kbits = (unsigned long long)__double_as_longlong(key);  // non-negative: orders like the value
          }
        }
        if (last) {
          if (keep && key_id_less(kbits, (uint32_t)cand, best_k, best_i)) { best_k = kbits; best_i = (uint32_t)cand; }
          continue;
        }
        // append the row's survivors in candidate order
        const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
        if (lane == 0) s_wave[wv] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t before = 0, row_total = 0;
        for (int w = 0; w < kSearchThreads / 64; ++w) {
          if (w < wv) before += s_wave[w];
          row_total += s_wave[w];
        }
        int nbuf = s_nbuf;
        if (nbuf + (int)row_total > kSearchBuf) {  // uniform: make room, only the W smallest can matter
          __syncthreads();
          search_sort(b_key, b_id, nbuf);
          nbuf = min(nbuf, a.W);
          truncated = true;
        }
        if (keep) {
          const int at = nbuf + (int)before + __popcll(m & ((1ull << lane) - 1ull));
          b_key[at] = kbits;
          b_id[at] = (uint32_t)cand;
        }
        __syncthreads();
        if (t == 0) s_nbuf = nbuf + (int)row_total;
        __syncthreads();
      }
      atomicAdd(&s_expanded, (unsigned long long)my_expanded);
      if (last) {
        // the smallest (key, id) of the workgroup
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          const unsigned long long ok2 = __shfl_xor(best_k, off);
          const uint32_t oi = __shfl_xor(best_i, off);
          if (key_id_less(ok2, oi, best_k, best_i)) { best_k = ok2; best_i = oi; }
        }
        if (lane == 0) { s_bk[wv] = best_k; s_bi[wv] = best_i; }
        __syncthreads();
        best_k = s_bk[0]; best_i = s_bi[0];
        for (int w = 1; w < kSearchThreads / 64; ++w)
          if (key_id_less(s_bk[w], s_bi[w], best_k, best_i)) { best_k = s_bk[w]; best_i = s_bi[w]; }
        if (best_i != ~0u) {  // uniform
          const int r = (int)best_i / NCH, c = (int)best_i - r * NCH;
          int pa, pb, pk;
          choice(c, it, pa, pb, pk);
          const uint8_t *par_path = cur + (size_t)r * a.state_stride + kStateBytes;
          for (int i = t; i < P - 1; i += blockDim.x) {
            res->pools[i] = par_path[i];
            res->pools_b[i] = SPLIT ? par_path[a.path_stride + i] : par_path[i];
            res->tps[i] = STP ? par_path[2 * a.path_stride + i] : it;
          }
          if (t == 0) {
            const SState *par = j == 0 ? nullptr : reinterpret_cast<const SState *>(cur + (size_t)r * a.state_stride);
            SAcc o;
            int runs;
            search_step<MODE>(T, par, j, pa, pb, pk, G, a.max_runs, o, runs);
            const SBound b = search_bound_of<MODE>(T, o, j, nbm1);
            res->pools[P - 1] = pa;
            res->pools_b[P - 1] = pb;
            res->tps[P - 1] = pk;
            if (STP) res->desc[2] = P > 1 ? (int)par_path[2 * a.path_stride] : pk;  // stage 0's
            res->T = b.T;
            res->C = b.C;
            res->key = a.objective == 0 ? b.T : b.C;
            res->found = 1;
          }
        }
        break;
      }
      __syncthreads();
      int n_next = s_nbuf;
      if (n_next > a.W) {  // uniform: keep the W smallest bounds, in that order
        search_sort(b_key, b_id, n_next);
        n_next = a.W;
        truncated = true;
      }
      if (n_next == 0) break;  // uniform
      // write the next frontier
      for (int k = t; k < n_next; k += blockDim.x) {
        const int cand = (int)b_id[k];
        const int r = cand / NCH, c = cand - r * NCH;
        int pa, pb, pk;
        choice(c, it, pa, pb, pk);
        uint8_t *const out = nxt + (size_t)k * a.state_stride;
        const SState *par = j == 0 ? nullptr : reinterpret_cast<const SState *>(cur + (size_t)r * a.state_stride);
        SAcc o;
        int runs;
        search_step<MODE>(T, par, j, pa, pb, pk, G, a.max_runs, o, runs);
        SState st;
        if (par) {
          st = *par;
          const uint8_t *par_path = cur + (size_t)r * a.state_stride + kStateBytes;
          for (int i = 0; i < j; ++i) {
            out[kStateBytes + i] = par_path[i];
            if (SPLIT) out[kStateBytes + a.path_stride + i] = par_path[a.path_stride + i];
            if (STP) out[kStateBytes + 2 * a.path_stride + i] = par_path[2 * a.path_stride + i];
          }
        } else {
          for (int x = 0; x < kSearchMaxPools; ++x) st.cnt[x] = 0;
        }
        st.sum = o.sum; st.maxt = o.maxt; st.c_open = o.c_open; st.xb_open = o.xb_open;
        st.sum_b = o.sum_b; st.maxt_b = o.maxt_b; st.c_open_b = o.c_open_b; st.xb_open_b = o.xb_open_b;
        st.msync = o.msync; st.mupd = o.mupd; st.dol = o.dol; st.comm = o.comm;
        if (BOTH) {
          st.cnt[pa] = (uint16_t)(st.cnt[pa] + T.tpv[pk]);
          st.cnt[pb] = (uint16_t)(st.cnt[pb] + T.tpv[pk]);
        } else if (STP) {
          st.cnt[pa] = (uint16_t)(st.cnt[pa] + T.tpv[pk]);
        } else if (!SPLIT) {
          st.cnt[pa] = (uint16_t)(st.cnt[pa] + 1);
        } else {
          st.cnt[pa] = (uint16_t)(st.cnt[pa] + 1);
          st.cnt[pb] = (uint16_t)(st.cnt[pb] + 1);
        }
        st.pool = (uint8_t)pa;
        st.pool_b = (uint8_t)pb;
        st.tpi = (uint8_t)pk;
        st.runs = (uint8_t)runs;
        for (int x = 0; x < 4; ++x) st.pad[x] = 0;
        *reinterpret_cast<SState *>(out) = st;
        out[kStateBytes + j] = (uint8_t)pa;
        if (SPLIT) out[kStateBytes + a.path_stride + j] = (uint8_t)pb;
        if (STP) out[kStateBytes + 2 * a.path_stride + j] = (uint8_t)pk;
      }
      n_cur = n_next;
    }
    __syncthreads();
    if (t == 0) {
      res->truncated = truncated ? 1u : 0u;
      res->expanded = s_expanded;
    }
  }
}

// Smallest (key, sub-problem) over the sub-problems' winners; also the totals.
__global__ __launch_bounds__(256) void k_search_pick(const SubResult *results, uint32_t n_sub, SubResult *out) {
  __shared__ unsigned long long s_k[4], s_e[4];
  __shared__ uint32_t s_i[4], s_t[4];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  unsigned long long bk = ~0ull, expanded = 0;
  uint32_t bi = ~0u, trunc = 0;
  for (uint32_t i = t; i < n_sub; i += blockDim.x) {
    const SubResult &r = results[i];
    expanded += r.expanded;
    trunc |= r.truncated;
    if (r.found) {
      const unsigned long long k = (unsigned long long)__double_as_longlong(r.key);
      if (key_id_less(k, i, bk, bi)) { bk = k; bi = i; }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long ok = __shfl_xor(bk, off);
    const uint32_t oi = __shfl_xor(bi, off);
    if (key_id_less(ok, oi, bk, bi)) { bk = ok; bi = oi; }
    expanded += __shfl_xor(expanded, off);
    trunc |= __shfl_xor(trunc, off);
  }
  if (lane == 0) { s_k[wv] = bk; s_i[wv] = bi; s_e[wv] = expanded; s_t[wv] = trunc; }
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 4; ++w) {
      if (key_id_less(s_k[w], s_i[w], bk, bi)) { bk = s_k[w]; bi = s_i[w]; }
      expanded += s_e[w];
      trunc |= s_t[w];
    }
    s_i[0] = bi; s_e[0] = expanded; s_t[0] = trunc;
  }
  __syncthreads();
  bi = s_i[0];
  if (bi == ~0u) {
    if (t == 0) { out->found = 0; out->truncated = s_t[0]; out->expanded = s_e[0]; out->P = 0; }
    return;
  }
  const unsigned long long *src = reinterpret_cast<const unsigned long long *>(results + bi);
  unsigned long long *dst = reinterpret_cast<unsigned long long *>(out);
  for (uint32_t w = t; w < sizeof(SubResult) / 8; w += blockDim.x) dst[w] = src[w];
  __syncthreads();
  if (t == 0) { out->truncated = s_t[0]; out->expanded = s_e[0]; }
}

// ------------------------------------------------------------------ listed placements

struct PlaceArgs {
  uint64_t count;
  const int32_t *desc;    // [count][5] pp index, partition, tp index, dp index, mb index
  const int32_t *pools;   // [count][pool_stride] pool of every stage
  const int32_t *pools_b; // optional, same shape: pool of the other half of every stage's replicas
  const int32_t *tps;     // optional, same shape: TP index of every stage (else the descriptor's)
  uint32_t pool_stride;
  const SubResult *one;   // alternative to desc / pools: the placement held by this record
  const SearchPP *pps;
  int n_pp;
  int objective, has_bound;
  double bound;
  double *T, *C;
  uint64_t *mem;
  uint32_t *mask;
};

constexpr int kPlaceWaves = 4;

// Stages that split their D replicas over two pools, half on each, also across zones (the D
// tuples of a stage, Sec. 4.2): the replicas on the first pools and those on the second pools
// form two kinds of pipeline; T_iter takes the slower kind (Sec. 4.3: max over pipelines), a
// split stage's all-reduce runs over the slowest link of a ring through both pools, and the
// traffic between zones -- of the pipelines, each kind carrying half of the replicas, and of
// the ring -- is paid for.  With a TP index per stage (tps; else it for all) both halves of a
// stage use the stage's degree.  One wave; valid descriptor, pools and TP indices; nb > 0.
__device__ __forceinline__ void eval_split_wave(const DevPlan &pl, const int32_t *pa, const int32_t *pb,
                                                const int32_t *tps, int P, uint32_t rs, int it, int im,
                                                int64_t nb, int64_t D, RefineLds &L, double *t_second,
                                                int *cnt, double &T, double &C, uint64_t &peak,
                                                uint32_t &mask) {
  const int G = pl.G, Z = pl.Z, ZG = pl.ZGr, MB = pl.MB, TP = pl.TP;
  const int lane = threadIdx.x & 63;
  const double p2p = (double)pl.p2p[im];
  double max_a = 0.0, max_b = 0.0, t_sync = 0.0, t_upd = 0.0;
  uint32_t oom = 0, h1 = 0, odd = 0;
  for (int i = lane; i < P; i += 64) {
    const int a = pa[i], b = pb[i];
    const int ga = a % G, za = a / G, gb = b % G, zb = b / G;
    const int ti = tps ? tps[i] : it;  // this stage's TP index and degree
    const int64_t tp = pl.tpv[ti];
    atomicAdd(&cnt[a], (int)tp);  // GPUs of one replica, counted once per half
    atomicAdd(&cnt[b], (int)tp);
    if (a != b && (D & 1)) odd = 1u;
    const size_t si = (size_t)rs + i;
    const uint64_t params = pl.st_params[si];
    const uint64_t bytes = stage_bytes_of(params, pl.st_n[si], pl.bpp, i, P, (int)tp, nb, pl.act[im * TP + ti]);
    const uint64_t m1 = bytes + pl.res[ga], m2 = bytes + pl.res[gb];
    if (m1 > pl.cap[ga] || m2 > pl.cap[gb]) oom = 1u;
    if (tp > pl.node[ga] || tp > pl.node[gb]) h1 = 1u;
    peak = m1 > peak ? m1 : peak;
    peak = m2 > peak ? m2 : peak;
    double xa = 0.0, xb = 0.0, traffic = 0.0;
    if (i < P - 1) {
      const int zna = pa[i + 1] / G, znb = pb[i + 1] / G;
      xa += p2p / link_bw(pl, za, zna, p2p);
      xb += p2p / link_bw(pl, zb, znb, p2p);
      if (pl.egress) {  // each kind of pipeline carries half of the replicas
        if (zna != za) traffic += (double)nb * (0.5 * (double)D) * p2p * (pl.egress[za * Z + zna] + pl.egress[zna * Z + za]);
        if (znb != zb) traffic += (double)nb * (0.5 * (double)D) * p2p * (pl.egress[zb * Z + znb] + pl.egress[znb * Z + zb]);
      }
    }
    if (i > 0) {
      xa += p2p / link_bw(pl, za, pa[i - 1] / G, p2p);
      xb += p2p / link_bw(pl, zb, pb[i - 1] / G, p2p);
    }
    const double ta = pl.st_c[((si * G + ga) * MB + im) * TP + ti] + xa;
    const double tb = pl.st_c[((si * G + gb) * MB + im) * TP + ti] + xb;
    max_a = fmax(max_a, ta);
    max_b = fmax(max_b, tb);
    if (D > 1) {
      const uint64_t shard = (params + (uint64_t)tp - 1) / (uint64_t)tp;
      const double buffer = (double)shard * (double)pl.gb;
      double link = link_bw(pl, za, za, buffer);
      if (zb != za)
        link = fmin(fmin(link, link_bw(pl, zb, zb, buffer)),
                    fmin(link_bw(pl, za, zb, buffer), link_bw(pl, zb, za, buffer)));
      const double ring_bytes = 2.0 * (double)(D - 1) / (double)D * buffer;
      t_sync = fmax(t_sync, ring_bytes / link);
      if (pl.egress && zb != za) traffic += ring_bytes * (pl.egress[za * Z + zb] + pl.egress[zb * Z + za]);
    }
    t_upd = fmax(t_upd, fmax(pl.st_u[(si * G + ga) * TP + ti], pl.st_u[(si * G + gb) * TP + ti]));
    L.t[i] = ta;
    t_second[i] = tb;
    L.dol[i] = (double)(D * tp) * (0.5 * (pl.price[ga] + pl.price[gb]));
    L.comm[i] = traffic;
  }
  if (__builtin_amdgcn_ballot_w64(oom != 0) != 0) mask |= 1u;
  if (__builtin_amdgcn_ballot_w64(h1 != 0) != 0) mask |= 8u;
  if (__builtin_amdgcn_ballot_w64(odd != 0) != 0) mask |= 2u;  // D replicas cannot be halved
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint64_t o = __shfl_xor((unsigned long long)peak, off);
    peak = o > peak ? o : peak;
  }
  max_a = wave_max_f64(max_a);
  max_b = wave_max_f64(max_b);
  t_sync = wave_max_f64(t_sync);
  t_upd = wave_max_f64(t_upd);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  bool over = false;  // every pool holds the halves placed on it
  for (int p = lane; p < ZG; p += 64)
    if ((int64_t)cnt[p] * D > 2 * (int64_t)pl.avail[p]) over = true;
  if (__builtin_amdgcn_ballot_w64(over) != 0) mask |= 2u;
  double sum_a = 0.0, sum_b = 0.0, dollars = 0.0, traffic = 0.0;
  for (int i = 0; i < P; ++i) {
    sum_a += L.t[i];
    sum_b += t_second[i];
    dollars += L.dol[i];
    traffic += L.comm[i];
  }
  const double t_pp = fmax(sum_a + (double)(nb - 1) * max_a, sum_b + (double)(nb - 1) * max_b);
  T = (t_pp + t_sync) + t_upd;
  C = dollars / 3600.0 * T + traffic;
}

// The simulator (Sec. 4.3) for plans whose stages choose their pools freely: one wave per
// plan, lane i takes stages i, i + 64, ...; sums in stage order.  With a TP index per stage
// every per-stage quantity (memory shard, activation bytes, profiled times, node size, gradient
// shard, GPUs against the quota, rent) uses the stage's own degree.  A descriptor, pool or TP
// index out of range yields mask = 0xFFFFFFFF, T = C = +inf, mem = 0.
__global__ __launch_bounds__(kPlaceWaves * 64) void k_eval_placements(DevPlan pl, PlaceArgs a) {
  __shared__ RefineLds lds[kPlaceWaves];
  __shared__ double s_second[kPlaceWaves][kMaxStages];  // stage times of the second kind of pipeline
  __shared__ int s_cnt[kPlaceWaves][kSearchMaxPools];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint64_t ci = (uint64_t)blockIdx.x * kPlaceWaves + wv;
  if (ci >= a.count) return;  // whole waves leave; no barrier below
  const int G = pl.G, Z = pl.Z, ZG = pl.ZGr, MB = pl.MB, TP = pl.TP, DP = pl.DP;
  int ip, q, it, id, im;
  if (a.one) { ip = a.one->desc[0]; q = a.one->desc[1]; it = a.one->desc[2]; id = a.one->desc[3]; im = a.one->desc[4]; }
  else { const int32_t *d = a.desc + ci * 5; ip = d[0]; q = d[1]; it = d[2]; id = d[3]; im = d[4]; }
  double T = __builtin_huge_val(), C = T;
  uint64_t peak = 0;
  uint32_t mask = 0xFFFFFFFFu;
  bool valid = ip >= 0 && ip < a.n_pp && it >= 0 && it < TP && id >= 0 && id < DP && im >= 0 && im < MB && q >= 0;
  if (valid) valid = q < a.pps[ip].n_part;
  const int P = valid ? a.pps[ip].P : 0;
  if (valid && !a.one && (uint32_t)P > a.pool_stride) valid = false;
  RefineLds &L = lds[wv];
  int *cnt = s_cnt[wv];
  const bool split = a.one ? (a.one->desc[5] == SEARCH_SPLIT || a.one->desc[5] == SEARCH_SPLIT_TP)
                           : a.pools_b != nullptr;  // stages may split their replicas
  const int32_t *const tps = a.one ? a.one->tps : (a.tps ? a.tps + ci * a.pool_stride : nullptr);
  if (valid) {
    for (int p = lane; p < kSearchMaxPools; p += 64) cnt[p] = 0;
    bool bad = false;
    for (int i = lane; i < P; i += 64) {
      const int p = a.one ? a.one->pools[i] : a.pools[ci * a.pool_stride + i];
      if (p < 0 || p >= ZG) bad = true;
      if (split) {
        const int p2 = a.one ? a.one->pools_b[i] : a.pools_b[ci * a.pool_stride + i];
        if (p2 < 0 || p2 >= ZG) bad = true;
      }
      if (tps && (tps[i] < 0 || tps[i] >= TP)) bad = true;
    }
    if (__builtin_amdgcn_ballot_w64(bad) != 0) valid = false;
  }
  if (valid) {
    mask = 0;
    const uint32_t rs = a.pps[ip].rs0 + (uint32_t)q * (uint32_t)P;
    const int64_t nb = pl.nb[im * DP + id], D = pl.dpv[id];
    if (nb == 0) {
      mask = 4u;
    } else if (split) {
      __builtin_amdgcn_wave_barrier();
      eval_split_wave(pl, a.one ? a.one->pools : a.pools + ci * a.pool_stride,
                      a.one ? a.one->pools_b : a.pools_b + ci * a.pool_stride,
                      tps, P, rs, it, im, nb, D, L, s_second[wv], cnt, T, C, peak, mask);
      if (a.has_bound) {
        if (a.objective == 0) { if (C > a.bound) mask |= 32u; }
        else if (1.0 / T < a.bound) mask |= 32u;
      }
    } else {
      const double p2p = (double)pl.p2p[im];
      __builtin_amdgcn_wave_barrier();
      double max_t = 0.0, t_sync = 0.0, t_upd = 0.0;
      uint32_t oom = 0, h1 = 0;
      for (int i = lane; i < P; i += 64) {
        const int p = a.one ? a.one->pools[i] : a.pools[ci * a.pool_stride + i];
        const int pn = i < P - 1 ? (a.one ? a.one->pools[i + 1] : a.pools[ci * a.pool_stride + i + 1]) : p;
        const int pv = i > 0 ? (a.one ? a.one->pools[i - 1] : a.pools[ci * a.pool_stride + i - 1]) : p;
        const int g = p % G, z = p / G, zn = pn / G, zp = pv / G;
        const int ti = tps ? tps[i] : it;      // this stage's TP index and degree
        const int64_t tpi = pl.tpv[ti];
        atomicAdd(&cnt[p], (int)tpi);          // GPUs of one replica
        const size_t si = (size_t)rs + i;
        const uint64_t params = pl.st_params[si];
        const uint64_t bytes = stage_bytes_of(params, pl.st_n[si], pl.bpp, i, P, (int)tpi, nb, pl.act[im * TP + ti]);
        const uint64_t m = bytes + pl.res[g];
        if (m > pl.cap[g]) oom = 1u;
        if (tpi > pl.node[g]) h1 = 1u;
        peak = m > peak ? m : peak;
        double x = 0.0, comm = 0.0;
        if (i < P - 1) {
          x += p2p / link_bw(pl, z, zn, p2p);
          if (pl.egress && zn != z)
            comm = (double)nb * (double)D * p2p * (pl.egress[z * Z + zn] + pl.egress[zn * Z + z]);
        }
        if (i > 0) x += p2p / link_bw(pl, z, zp, p2p);
        const double ts = pl.st_c[((si * G + g) * MB + im) * TP + ti] + x;
        max_t = fmax(max_t, ts);
        if (D > 1) {
          const uint64_t shard = (params + (uint64_t)tpi - 1) / (uint64_t)tpi;
          const double gbytes = (double)shard * (double)pl.gb;
          t_sync = fmax(t_sync, 2.0 * (double)(D - 1) / (double)D * gbytes / link_bw(pl, z, z, gbytes));
        }
        t_upd = fmax(t_upd, pl.st_u[(si * G + g) * TP + ti]);
        L.t[i] = ts;
        L.dol[i] = (double)(D * tpi) * pl.price[g];
        L.comm[i] = comm;
      }
      if (__builtin_amdgcn_ballot_w64(oom != 0) != 0) mask |= 1u;
      if (__builtin_amdgcn_ballot_w64(h1 != 0) != 0) mask |= 8u;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const uint64_t o = __shfl_xor((unsigned long long)peak, off);
        peak = o > peak ? o : peak;
      }
      max_t = wave_max_f64(max_t);
      t_sync = wave_max_f64(t_sync);
      t_upd = wave_max_f64(t_upd);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      bool over = false;  // quota: D replicas of every stage on the pool, its tp GPUs each
      for (int p = lane; p < ZG; p += 64)
        if ((int64_t)cnt[p] * D > (int64_t)pl.avail[p]) over = true;
      if (__builtin_amdgcn_ballot_w64(over) != 0) mask |= 2u;
      double sum_t = 0.0, dollars = 0.0, comm = 0.0;
      for (int i = 0; i < P; ++i) {
        sum_t += L.t[i];
        dollars += L.dol[i];
        comm += L.comm[i];
      }
      T = (sum_t + (double)(nb - 1) * max_t) + t_sync + t_upd;
      C = dollars / 3600.0 * T + comm;
      if (a.has_bound) {
        if (a.objective == 0) { if (C > a.bound) mask |= 32u; }
        else if (1.0 / T < a.bound) mask |= 32u;
      }
    }
  }
  if (lane == 0) {
    if (a.T) a.T[ci] = T;
    if (a.C) a.C[ci] = C;
    if (a.mem) a.mem[ci] = mask == 0xFFFFFFFFu ? 0 : peak;
    if (a.mask) a.mask[ci] = mask;
  }
}

// ------------------------------------------------------------------ a pool per replica

constexpr int64_t kReplicaMaxDegree = 65536;  // replicas per stage a listed plan may name one by one

struct ReplicaArgs {
  uint64_t count;
  const int32_t *desc;    // [count][5] pp index, partition, tp index, dp index, mb index
  const int32_t *pools;   // [count][stride]: the pool of replica r of stage i at i * D + r
  uint64_t stride;
  const int32_t *tps;     // optional, [count][tps_stride]: TP index of every stage (else the descriptor's)
  uint32_t tps_stride;
  const SearchPP *pps;
  int n_pp;
  int objective, has_bound;
  double bound;
  double *T, *C;
  uint64_t *mem;
  uint32_t *mask;
};

__device__ __forceinline__ double wave_min_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmin(v, __shfl_xor(v, off));
  return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// The plan tuple in full (Sec. 4.2: D tuples per stage): replica r of all stages is pipeline r,
// T_iter = max over the D pipelines + T_sync + T_update (Sec. 4.3); the all-reduce of a stage is
// a ring through its replicas in their order at the pace of its slowest link; traffic between
// zones is paid for where a pipeline or a ring crosses; a pool's quota counts the GPUs it gives.
// One wave per plan: lane l takes the pipelines l, l + 64, ... and walks their stages in order,
// so a pipeline's sum is taken in stage order.  A descriptor or pool out of range, fewer than
// P x D entries per plan or more than 65 536 replicas yield mask = 0xFFFFFFFF, T = C = +inf, mem = 0.
__global__ __launch_bounds__(kPlaceWaves * 64) void k_eval_replicas(DevPlan pl, ReplicaArgs a) {
  __shared__ int s_cnt[kPlaceWaves][kSearchMaxPools];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const uint64_t ci = (uint64_t)blockIdx.x * kPlaceWaves + wv;
  if (ci >= a.count) return;  // whole waves leave; no barrier below
  const int G = pl.G, Z = pl.Z, ZG = pl.ZGr, MB = pl.MB, TP = pl.TP, DP = pl.DP;
  const int32_t *d = a.desc + ci * 5;
  const int ip = d[0], q = d[1], it = d[2], id = d[3], im = d[4];
  double T = __builtin_huge_val(), C = T;
  uint64_t peak = 0;
  uint32_t mask = 0xFFFFFFFFu;
  bool valid = ip >= 0 && ip < a.n_pp && it >= 0 && it < TP && id >= 0 && id < DP && im >= 0 && im < MB && q >= 0;
  if (valid) valid = q < a.pps[ip].n_part;
  const int P = valid ? a.pps[ip].P : 0;
  const int64_t D = valid ? (int64_t)pl.dpv[id] : 0;
  if (valid && (D > kReplicaMaxDegree || (uint64_t)P * (uint64_t)D > a.stride)) valid = false;
  if (valid && a.tps && (uint32_t)P > a.tps_stride) valid = false;
  const int32_t *pools = a.pools + ci * a.stride;
  const int32_t *const tps = a.tps ? a.tps + ci * a.tps_stride : nullptr;
  int *cnt = s_cnt[wv];
  if (valid) {
    for (int p = lane; p < kSearchMaxPools; p += 64) cnt[p] = 0;
    bool bad = false;
    for (int64_t k = lane; k < (int64_t)P * D; k += 64)
      if (pools[k] < 0 || pools[k] >= ZG) bad = true;
    if (tps)
      for (int i = lane; i < P; i += 64)
        if (tps[i] < 0 || tps[i] >= TP) bad = true;
    if (__builtin_amdgcn_ballot_w64(bad) != 0) valid = false;
  }
  if (valid) {
    mask = 0;
    const uint32_t rs = a.pps[ip].rs0 + (uint32_t)q * (uint32_t)P;
    const int64_t nb = pl.nb[im * DP + id];
    if (nb == 0) {
      mask = 4u;
    } else {
      const double p2p = (double)pl.p2p[im];
      __builtin_amdgcn_wave_barrier();
      double t_pipe = 0.0, t_upd = 0.0, t_sync = 0.0, rent = 0.0, traffic = 0.0;
      uint32_t oom = 0, h1 = 0;
      // the pipelines
      for (int64_t r = lane; r < D; r += 64) {
        double total = 0.0, slowest = 0.0;
        for (int i = 0; i < P; ++i) {
          const int p = pools[(int64_t)i * D + r], g = p % G, z = p / G;
          const int ti = tps ? tps[i] : it;  // the stage's TP index and degree
          const int64_t tp = pl.tpv[ti];
          atomicAdd(&cnt[p], (int)tp);  // GPUs the pool gives
          const size_t si = (size_t)rs + i;
          const uint64_t bytes = stage_bytes_of(pl.st_params[si], pl.st_n[si], pl.bpp, i, P, (int)tp, nb, pl.act[im * TP + ti]);
          const uint64_t m = bytes + pl.res[g];
          if (m > pl.cap[g]) oom = 1u;
          if (tp > pl.node[g]) h1 = 1u;
          peak = m > peak ? m : peak;
          double x = 0.0;
          if (i < P - 1) {
            const int zn = pools[(int64_t)(i + 1) * D + r] / G;
            x += p2p / link_bw(pl, z, zn, p2p);
            if (pl.egress && zn != z)  // one replica's microbatches, both directions
              traffic += (double)nb * p2p * (pl.egress[z * Z + zn] + pl.egress[zn * Z + z]);
          }
          if (i > 0) x += p2p / link_bw(pl, z, pools[(int64_t)(i - 1) * D + r] / G, p2p);
          const double ts = pl.st_c[((si * G + g) * MB + im) * TP + ti] + x;
          total += ts;
          slowest = fmax(slowest, ts);
          t_upd = fmax(t_upd, pl.st_u[(si * G + g) * TP + ti]);
          rent += (double)tp * pl.price[g];
        }
        t_pipe = fmax(t_pipe, total + (double)(nb - 1) * slowest);
      }
      // the rings
      if (D > 1)
        for (int i = 0; i < P; ++i) {  // uniform
          const uint64_t params = pl.st_params[rs + i];
          const uint64_t tp = (uint64_t)pl.tpv[tps ? tps[i] : it];
          const uint64_t shard = (params + tp - 1) / tp;
          const double buffer = (double)shard * (double)pl.gb;
          const double ring_bytes = 2.0 * (double)(D - 1) / (double)D * buffer;
          double link = __builtin_huge_val();
          for (int64_t r = lane; r < D; r += 64) {
            const int zr = pools[(int64_t)i * D + r] / G, zs = pools[(int64_t)i * D + (r + 1 == D ? 0 : r + 1)] / G;
            link = fmin(link, link_bw(pl, zr, zs, buffer));
            if (pl.egress && zr != zs) traffic += ring_bytes * pl.egress[zr * Z + zs];
          }
          t_sync = fmax(t_sync, ring_bytes / wave_min_f64(link));
        }
      if (__builtin_amdgcn_ballot_w64(oom != 0) != 0) mask |= 1u;
      if (__builtin_amdgcn_ballot_w64(h1 != 0) != 0) mask |= 8u;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const uint64_t o = __shfl_xor((unsigned long long)peak, off);
        peak = o > peak ? o : peak;
      }
      t_pipe = wave_max_f64(t_pipe);
      t_upd = wave_max_f64(t_upd);
      rent = wave_sum_f64(rent);
      traffic = wave_sum_f64(traffic);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      bool over = false;
      for (int p = lane; p < ZG; p += 64)
        if ((int64_t)cnt[p] > (int64_t)pl.avail[p]) over = true;
      if (__builtin_amdgcn_ballot_w64(over) != 0) mask |= 2u;
      T = (t_pipe + t_sync) + t_upd;
      C = rent / 3600.0 * T + traffic;
      if (a.has_bound) {
        if (a.objective == 0) { if (C > a.bound) mask |= 32u; }
        else if (1.0 / T < a.bound) mask |= 32u;
      }
    }
  }
  if (lane == 0) {
    if (a.T) a.T[ci] = T;
    if (a.C) a.C[ci] = C;
    if (a.mem) a.mem[ci] = mask == 0xFFFFFFFFu ? 0 : peak;
    if (a.mask) a.mask[ci] = mask;
  }
}

}  // namespace sailor
