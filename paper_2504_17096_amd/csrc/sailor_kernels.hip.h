// HIP kernels of the batched plan evaluator (gfx950, wave64).
//
// Set-up kernels (once per plan): k_small_tables, k_stage_tables, k_shape_agg;
//            k_quota_table    again whenever the availability changes.
// Hot path:  k_units<SCAN>    full-space fp32 evaluation + per-unit minima, early pruning
//            k_select_kth     radix select of the k-th smallest fp32 key
//            k_units<COLLECT> re-evaluates the few units that can hold a winner
//            k_refine         fp64 / exact-integer stage-by-stage re-evaluation
//            k_pick_best / k_rank_topk   final selection
//            k_eval_rows / k_eval_direct   per-candidate outputs for sailor_eval_batch
//                             (index ranges / index lists)
// Beside it: k_sim_1f1b       event-by-event 1F1B schedule of listed plans
//
// The simulator arithmetic follows Sailor, Sec. 4.3 (memory, iteration time, cost);
// T_pp = sum of stage times + (N_b - 1) * straggler is the 1F1B composition of
// Sec. 4.2.2 with the straggler counted N_b times in total.
#pragma once

#include <hip/hip_runtime.h>

#include "sailor_dev.h"

namespace sailor {

// ------------------------------------------------------------------ helpers

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fminf(v, __shfl_xor(v, off));
  return v;
}

__device__ __forceinline__ size_t agg_slot(const DevPlan &pl, uint32_t shape, int tp, int seg) {
  return ((size_t)shape * pl.TP + tp) * 3 + seg;
}

// Bandwidth a message of `bytes` sees from zone a to zone b: the link's fitted polynomial
// in log2(bytes) (cluster profiling, Sec. 4.1), kept inside [peak / 1000, peak]; the
// constant peak when the problem carries no polynomial.
__device__ __forceinline__ double link_bw(const DevPlan &pl, int a, int b, double bytes) {
  const double peak = pl.bw[a * pl.Z + b];
  if (pl.n_bw_coef <= 0 || bytes < 1.0) return peak;
  const double *c = pl.bw_poly + (size_t)(a * pl.Z + b) * pl.n_bw_coef;
  const double x = log2(bytes);
  double v = c[pl.n_bw_coef - 1];
  for (int k = pl.n_bw_coef - 2; k >= 0; --k) v = v * x + c[k];  // Horner
  // (ordered comparisons: the coefficients are validated finite and the device code is built
  // without NaN support, so the limits must not lean on how a NaN compares)
  if (v >= peak) v = peak;
  if (v <= peak * 1e-3) v = peak * 1e-3;
  return v;
}

// Bit q of the two-word mask of pool p (pool x pool relations for up to 128 pools).
__device__ __forceinline__ bool pool_bit(const uint64_t *mask, int p, int q) {
  return (mask[2 * p + (q >> 6)] >> (q & 63)) & 1ull;
}

// ------------------------------------------------------------------ set-up kernels

// Reciprocal bandwidths, two-way egress, and the per-(mb, dp, tp) scalars of a plan.
__global__ void k_small_tables(DevPlan pl) {
  const int t = threadIdx.x, nt = blockDim.x;
  const int Z = pl.Z;
  for (int i = t; i < Z * Z; i += nt) {
    int a = i / Z, b = i % Z;
    for (int m = 0; m < pl.MB; ++m) {
      const double bytes = (double)pl.p2p[m], bwv = link_bw(pl, a, b, bytes);
      pl.bwp[m * Z * Z + i] = bwv;
      pl.tsec_f[m * Z * Z + i] = (float)(bytes / bwv);
    }
    double e = 0.0;
    if (pl.egress && a != b) e = pl.egress[a * Z + b] + pl.egress[b * Z + a];
    pl.egs_f[i] = (float)e;
  }
  for (int g = t; g < pl.GX; g += nt) {
    const int ga = pl.xt[g] & 255, gb = pl.xt[g] >> 8;
    pl.price_f[g] = (float)(ga == gb ? pl.price[ga] : 0.5 * (pl.price[ga] + pl.price[gb]));
  }
  for (int p = t; p < pl.ZG; p += nt) {
    const int x = pl.xt[p % pl.GX], ga = x & 255, gb = x >> 8, z = p / pl.GX;
    uint32_t m = 0;  // H1: tensor parallelism stays inside a node
    for (int k = 0; k < pl.TP; ++k)
      if (pl.tpv[k] > pl.node[ga] || pl.tpv[k] > pl.node[gb]) m |= 1u << k;
    pl.h1m[p] = m;
    uint64_t im[2] = {0, 0};  // pools of the same zone with a real type in common (itself included)
    for (int q = 0; q < pl.ZG; ++q) {
      const int y = pl.xt[q % pl.GX], qa = y & 255, qb = y >> 8;
      if (q / pl.GX == z && (qa == ga || qa == gb || qb == ga || qb == gb)) im[q >> 6] |= 1ull << (q & 63);
    }
    pl.isect[2 * p] = im[0];
    pl.isect[2 * p + 1] = im[1];
  }
  for (int m = t; m < pl.MB; m += nt) {
    // N_b * D = B / mb whenever the batch divides; the product is exact in fp64 for
    // realistic sizes and is rounded once
    pl.xb_f[m] = (float)((double)(pl.B / pl.mbv[m]) * (double)pl.p2p[m]);
    uint32_t bits = 0;
    for (int d = 0; d < pl.DP; ++d) {
      int64_t per = (int64_t)pl.dpv[d] * pl.mbv[m];
      int32_t nb = (pl.B % per == 0) ? (int32_t)(pl.B / per) : 0;
      pl.nb[m * pl.DP + d] = nb;
      pl.nbm1_f[m * pl.DP + d] = (float)(nb - 1);
      if (nb > 0) bits |= 1u << d;
    }
    pl.divis[m] = bits;
  }
  for (int d = t; d < pl.DP; d += nt) {
    double D = (double)pl.dpv[d];
    pl.cd_f[d] = (float)(2.0 * (D - 1.0) / D);
    pl.dph_f[d] = (float)(D / 3600.0);
  }
}

struct StageArgs {
  const uint64_t *layer_params;  // [L]
  const double *t_fwd, *t_bwd;   // [G][MB][TP][Lc]
  const double *t_upd;           // [G][TP][Lc]
  const uint8_t *st_flags;       // bit 0: first stage of its row, bit 1: last
  uint64_t embed, head;
  int L, uniform;
};

// Per stage of every partition row: parameters, summed layer times per (type, mb, tp).
__global__ void k_stage_tables(DevPlan pl, StageArgs a) {
  const int rs = blockIdx.x;
  const int n = pl.st_n[rs], first = pl.st_first[rs];
  const int G = pl.G, MB = pl.MB, TP = pl.TP;
  if (threadIdx.x == 0) {
    uint64_t p = 0;
    for (int l = first; l < first + n; ++l) p += a.layer_params[l];
    if (a.st_flags[rs] & 1) p += a.embed;
    if (a.st_flags[rs] & 2) p += a.head;
    pl.st_params[rs] = p;
  }
  const int Lc = a.uniform ? 1 : a.L;
  for (int i = threadIdx.x; i < G * MB * TP; i += blockDim.x) {
    double f = 0.0, b = 0.0;
    if (a.uniform) {
      f = (double)n * a.t_fwd[i];
      b = (double)n * a.t_bwd[i];
    } else {
      const double *rf = a.t_fwd + (size_t)i * Lc, *rb = a.t_bwd + (size_t)i * Lc;
      for (int l = first; l < first + n; ++l) { f += rf[l]; b += rb[l]; }
    }
    pl.st_c[(size_t)rs * G * MB * TP + i] = f + b;
    pl.st_f[(size_t)rs * G * MB * TP + i] = f;
    pl.st_b[(size_t)rs * G * MB * TP + i] = b;
  }
  for (int i = threadIdx.x; i < G * TP; i += blockDim.x) {
    double u = 0.0;
    if (a.uniform) {
      u = (double)n * a.t_upd[i];
    } else {
      const double *ru = a.t_upd + (size_t)i * Lc;
      for (int l = first; l < first + n; ++l) u += ru[l];
    }
    pl.st_u[(size_t)rs * G * TP + i] = u;
  }
}

// model + activation bytes of a worker of stage i of P (Sec. 4.3) from the stage's parameter
// and layer counts; reserved bytes are added where the GPU type is known
__device__ __forceinline__ uint64_t stage_bytes_of(uint64_t params, int32_t layers, uint32_t bpp,
                                                   int i, int P, int tp, int64_t nb, uint64_t act) {
  const uint64_t shard = (params + (uint64_t)tp - 1) / (uint64_t)tp;
  const int64_t inflight = (int64_t)(P - i) < nb ? (int64_t)(P - i) : nb;
  return shard * (uint64_t)bpp + (uint64_t)inflight * (uint64_t)layers * act;
}

__device__ __forceinline__ uint64_t stage_bytes(const DevPlan &pl, uint32_t rs, int i, int P,
                                                int tp, int64_t nb, uint64_t act) {
  return stage_bytes_of(pl.st_params[rs + i], pl.st_n[rs + i], pl.bpp, i, P, tp, nb, act);
}

// Segment aggregates of one shape: everything of a segment that does not depend on
// the pool it is placed on.
__global__ void k_shape_agg(DevPlan pl) {
  const uint32_t shp = blockIdx.x;
  const ShapeRec sh = pl.shapes[shp];
  const int G = pl.G, GX = pl.GX, MB = pl.MB, TP = pl.TP, DP = pl.DP, P = sh.P;
  const int t = threadIdx.x, nt = blockDim.x;
  // need[tp][seg][mb][dp], syncz, upd
  for (int it = t; it < TP * 3 * MB * DP; it += nt) {
    int d = it % DP, m = (it / DP) % MB, seg = (it / (DP * MB)) % 3, k = it / (DP * MB * 3);
    uint64_t mx = 0;
    int64_t nb = pl.nb[m * DP + d];
    if (seg < sh.s && nb > 0) {
      uint64_t act = pl.act[m * TP + k];
      for (int i = sh.lo[seg]; i < sh.lo[seg] + sh.n[seg]; ++i) {
        uint64_t b = stage_bytes(pl, sh.row_stage, i, P, pl.tpv[k], nb, act);
        mx = b > mx ? b : mx;
      }
    }
    pl.need[(agg_slot(pl, shp, k, seg) * MB + m) * DP + d] = mx;
  }
  for (int it = t; it < TP * 3 * pl.Z; it += nt) {
    int z = it % pl.Z, seg = (it / pl.Z) % 3, k = it / (pl.Z * 3);
    double mx = 0.0;  // seconds of the slowest stage's gradient buffer over the zone's link
    if (seg < sh.s)
      for (int i = sh.lo[seg]; i < sh.lo[seg] + sh.n[seg]; ++i) {
        uint64_t shard = (pl.st_params[sh.row_stage + i] + pl.tpv[k] - 1) / (uint64_t)pl.tpv[k];
        const double bytes = (double)shard * (double)pl.gb;
        mx = fmax(mx, bytes / link_bw(pl, z, z, bytes));
      }
    pl.syncz[agg_slot(pl, shp, k, seg) * pl.Z + z] = (float)mx;
  }
  for (int it = t; it < TP * 3 * GX; it += nt) {
    int g = it % GX, seg = (it / GX) % 3, k = it / (GX * 3);
    const int ga = pl.xt[g] & 255, gb = pl.xt[g] >> 8;
    double mx = 0.0;
    if (seg < sh.s)
      for (int i = sh.lo[seg]; i < sh.lo[seg] + sh.n[seg]; ++i) {
        mx = fmax(mx, pl.st_u[((size_t)(sh.row_stage + i) * G + ga) * TP + k]);
        mx = fmax(mx, pl.st_u[((size_t)(sh.row_stage + i) * G + gb) * TP + k]);
      }
    pl.upd[agg_slot(pl, shp, k, seg) * GX + g] = (float)mx;
  }
  for (int it = t; it < TP * 3 * GX * MB; it += nt) {
    int m = it % MB, g = (it / MB) % GX, seg = (it / (MB * GX)) % 3, k = it / (MB * GX * 3);
    const int ga = pl.xt[g] & 255, gb = pl.xt[g] >> 8;
    float4 v = make_float4(0.f, 0.f, kNegInf, kNegInf);
    if (seg < sh.s) {
      const int lo = sh.lo[seg], n = sh.n[seg];
      double sum = 0.0, mxi = -__builtin_huge_val(), fst = 0.0, lst = 0.0;
      for (int i = lo; i < lo + n; ++i) {
        // replicas of two types: the slower one sets the stage's pace (straggler, Sec. 4.3)
        double c = fmax(pl.st_c[(((size_t)(sh.row_stage + i) * G + ga) * MB + m) * TP + k],
                        pl.st_c[(((size_t)(sh.row_stage + i) * G + gb) * MB + m) * TP + k]);
        sum += c;
        if (i == lo) fst = c;
        if (i == lo + n - 1) lst = c;
        if (i > lo && i < lo + n - 1) mxi = fmax(mxi, c);
      }
      v = make_float4((float)sum, (float)fst, (float)lst, (float)mxi);
    }
    pl.ta[(agg_slot(pl, shp, k, seg) * GX + g) * MB + m] = v;
  }
  __syncthreads();
  __threadfence();
  // memok bit d: largest worker of the segment fits the type's memory
  for (int it = t; it < TP * 3 * GX * MB; it += nt) {
    int m = it % MB, g = (it / MB) % GX, seg = (it / (MB * GX)) % 3, k = it / (MB * GX * 3);
    const int ga = pl.xt[g] & 255, gb = pl.xt[g] >> 8;
    uint32_t bits = 0;
    if (seg < sh.s)
      for (int d = 0; d < DP; ++d) {
        uint64_t need = pl.need[(agg_slot(pl, shp, k, seg) * MB + m) * DP + d];
        if (pl.nb[m * DP + d] > 0 && need + pl.res[ga] <= pl.cap[ga] && need + pl.res[gb] <= pl.cap[gb])
          bits |= 1u << d;
      }
    pl.memok[(agg_slot(pl, shp, k, seg) * GX + g) * MB + m] = bits;
  }
}

// ------------------------------------------------------------------ fp32 evaluation

struct Rec {       // one segment placed on one pool, for one (mb, tp); 32 bytes
  float sumT;      // sum of its stage times without the cross-segment transfers
  float tF, tL;    // first / last stage time without the cross-segment transfers
  float tI;        // slowest interior stage
  float syncb;     // slowest stage: gradient bytes / intra-zone bandwidth
  float upd;       // slowest update
  float pricen;    // stages * tp * $/h: rent of one replica of the segment
  uint32_t bits;   // bit d: valid for dp index d (memory, quota, batch, H1)
};

struct LaneC {     // scalars of a (mb, dp) pair
  float nbm1, cd, dph, xb;
};

__device__ __forceinline__ Rec make_rec(float4 ta, float sync, float upd, float price, float w,
                                        int n, int tp, uint32_t bits) {
  Rec r;  // w: seconds of one transfer inside the zone
  r.sumT = fmaf((float)(2 * (n - 1)), w, ta.x);
  r.tF = (n == 1) ? ta.y : ta.y + w;
  r.tL = (n == 1) ? kNegInf : ta.z + w;
  r.tI = (n >= 3) ? fmaf(2.0f, w, ta.w) : kNegInf;
  r.syncb = sync;
  r.upd = upd;
  r.pricen = (float)(n * tp) * price;
  r.bits = bits;
  return r;
}

// A segment record in LDS: two 16-byte halves in arrays of their own (the records a wave reads
// together then lie 16 bytes apart and spread over all banks; 32-byte records leave half of
// them idle) and the validity bits once more in a dense array for the tests that need
// nothing else.
__device__ __forceinline__ void rec_store(float4 *lo, float4 *hi, uint32_t *bits, int i, const Rec &r) {
  lo[i] = make_float4(r.sumT, r.tF, r.tL, r.tI);
  hi[i] = make_float4(r.syncb, r.upd, r.pricen, __uint_as_float(r.bits));
  bits[i] = r.bits;
}

__device__ __forceinline__ Rec rec_load(const float4 *lo, const float4 *hi, int i) {
  const float4 a = lo[i], b = hi[i];
  Rec r;
  r.sumT = a.x; r.tF = a.y; r.tL = a.z; r.tI = a.w;
  r.syncb = b.x; r.upd = b.y; r.pricen = b.z;
  r.bits = __float_as_uint(b.w);
  return r;
}

// Iteration time and cost of a plan, accumulated segment by segment.  Everything that
// depends only on the leading segments is finished before the pool of the next segment
// is known, so the scan hoists it out of its inner loops; the order of the floating
// point additions is fixed here, and both evaluation kernels go through these steps, so
// they return bit-identical values.
struct Acc {
  float tmax;  // slowest stage of the closed segments
  float sum;   // sum of stage times incl. the transfers across closed boundaries
  float syn, up, pr, egs;
  float tf, tl, ti;  // open segment: first / last / slowest interior stage
};

// the first segment
__device__ __forceinline__ Acc acc_begin(const Rec &r) {
  Acc a;
  a.tmax = kNegInf;
  a.sum = r.sumT;
  a.syn = r.syncb;
  a.up = r.upd;
  a.pr = r.pricen;
  a.egs = 0.f;
  a.tf = r.tF;
  a.tl = r.tL;
  a.ti = r.tI;
  return a;
}

// Closes the open segment over a boundary with transfer times wf (activations, sent by the
// open segment's last stage) and wb (gradients, sent by the next segment's first stage),
// and opens segment r behind it.
__device__ __forceinline__ Acc acc_cross(const Acc &p, const Rec &r, float wf, float wb, float eg,
                                         bool open_is_single, bool first_boundary) {
  Acc a;
  // a one-stage segment's only stage also pays the outgoing transfer (fma with an exact
  // 0 / 1 factor equals the plain sum)
  const float tf = fmaf(open_is_single ? 1.0f : 0.0f, wf, p.tf);
  a.tmax = fmaxf(p.tmax, fmaxf(fmaxf(tf, p.tl + wf), p.ti));
  a.sum = (p.sum + r.sumT) + (wf + wb);
  a.syn = fmaxf(p.syn, r.syncb);
  a.up = fmaxf(p.up, r.upd);
  a.pr = p.pr + r.pricen;
  a.egs = first_boundary ? eg : p.egs + eg;
  a.tf = r.tF + wb;
  a.tl = r.tL;
  a.ti = r.tI;
  return a;
}

// Closes the last segment: T_iter = T_pp + T_sync + T_update, C_iter = C_comp + C_comm.
__device__ __forceinline__ void acc_finish(const Acc &p, const LaneC &lc, float &T, float &C) {
  const float tmax = fmaxf(p.tmax, fmaxf(fmaxf(p.tf, p.tl), p.ti));
  const float tpp = fmaf(lc.nbm1, tmax, p.sum);
  T = fmaf(lc.cd, p.syn, tpp) + p.up;
  C = fmaf(p.pr * lc.dph, T, lc.xb * p.egs);
}

// Quota table, rebuilt whenever the availability changes: a replica that takes w GPUs
// from a pool (its stages there times their tensor-parallel degrees) can be placed for
// the data-parallel degrees whose bit is set (Sec. 4: resource quotas).
// A pool that is a pair of types gives half of the replicas from each (an even number of
// them); qh serves plans whose segments draw on one real pool together: x half-GPUs per
// replica of the plan fit the real pool for the degrees whose bit is set.
// gen: the availability generation (0 while the plan is built); when an entry of qh changes,
// row_gen[0] receives it, so that a scan can tell whether the shared-pool checks of a unit's
// last evaluation still hold.
__global__ void k_quota_table(DevPlan pl, const int32_t *avail, int32_t *avail_copy, uint32_t gen) {
  // avail: the table to build from -- pl.avail, or a newer one in host-mapped memory, which
  // is then also copied to avail_copy (= pl.avail) for the kernels that read it later; that
  // saves a separate upload in front of this kernel
  if (avail_copy && blockIdx.x == 0)
    for (int r = threadIdx.x; r < pl.ZGr; r += blockDim.x) avail_copy[r] = avail[r];
  const int n = (pl.W_max + 1) * pl.ZG;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const int p = i % pl.ZG, w = i / pl.ZG;
    const int x = pl.xt[p % pl.GX], ga = x & 255, gb = x >> 8, z = p / pl.GX;
    const int64_t avail_a = avail[z * pl.G + ga], avail_b = avail[z * pl.G + gb];
    uint32_t bits = 0;
    for (int d = 0; d < pl.DP; ++d) {
      const int64_t D = pl.dpv[d];
      if (ga == gb ? (int64_t)w * D <= avail_a
                   : (D % 2 == 0 && (int64_t)w * D <= 2 * avail_a && (int64_t)w * D <= 2 * avail_b))
        bits |= 1u << d;
    }
    pl.qw[i] = bits;
  }
  if (!pl.mixed) return;
  const int nh = (2 * pl.W_max + 1) * pl.ZGr;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < nh; i += gridDim.x * blockDim.x) {
    const int r = i % pl.ZGr, x = i / pl.ZGr;
    const int64_t avail2 = 2 * (int64_t)avail[r];
    uint32_t bits = 0;
    for (int d = 0; d < pl.DP; ++d)
      if ((int64_t)x * pl.dpv[d] <= avail2) bits |= 1u << d;
    if (gen == 0u) {
      pl.qh[i] = bits;
    } else if (pl.qh[i] != bits) {
      pl.qh[i] = bits;
      atomicMax(&pl.row_gen[0], gen);
    }
  }
}

// Plans whose segments draw on one real pool together (possible once pairs of types exist):
// bit d is set when dpv[d] replicas of all segments fit every real pool.  p[j], w[j]: pool and
// GPUs per replica of segment j.
__device__ __forceinline__ uint32_t joint_quota_bits(const DevPlan &pl, int n_seg, int p0, int p1,
                                                     int p2, int w0, int w1, int w2) {
  // six slots (two per segment) of (real pool, half-GPUs per replica); constant trip counts,
  // so that everything stays in registers
  int r[6], h[6];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int p = j == 0 ? p0 : (j == 1 ? p1 : p2), w = j == 0 ? w0 : (j == 1 ? w1 : w2);
    const bool used = j < n_seg;
    const int x = pl.xt[used ? p % pl.GX : 0], ga = x & 255, gb = x >> 8, z = used ? p / pl.GX : 0;
    r[2 * j] = z * pl.G + ga;
    r[2 * j + 1] = z * pl.G + gb;
    h[2 * j] = !used ? 0 : (ga == gb ? 2 * w : w);
    h[2 * j + 1] = (!used || ga == gb) ? 0 : w;
  }
  uint32_t bits = 0xFFFFFFFFu;
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    int total = 0;
#pragma unroll
    for (int k = 0; k < 6; ++k) total += (r[k] == r[i]) ? h[k] : 0;
    // (a pool that several slots name is checked several times against the same total)
    if (h[i] != 0) bits &= pl.qh[(size_t)total * pl.ZGr + r[i]];
  }
  return bits;
}

enum { MODE_SCAN = 0, MODE_COLLECT = 1 };

struct ScanArgs {
  float *umin_s, *umin_l;   // [n_units] minima over strictly / loosely constrained candidates
  uint32_t *counters;       // see Counter
  const uint32_t *tau_src;  // COLLECT: fp32 bits of the threshold, scaled by band ...
  float band;
  float tau_host;           // ... or, when use_tau_host is set, this threshold
  int use_tau_host;
  int count_only;           // COLLECT: count the candidates under the threshold, keep none
  uint32_t n_sub;           // COLLECT: workgroups that share one unit
  float lim_s, lim_l;       // constraint limits (strict, loose) on cost or on time
  SurvRec *surv;
  uint32_t surv_cap;
  float *ucost;             // SCAN, optional: ticks of the 100 MHz clock each unit took
  int ignore_quota;         // SCAN at plan creation: treat every pool as large enough
  const uint32_t *ulist;    // COLLECT, optional: the units to visit and, in counters[CNT_NLIST],
                            // how many; the grid then strides over the list
  uint32_t *unit_gen;       // SCAN, optional: per unit, the availability generation its minima
  uint32_t cur_gen;         // were computed at; a scan stamps what it computes with cur_gen
  uint32_t *unit_seq;       // SCAN, with unit_gen: per unit, the call that evaluated it last
  uint32_t call_seq;
  int incremental;          // SCAN: units whose validity bits come out as they were at their
                            // last evaluation keep their minima and are not evaluated again
  uint32_t *ubits;          // SCAN, with unit_gen: per unit, the validity bits of its records
  uint32_t ubits_stride;    // (and the shared-pool quota words) as last staged; words per unit
  uint32_t *near_list;      // SCAN, optional (best plan): units whose loose minimum lies within
  float near_band;          // near_band of the smallest strict key seen so far are appended
                            // here (count in counters[CNT_NLIST]); the running minimum only
                            // falls, so the list holds every unit within the band of the final one
  const float *ulb_con;     // SCAN, optional, with a constraint: per unit, the smallest value the
                            // constrained quantity takes on any plan of the unit that memory, node
                            // size and batch allow (availability ignored; the same fp32 arithmetic,
                            // so an exact bound): a unit whose bound fails the loose limit holds
                            // nothing and is not staged at all (Sec. 4.2.1, H3, applied to a unit)
  int direct;               // COLLECT without a scan before it: ulist names the only units whose
  uint32_t n_list_host;     // bound meets the limit (n_list_host of them); every candidate of
                            // theirs that is valid and within the loose limit is kept
  const float *ulb_key;     // SCAN, optional, with near_list: the same bound for the objective;
                            // a unit that cannot come within near_band of the running minimum
                            // is passed over
};

enum Counter { CNT_SURV = 0, CNT_REF = 1, CNT_FEAS = 2, CNT_GMIN = 3, CNT_TAU0 = 4, CNT_TAU1 = 5,
               CNT_NLOOSE = 6, CNT_NSTRICT = 7,  // count-only collect passes
               CNT_NLIST = 8,                    // length of the collect pass's unit list
               CNT_DONE = 9,                     // workgroups of the final kernel that have finished
               CNT_COUNT = 16 };

__device__ __forceinline__ uint32_t counter_reset_value(int i) {
  const int c = i % CNT_COUNT;
  return (c >= CNT_GMIN && c <= CNT_TAU1) ? 0x7f800000u : 0u;  // thresholds start at +inf
}

// zeroes the counters selected by mask (a fill kernel, usable under stream capture)
__global__ void k_zero_counters(uint32_t *c, uint32_t mask) {
  if (threadIdx.x < CNT_COUNT && ((mask >> threadIdx.x) & 1u)) c[threadIdx.x] = 0u;
}

__global__ void k_init_counters(uint32_t *c, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) c[i] = counter_reset_value(i);
}

// One candidate of the scan: update the running minima, or append it to the survivors.
template <int MODE, int OBJ, bool HASB>
__device__ __forceinline__ void visit(const ScanArgs &a, float T, float C, bool feas, float tau,
                                      uint64_t idx, uint32_t shape, float &ms, float &ml) {
  const float key = OBJ == 0 ? T : C;
  const float con = OBJ == 0 ? C : T;
  if (MODE == MODE_SCAN) {
    const float kf = feas ? key : kPosInf;
    if (HASB) {
      ms = fminf(ms, con <= a.lim_s ? kf : kPosInf);
      ml = fminf(ml, con <= a.lim_l ? kf : kPosInf);
    } else {
      ms = fminf(ms, kf);
    }
  } else {
    const bool loose = feas && (!HASB || con <= a.lim_l);
    if (a.count_only) {  // uniform
      const bool strict = !HASB || con <= a.lim_s;
      const uint64_t m_loose = __builtin_amdgcn_ballot_w64(loose && key <= tau);
      const uint64_t m_strict = __builtin_amdgcn_ballot_w64(loose && strict && key <= tau);
      if (m_loose != 0 && (threadIdx.x & 63) == 0) {
        atomicAdd(&a.counters[CNT_NLOOSE], (uint32_t)__popcll(m_loose));
        if (m_strict != 0) atomicAdd(&a.counters[CNT_NSTRICT], (uint32_t)__popcll(m_strict));
      }
    } else {
      // one atomic per wave: the first lane that keeps its candidate reserves the slots of all
      const bool take = loose && key <= tau;
      const uint64_t m_take = __builtin_amdgcn_ballot_w64(take);
      if (m_take == 0) return;
      const int lane = (int)(threadIdx.x & 63u), leader = __builtin_ctzll(m_take);
      uint32_t base = 0;
      if (lane == leader) base = atomicAdd(&a.counters[CNT_SURV], (uint32_t)__popcll(m_take));
      base = (uint32_t)__shfl((int)base, leader);
      if (!take) return;
      const bool strict = !HASB || con <= a.lim_s;
      const uint32_t slot = base + (uint32_t)__popcll(m_take & ((1ull << lane) - 1ull));
      if (slot < a.surv_cap) {
        SurvRec sv;
        sv.idx = idx;
        sv.key = strict ? key : kPosInf;
        sv.key_loose = key;
        sv.shape = shape;
        sv.pad = 0;
        a.surv[slot] = sv;
      }
    }
  }
}

// q = n / d for n * d < 2^32 with m = ceil(2^32 / d) (m = 0 encodes d = 1)
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t m) {
  return m ? __umulhi(n, m) : n;
}

struct LaneItem {  // what a lane owns for one chunk of the lane space
  int mb, dp, a1;
  bool active;
  LaneC lc;
  uint32_t dpbit;
};

// Lane item e of a lane space laid out as mb + MB * (a1 + n_a1 * dp): the dp digit is the
// slowest, so a wave holds one or two dp values and whole waves drop out together when
// their data-parallel degree cannot be placed.  mg = ceil(2^32 / (MB * n_a1)).
__device__ __forceinline__ LaneItem lane_item(const DevPlan &pl, int e, int n_items, int n_a1,
                                              uint32_t mg) {
  LaneItem it;
  it.active = e < n_items;
  const uint32_t ee = it.active ? (uint32_t)e : 0u;
  const uint32_t dp = fast_div(ee, mg), rem = ee - dp * (uint32_t)(pl.MB * n_a1);
  const uint32_t a1 = fast_div(rem, pl.mg_mb);
  it.a1 = (int)a1;
  it.dp = (int)dp;
  it.mb = (int)(rem - a1 * (uint32_t)pl.MB);
  it.lc.nbm1 = pl.nbm1_f[it.mb * pl.DP + it.dp];
  it.lc.cd = pl.cd_f[it.dp];
  it.lc.dph = pl.dph_f[it.dp];
  it.lc.xb = pl.xb_f[it.mb];
  it.dpbit = it.active ? (1u << it.dp) : 0u;
  return it;
}

__device__ __forceinline__ bool wave_any(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0; }

// The lanes of a workgroup own the (mb, pool of segment 1, dp) triples; the pools of the
// later segments are walked in uniform loops, so their record addresses, zones and
// transfer terms are the same for the whole wave.
//   one or two segments: lanes cover every pool 1; in the loop over pool 2 a lane whose own
//     pool equals it sits that iteration out;
//   three segments: pool 2 is the outer uniform loop, lanes cover the ZG - 1 other pools,
//     pool 3 is the inner uniform loop.
// Invalid plans are pruned early (cf. H2, Sec. 4.2.1): as soon as the validity bits of the
// segments placed so far are zero in every lane of a wave, the wave skips everything that
// depends on the remaining segments.
// With pairs of types (MIXED) different pools can draw on one real pool; the plans concerned
// (isect) get the joint quota check, the others keep the per-segment bits.
template <int S, int MODE, int OBJ, bool HASB, bool MIXED>
__device__ __forceinline__ void unit_body(const DevPlan &pl, const ScanArgs &a, const UnitRec &u,
                                          const float4 *rec_lo, const float4 *rec_hi,
                                          const uint32_t *rbits, const float4 *pair,
                                          const uint32_t *q13, const uint64_t *isect, int w0,
                                          int w1, int w2, float tau, int sub, int n_sub,
                                          float &ms, float &ml) {
  // the chunks of the lane space are dealt round-robin to the waves of the n_sub
  // workgroups that share the unit
  const int ZG = pl.ZG, G = pl.GX, MB = pl.MB, DP = pl.DP, Z = pl.Z;
  const int lane = threadIdx.x & 63;
  const int wave = (int)(threadIdx.x >> 6) + (int)(blockDim.x >> 6) * sub;
  const int nwave = (int)(blockDim.x >> 6) * n_sub;
  const bool single0 = u.n[0] == 1, single1 = u.n[1] == 1;
  const int tp = u.tp[0];
  const uint64_t ubase = u.base;
  if (S <= 2) {
    const int nin = MB * DP * ZG;
    for (int e0 = wave * 64; e0 < nin; e0 += nwave * 64) {
      const LaneItem it = lane_item(pl, e0 + lane, nin, ZG, pl.mg_mbzg);
      const int a1 = it.a1;
      const uint32_t b0 = rbits[a1 * MB + it.mb] & it.dpbit;
      if (!wave_any(b0 != 0)) continue;
      const Rec r0 = rec_load(rec_lo, rec_hi, a1 * MB + it.mb);
      const int z1 = (int)fast_div((uint32_t)a1, pl.mg_g);
      const float4 *pair1 = pair + (it.mb * Z + z1) * Z;  // transfers out of this lane's first zone
      const Acc A0 = acc_begin(r0);
      // index of the candidate whose outer digits are all zero
      const uint64_t idx0 = ubase + (uint64_t)(it.mb + MB * (tp + pl.TP * (it.dp + DP * a1)));
      if (S == 1) {
        float T, C;
        acc_finish(A0, it.lc, T, C);
        visit<MODE, OBJ, HASB>(a, T, C, b0 != 0, tau, idx0, u.shape, ms, ml);
        continue;
      }
      int z2 = u.o_lo / G, g2 = u.o_lo % G;
      for (int a2 = u.o_lo; a2 < u.o_lo + u.o_cnt; ++a2) {
        const int i1 = (ZG + a2) * MB + it.mb;
        uint32_t b1 = (a1 != a2) ? (b0 & rbits[i1]) : 0u;
        if (MIXED && b1 != 0 && pool_bit(isect, a2, a1))
          b1 &= joint_quota_bits(pl, 2, a1, a2, 0, w0, w1, 0);
        if (wave_any(b1 != 0)) {
          const Rec r1 = rec_load(rec_lo, rec_hi, i1);
          const float4 p12 = pair1[z2];
          const Acc A1 = acc_cross(A0, r1, p12.x, p12.y, p12.z, single0, true);
          int rel2 = a2 - a1 - 1;
          if (rel2 < 0) rel2 += ZG;
          float T, C;
          acc_finish(A1, it.lc, T, C);
          visit<MODE, OBJ, HASB>(a, T, C, b1 != 0, tau,
                                 idx0 + (uint64_t)pl.inner * (uint64_t)rel2, u.shape, ms, ml);
        }
        if (++g2 == G) { g2 = 0; ++z2; }
      }
    }
  } else {
    const int nin = MB * DP * (ZG - 1);
    int z2 = u.o_lo / G, g2 = u.o_lo % G;
    for (int a2 = u.o_lo; a2 < u.o_lo + u.o_cnt; ++a2) {

      for (int e0 = wave * 64; e0 < nin; e0 += nwave * 64) {
        const LaneItem it = lane_item(pl, e0 + lane, nin, ZG - 1, pl.mg_mbzg1);
        const int a1 = it.a1 + (it.a1 >= a2 ? 1 : 0);  // skip the pool of segment 2
        const int i0 = a1 * MB + it.mb, i1 = (ZG + a2) * MB + it.mb;
        const uint32_t b1 = rbits[i0] & it.dpbit & rbits[i1];
        if (!wave_any(b1 != 0)) continue;
        const Rec r0 = rec_load(rec_lo, rec_hi, i0);
        const Rec r1 = rec_load(rec_lo, rec_hi, i1);
        const int z1 = (int)fast_div((uint32_t)a1, pl.mg_g);
        const float4 *pairm = pair + it.mb * Z * Z;
        const float4 p12 = pairm[z1 * Z + z2];
        const Acc A1 = acc_cross(acc_begin(r0), r1, p12.x, p12.y, p12.z, single0, true);
        const uint32_t q13a = MIXED ? 0u : q13[a1];
        int rel2 = a2 - a1 - 1;
        if (rel2 < 0) rel2 += ZG;
        const uint64_t idx0 = ubase + (uint64_t)(it.mb + MB * (tp + pl.TP * (it.dp + DP * a1))) +
                              (uint64_t)pl.inner * (uint64_t)rel2;
        int z3 = 0, g3 = 0;
        for (int a3 = 0; a3 < ZG; ++a3) {
          if (a3 != a2) {  // uniform
            const int i2 = (2 * ZG + a3) * MB + it.mb;
            uint32_t b2 = b1 & rbits[i2];
            if (MIXED) {
              if (b2 != 0 && (pool_bit(isect, a2, a1) || pool_bit(isect, a2, a3) || pool_bit(isect, a3, a1)))
                b2 &= joint_quota_bits(pl, 3, a1, a2, a3, w0, w1, w2);
            } else if (a3 == a1) {
              b2 &= q13a;  // segments 1 and 3 share one pool's quota
            }
            if (wave_any(b2 != 0)) {
              const Rec r2 = rec_load(rec_lo, rec_hi, i2);
              const float4 p23 = pairm[z2 * Z + z3];
              const Acc A2 = acc_cross(A1, r2, p23.x, p23.y, p23.z, single1, false);
              int rel3 = a3 - a2 - 1;
              if (rel3 < 0) rel3 += ZG;
              float T, C;
              acc_finish(A2, it.lc, T, C);
              visit<MODE, OBJ, HASB>(a, T, C, b2 != 0, tau,
                                     idx0 + pl.stride3 * (uint64_t)rel3, u.shape, ms, ml);
            }
          }
          if (++g3 == G) { g3 = 0; ++z3; }
        }
      }
      if (++g2 == G) { g2 = 0; ++z2; }
    }
  }
}

// Records a scanned unit's minima and folds them into the global minimum (and, for the best
// plan, the list of units near it).  One thread.
__device__ __forceinline__ void unit_publish(const ScanArgs &a, uint32_t uidx, float ms, float ml) {
  // keys are non-negative, so their bit patterns order like unsigned integers
  // (a stale read only costs a redundant atomic; most units lose and skip theirs)
  const uint32_t seen = __hip_atomic_load(&a.counters[CNT_GMIN], __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
  if (__float_as_uint(ms) < seen) atomicMin(&a.counters[CNT_GMIN], __float_as_uint(ms));
  if (a.near_list && ml < kPosInf) {
    // (a stale `seen` is larger than the true running minimum and only lengthens the list)
    const float running = fminf(__uint_as_float(seen), ms);
    if (ml <= running * a.near_band) a.near_list[atomicAdd(&a.counters[CNT_NLIST], 1u)] = uidx;
  }
}

// LDS of a scan workgroup: the records of [3][ZG][MB] (segment, pool, mb) as two float4 arrays
// and a dense array of their validity bits, the transfer table, the shared-pool masks.
__host__ __device__ inline size_t unit_lds_records(int ZG, int MB) {
  return ((size_t)3 * ZG * MB + 3) & ~(size_t)3;  // a multiple of 4, so that what follows stays 16-byte aligned
}

// One workgroup per unit: stage the unit's segment records in LDS, then every lane walks
// its (mb, dp, pool 1) triple over the unit's outer pool digits.  Everything the staging
// needs comes from the unit record and tables that do not depend on one another, so all of
// its global loads are in flight together and one barrier ends it.
template <int MODE, int OBJ, bool HASB, bool MIXED>
__device__ __forceinline__ void unit_work(const DevPlan &pl, const ScanArgs &a, uint32_t uidx,
                                          int sub, uint32_t n_sub, uint4 *lds_raw) {
  const unsigned long long t_begin = (MODE == MODE_SCAN && a.ucost) ? wall_clock64() : 0ull;
  const UnitRec u = pl.units[uidx];
  float tau = kPosInf;
  if (MODE == MODE_SCAN && (a.ulb_con || a.ulb_key)) {
    bool dead = false;  // must come out the same in every wave of the workgroup
    if (HASB && a.ulb_con) dead = !(a.ulb_con[uidx] <= a.lim_l);
    if (a.ulb_key && a.near_list) {
      // the running minimum changes while the workgroup reads it: one thread reads, all follow
      __shared__ uint32_t s_seen;
      if (threadIdx.x == 0)
        s_seen = __hip_atomic_load(&a.counters[CNT_GMIN], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
      dead = dead || a.ulb_key[uidx] > __uint_as_float(s_seen) * a.near_band;
    }
    if (dead) {
      if (threadIdx.x == 0) {
        a.umin_s[uidx] = kPosInf;
        a.umin_l[uidx] = kPosInf;
        if (a.unit_gen) a.unit_gen[uidx] = a.cur_gen;  // (not counted as evaluated: unit_seq stays)
        if (a.ucost) a.ucost[uidx] = 0.f;
      }
      return;
    }
  }
  if (MODE == MODE_COLLECT) {
    tau = a.use_tau_host ? a.tau_host : __uint_as_float(*a.tau_src) * a.band;
    if (!a.direct) {  // (without a scan before this pass there are no minima to consult)
      const float um = a.umin_l[uidx];
      if (!(um < kPosInf && um <= tau)) return;  // uniform over the workgroup
    }
  }
  const int ZG = pl.ZG, G = pl.GX, MB = pl.MB, Z = pl.Z, S = u.s;
  const size_t n_rec = unit_lds_records(ZG, MB);
  float4 *rec_lo = reinterpret_cast<float4 *>(lds_raw);               // [S][ZG][MB], first halves
  float4 *rec_hi = rec_lo + n_rec;                                    // second halves
  uint32_t *rbits = reinterpret_cast<uint32_t *>(rec_hi + n_rec);     // validity bits alone
  float4 *pair = reinterpret_cast<float4 *>(rbits + n_rec);           // [MB][Z][Z]
  uint64_t *isect = reinterpret_cast<uint64_t *>(pair + MB * Z * Z);  // [ZG][2]
  uint32_t *q13 = reinterpret_cast<uint32_t *>(isect + 2 * ZG);       // [ZG]
  __shared__ float red[2][kMaxUnitThreads / 64];
  __shared__ uint32_t s_any[kMaxUnitThreads / 64];  // per wave, bit j: a pool can host segment j
  const int t = threadIdx.x;

  const int n0 = u.n[0], n1 = u.n[1], n2 = u.n[2];
  const int k0 = u.tp[0], k1 = u.tp[1], k2 = u.tp[2];            // tp index of each segment
  const int tv0 = pl.tpv[k0], tv1 = pl.tpv[k1], tv2 = pl.tpv[k2];
  const int w0 = n0 * tv0, w1 = n1 * tv1, w2 = n2 * tv2;        // GPUs of one replica
  // Re-planning after an availability change: the unit is staged as always, and if every
  // validity word comes out as at its last evaluation its minima still hold.  With pairs of
  // types the shared-pool table is read during the evaluation, not the staging: a unit of two
  // or three segments is evaluated again whenever that table has changed since.
  const bool joint_changed = MIXED && MODE == MODE_SCAN && a.incremental && S >= 2 &&
                             pl.row_gen[0] > a.unit_gen[uidx];
  const bool keep_bits = MODE == MODE_SCAN && a.ubits != nullptr;
  uint32_t *const ub = keep_bits ? a.ubits + (size_t)uidx * a.ubits_stride : nullptr;
  uint32_t any_here = 0;
  for (int i = t; i < S * ZG * MB; i += blockDim.x) {
    const uint32_t sp = fast_div((uint32_t)i, pl.mg_mb), mb = (uint32_t)i - sp * (uint32_t)MB;
    const int seg = sp >= 2u * ZG ? 2 : (sp >= (uint32_t)ZG ? 1 : 0), p = (int)sp - seg * ZG;
    const int z = (int)fast_div((uint32_t)p, pl.mg_g), g = p - z * G;
    const int k = seg == 0 ? k0 : (seg == 1 ? k1 : k2);
    const int w = seg == 0 ? w0 : (seg == 1 ? w1 : w2);
    const uint32_t sl = (u.shape * (uint32_t)pl.TP + (uint32_t)k) * 3u + (uint32_t)seg;
    const uint32_t gi = (sl * (uint32_t)G + (uint32_t)g) * (uint32_t)MB + mb;
    const float4 ta = pl.ta[gi];
    uint32_t q = a.ignore_quota ? 0xFFFFFFFFu : pl.qw[w * ZG + p];
    if ((pl.h1m[p] >> k) & 1u) q = 0;  // H1: tensor parallelism stays inside a node
    const uint32_t bits = pl.memok[gi] & q & pl.divis[mb];
    rec_store(rec_lo, rec_hi, rbits, i,
              make_rec(ta, pl.syncz[sl * Z + z], pl.upd[sl * G + g], pl.price_f[g],
                       pl.tsec_f[(mb * Z + z) * Z + z], seg == 0 ? n0 : (seg == 1 ? n1 : n2),
                       seg == 0 ? tv0 : (seg == 1 ? tv1 : tv2), bits));
    // a segment that no pool can host validly rules the whole unit out
    const bool counts = seg != 1 || (p >= (int)u.o_lo && p < (int)(u.o_lo + u.o_cnt));
    if (bits != 0 && counts) any_here |= 1u << seg;
    if (keep_bits && counts) {  // (segment 2's pools outside the unit's range do not concern it)
      if (!a.incremental) ub[i] = bits;
      else if (ub[i] != bits) { ub[i] = bits; any_here |= 8u; }
    }
  }
  if (S == 3 && !MIXED)
    for (int p = t; p < ZG; p += blockDim.x) {
      const uint32_t q = a.ignore_quota ? 0xFFFFFFFFu : pl.qw[(w0 + w2) * ZG + p];
      q13[p] = q;
      if (keep_bits) {
        uint32_t *const uq = ub + a.ubits_stride - ZG;  // behind the records' bits
        if (!a.incremental) uq[p] = q;
        else if (uq[p] != q) { uq[p] = q; any_here |= 8u; }
      }
    }
  if (MIXED)  // under ignore_quota no pool counts as shared
    for (int p = t; p < 2 * ZG; p += blockDim.x) isect[p] = a.ignore_quota ? 0ull : pl.isect[p];
  for (int i = t; i < MB * Z * Z; i += blockDim.x) {  // per mb: transfer a -> b, b -> a, egress
    const int m = i / (Z * Z), ab = i - m * Z * Z, za = ab / Z, zb = ab % Z;
    pair[i] = make_float4(pl.tsec_f[i], pl.tsec_f[(m * Z + zb) * Z + za], pl.egs_f[ab], 0.f);
  }
  {
    uint32_t wv = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)  // (bit 3: a validity word differs from the last evaluation's)
      if (__builtin_amdgcn_ballot_w64((any_here >> j) & 1u) != 0) wv |= 1u << j;
    if ((t & 63) == 0) s_any[t >> 6] = wv;
  }
  __syncthreads();
  uint32_t any_all = 0;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) any_all |= s_any[w];
  if (MODE == MODE_SCAN && a.incremental && !(any_all & 8u) && !joint_changed) {
    // every validity bit is what it was: the minima still hold (uniform over the workgroup)
    if (t == 0) unit_publish(a, uidx, a.umin_s[uidx], a.umin_l[uidx]);
    return;
  }
  any_all &= 7u;
  if (any_all != (1u << S) - 1u) {  // uniform over the workgroup
    if (MODE == MODE_SCAN && t == 0) {
      a.umin_s[uidx] = kPosInf;
      a.umin_l[uidx] = kPosInf;
      if (a.unit_gen) {
        a.unit_gen[uidx] = a.cur_gen;
        a.unit_seq[uidx] = a.call_seq;  // evaluated by this call
      }
      if (a.ucost) a.ucost[uidx] = (float)(wall_clock64() - t_begin);
    }
    return;
  }

  float ms = kPosInf, ml = kPosInf;
  // The unit's own share of the lane space, divided further among the n_sub workgroups.
  // Chunk c of the lane space goes to wave c mod (waves * n_shares), so with the part as the
  // fast digit of the share a part keeps the same chunks ((c / waves) mod n_parts == part)
  // whatever n_sub is: the collect pass must visit exactly what the scan saw.
  const int share = sub * (int)u.n_parts + (int)u.part, n_shares = (int)u.n_parts * (int)n_sub;
  if (S == 1) unit_body<1, MODE, OBJ, HASB, MIXED>(pl, a, u, rec_lo, rec_hi, rbits, pair, q13, isect, w0, w1, w2, tau, share, n_shares, ms, ml);
  else if (S == 2) unit_body<2, MODE, OBJ, HASB, MIXED>(pl, a, u, rec_lo, rec_hi, rbits, pair, q13, isect, w0, w1, w2, tau, share, n_shares, ms, ml);
  else unit_body<3, MODE, OBJ, HASB, MIXED>(pl, a, u, rec_lo, rec_hi, rbits, pair, q13, isect, w0, w1, w2, tau, share, n_shares, ms, ml);

  if (MODE == MODE_SCAN) {
    if (!HASB) ml = ms;
    ms = wave_min(ms);
    ml = wave_min(ml);
    if ((t & 63) == 0) { red[0][t >> 6] = ms; red[1][t >> 6] = ml; }
    __syncthreads();
    if (t == 0) {
      for (int w = 1; w < (int)(blockDim.x >> 6); ++w) {
        ms = fminf(ms, red[0][w]);
        ml = fminf(ml, red[1][w]);
      }
      a.umin_s[uidx] = ms;
      a.umin_l[uidx] = ml;
      if (a.unit_gen) {
        a.unit_gen[uidx] = a.cur_gen;
        a.unit_seq[uidx] = a.call_seq;  // evaluated by this call
      }
      unit_publish(a, uidx, ms, ml);
      if (a.ucost) a.ucost[uidx] = (float)(wall_clock64() - t_begin);
    }
  }
}

// SCAN: one workgroup per unit.  COLLECT: n_sub workgroups share a unit; with a unit list
// the grid strides over the list instead of covering every unit.
template <int MODE, int OBJ, bool HASB, bool MIXED>
__global__ __launch_bounds__(kMaxUnitThreads) void k_units(DevPlan pl, ScanArgs a) {
  extern __shared__ uint4 lds_raw[];
  if (MODE == MODE_SCAN) {
    unit_work<MODE, OBJ, HASB, MIXED>(pl, a, blockIdx.x, 0, 1u, lds_raw);
  } else if (!a.ulist) {
    unit_work<MODE, OBJ, HASB, MIXED>(pl, a, blockIdx.x / a.n_sub, (int)(blockIdx.x % a.n_sub), a.n_sub,
                               lds_raw);
  } else {
    const uint32_t n_list = a.direct ? a.n_list_host : a.counters[CNT_NLIST];
    const uint32_t per_round = gridDim.x / a.n_sub;
    const int sub = (int)(blockIdx.x % a.n_sub);
    for (uint32_t e = blockIdx.x / a.n_sub; e < n_list; e += per_round) {  // uniform
      unit_work<MODE, OBJ, HASB, MIXED>(pl, a, a.ulist[e], sub, a.n_sub, lds_raw);
      __syncthreads();  // the staging area is reused
    }
  }
}

// ------------------------------------------------------------------ k-th smallest key

// Radix select (11 + 11 + 10 bits) of the k-th smallest non-negative float among
// n = min(*count, cap) values read with a stride; +inf entries are ignored and fewer than
// k finite values yield +inf.  One workgroup of THREADS threads (1024 for thousands of values,
// 256 for a short list: fewer waves make the passes' barriers cheaper).  The result's bit pattern
// goes to *out.
// With a list: also writes the positions i < n_list_src whose list_src[i] is finite and at
// most result * band to list, and their number to *list_count (in no particular order).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_select_kth(const float *vals, int stride_words,
                                                     const uint32_t *count, uint32_t cap,
                                                     uint32_t k, uint32_t *out,
                                                     const float *list_src, uint32_t n_list_src,
                                                     float band, uint32_t *list,
                                                     uint32_t *list_count) {
  constexpr int kBinsPerThread = 2048 / THREADS, kWaves = THREADS / 64;
  __shared__ uint32_t hist[2048];
  __shared__ uint32_t wsum[kWaves];
  __shared__ uint32_t s_prefix, s_k, s_done, s_nlist;
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  // The first kSelectKeep values of every thread stay in registers for all three passes.
  // Their loads (and those of the list's source) do not wait for a count that comes from
  // memory: the buffers hold cap values, so the first value of every thread is requested
  // together with the count and taken as +inf afterwards if it lies beyond it (requesting
  // all kKept that way cost more than it saved when the list was short).
  constexpr int kSelectKeep = 8;
  constexpr uint32_t kKept = kSelectKeep * THREADS;
  uint32_t xr[kSelectKeep];
  float lr[kSelectKeep];
  const uint32_t n_early = count ? min(cap, (uint32_t)THREADS) : cap;
#pragma unroll
  for (int q = 0; q < kSelectKeep; ++q) {
    const uint32_t i = t + q * (uint32_t)THREADS;
    xr[q] = i < n_early ? __float_as_uint(vals[(size_t)i * stride_words]) : 0x7f800000u;
    lr[q] = (list && i < n_list_src) ? list_src[i] : kPosInf;
  }
  const uint32_t n = count ? min(*count, cap) : cap;
  if (t >= n) xr[0] = 0x7f800000u;
  if (count) {
#pragma unroll
    for (int q = 1; q < kSelectKeep; ++q) {
      const uint32_t i = t + q * (uint32_t)THREADS;
      if (i < n) xr[q] = __float_as_uint(vals[(size_t)i * stride_words]);
    }
  }
  if (t == 0) { s_prefix = 0; s_k = k; s_done = 0; s_nlist = 0; }
  const int shifts[3] = {21, 10, 0}, widths[3] = {11, 11, 10};
  for (int pass = 0; pass < 3; ++pass) {
#pragma unroll
    for (int b = 0; b < kBinsPerThread; ++b) hist[t + b * THREADS] = 0;
    __syncthreads();
    const int sh = shifts[pass], wd = widths[pass];
    const uint32_t prefix = s_prefix, kk = s_k;
    if (s_done) break;  // uniform
#pragma unroll
    for (int q = 0; q < kSelectKeep; ++q) {
      if ((uint32_t)q * (uint32_t)THREADS >= n) break;  // uniform: nothing is kept beyond the count
      const uint32_t x = xr[q];
      const bool match = x < 0x7f800000u && (pass == 0 || (x >> (sh + wd)) == prefix);
      const uint32_t bin = (x >> sh) & ((1u << wd) - 1);
      // Keys of a survivor list lie close together and share their leading digits: the
      // lanes that agree with the wave's first matching lane add to its bin once (hundreds
      // of atomics on one LDS word took 1 us per pass).
      const unsigned long long m = __builtin_amdgcn_ballot_w64(match);
      if (m == 0) continue;  // uniform over the wave
      const uint32_t bin0 = (uint32_t)__shfl((int)bin, __ffsll((long long)m) - 1);
      const bool same = match && bin == bin0;
      const unsigned long long ms = __builtin_amdgcn_ballot_w64(same);
      if (lane == __ffsll((long long)m) - 1) atomicAdd(&hist[bin0], (uint32_t)__popcll(ms));
      if (match && !same) atomicAdd(&hist[bin], 1u);
    }
    for (uint32_t i0 = t + kKept; i0 < n; i0 += 4u * blockDim.x) {  // four loads in flight
      uint32_t x4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t i = i0 + q * blockDim.x;
        x4[q] = i < n ? __float_as_uint(vals[(size_t)i * stride_words]) : 0x7f800000u;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t x = x4[q];
        const bool match = x < 0x7f800000u && (pass == 0 || (x >> (sh + wd)) == prefix);
        if (match) atomicAdd(&hist[(x >> sh) & ((1u << wd) - 1)], 1u);
      }
    }
    __syncthreads();
    // inclusive prefix sum over the bins, kBinsPerThread consecutive bins per thread
    uint32_t h[kBinsPerThread], mine = 0;
#pragma unroll
    for (int b = 0; b < kBinsPerThread; ++b) {
      h[b] = hist[kBinsPerThread * t + b];
      mine += h[b];
    }
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t v = __shfl_up(incl, off);
      if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wv; ++w) before += wsum[w];
    incl += before;
    uint32_t excl = incl - mine;
    if (excl < kk && kk <= incl) {  // exactly one thread: the k-th value lies in its bins
      int bin = 0;
#pragma unroll
      for (int b = 0; b < kBinsPerThread - 1; ++b)  // (constant subscripts: h stays in registers)
        if (bin == b && excl + h[b] < kk) { excl += h[b]; bin = b + 1; }
      s_prefix = (prefix << wd) | (uint32_t)(kBinsPerThread * t + bin);
      s_k = kk - excl;
    }
    if (t == THREADS - 1 && incl < kk) { s_done = 1; s_prefix = 0x7f800000u; }
    __syncthreads();
  }
  if (t == 0) *out = s_prefix;
  if (list) {
    __syncthreads();
    const float tau = __uint_as_float(s_prefix) * band;
#pragma unroll
    for (int q = 0; q < kSelectKeep; ++q) {
      const uint32_t i = t + q * (uint32_t)THREADS;
      if (lr[q] < kPosInf && lr[q] <= tau) list[atomicAdd(&s_nlist, 1u)] = i;
    }
    for (uint32_t i = t + kKept; i < n_list_src; i += blockDim.x) {
      const float v = list_src[i];
      if (v < kPosInf && v <= tau) list[atomicAdd(&s_nlist, 1u)] = i;
    }
    __syncthreads();
    if (t == 0) *list_count = s_nlist;
  }
}

// ------------------------------------------------------------------ fp64 re-evaluation

struct Cand {
  uint32_t shape;
  int P, s, mb, dp;          // indices into the value lists
  int tp[3];                 // tp index of each segment
  int a[3];
  int k1, k2;
};

// Element j of a three-element array by selects (a lane-dependent subscript would move the
// array to scratch memory).
template <typename T>
__device__ __forceinline__ int at3(const T *v, int j) {
  return j == 0 ? (int)v[0] : (j == 1 ? (int)v[1] : (int)v[2]);
}

// The digits of candidate idx, which lies in the given shape.
__device__ __forceinline__ void decode_in_shape(const DevPlan &pl, uint32_t shape, uint64_t idx,
                                                Cand &c) {
  const ShapeRec sh = pl.shapes[shape];
  const uint64_t rem = idx - sh.base;
  c.shape = shape;
  c.P = sh.P;
  c.s = sh.s;
  c.k1 = sh.k1;
  c.k2 = sh.k2;
  const uint32_t in = (uint32_t)(rem % pl.inner);
  uint32_t o = (uint32_t)(rem / pl.inner);
  c.mb = in % pl.MB;
  c.tp[0] = c.tp[1] = c.tp[2] = (in / pl.MB) % pl.TP;
  c.dp = (in / (pl.MB * pl.TP)) % pl.DP;
  c.a[0] = in / (pl.MB * pl.TP * pl.DP);
  c.a[1] = c.a[2] = -1;
  if (c.s >= 2) {
    c.a[1] = (c.a[0] + 1 + (int)(o % (pl.ZG - 1))) % pl.ZG;
    o /= (pl.ZG - 1);
    if (pl.pst) { c.tp[1] = (int)(o % pl.TP); o /= pl.TP; }
  }
  if (c.s == 3) {
    c.a[2] = (c.a[1] + 1 + (int)(o % (pl.ZG - 1))) % pl.ZG;
    o /= (pl.ZG - 1);
    if (pl.pst) c.tp[2] = (int)o;
  }
}

// Any index: find its block, then its shape.
__device__ __forceinline__ bool decode_index(const DevPlan &pl, uint64_t idx, Cand &c) {
  if (idx >= pl.N) return false;
  int b = 0;
  for (int i = 0; i < pl.n_blocks; ++i)
    if (idx >= pl.blocks[i].off) b = i;  // blocks are ordered and non-empty
  const BlockRec blk = pl.blocks[b];
  decode_in_shape(pl, blk.first_shape + (uint32_t)((idx - blk.off) / blk.shape_size), idx, c);
  return true;
}

constexpr int kRefineWaves = 4;  // waves per workgroup of k_refine

struct RefineLds {  // per-wave staging of the per-stage terms that are summed in stage order
  double t[kMaxStages], dol[kMaxStages], comm[kMaxStages];
};

__device__ __forceinline__ double wave_max_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off));
  return v;
}

// The two real types a | b << 8 of extended type x (the plain ones, then the pairs a < b in
// lexicographic order), by arithmetic: what DevPlan::xt holds, without the trip to memory
// in front of the loads that depend on it.
__device__ __forceinline__ int type_pair(int x, int G) {
  if (x < G) return x | (x << 8);
  int r = x - G, a = 0;
  while (a < G - 2 && r >= G - 1 - a) { r -= G - 1 - a; ++a; }
  return a | ((a + 1 + r) << 8);
}

// Stage-by-stage evaluation of one plan in fp64 and exact integers (Sec. 4.3) by one wave:
// lane i takes stages i, i + 64, ...; maxima are reduced across the wave, sums are taken in
// stage order (every lane adds the staged terms in the same order, so all lanes hold the
// same results).
__device__ __forceinline__ void eval_exact_wave(const DevPlan &pl, const Cand &c, int objective,
                                                int has_bound, double bound, RefineLds &lds,
                                                double &T, double &C, uint64_t &peak,
                                                uint32_t &mask) {
  const int G = pl.G, GX = pl.GX, Z = pl.Z, MB = pl.MB, TP = pl.TP, DP = pl.DP, P = c.P;
  const int lane = threadIdx.x & 63;
  const ShapeRec sh = pl.shapes[c.shape];
  const uint32_t rs = sh.row_stage;
  const int64_t D = pl.vals[c.dp];
  int xs[3];  // real types of each segment's pool
#pragma unroll
  for (int j = 0; j < 3; ++j) xs[j] = j < c.s ? type_pair(c.a[j] % GX, G) : 0;
  mask = 0;
  peak = 0;
  const int64_t nb = pl.nb[c.mb * DP + c.dp];
  const double p2p = (double)pl.p2p[c.mb];
  const double *bwp = pl.bwp + c.mb * Z * Z;  // bandwidth seen by a transfer of p2p bytes
  // quota per pool (GPUs of one replica there, times D) and H1
  // (counted in halves: a segment on a pair of types takes half of its replicas from each).
  // Everything read from memory is requested first, for all three segments at once: the
  // loads do not depend on one another, and a loop that fetched them as it went paid a trip
  // to memory for each.
  int zj[3], ga[3], gb[3];
  int64_t tpj[3], wj[3], av_a[3], av_b[3], nd_a[3], nd_b[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const bool used = j < c.s;
    ga[j] = xs[j] & 255;
    gb[j] = xs[j] >> 8;
    zj[j] = used ? c.a[j] / GX : 0;
    tpj[j] = used ? (int64_t)pl.vals[pl.DP + c.tp[j]] : 0;
    av_a[j] = used ? (int64_t)pl.avail[zj[j] * G + ga[j]] : 0;
    av_b[j] = used ? (int64_t)pl.avail[zj[j] * G + gb[j]] : 0;
    nd_a[j] = used ? (int64_t)pl.node[ga[j]] : 0;
    nd_b[j] = used ? (int64_t)pl.node[gb[j]] : 0;
  }
  if (nb == 0) {  // uniform over the wave (tested only now: the loads above need not wait for it)
    mask = 4u;    // batch not divisible
    T = C = __builtin_huge_val();
    return;
  }
#pragma unroll
  for (int j = 0; j < 3; ++j) wj[j] = (int64_t)sh.n[j] * tpj[j];
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    if (j >= c.s) continue;
#pragma unroll
    for (int slot = 0; slot < 2; ++slot) {
      if (slot == 1 && ga[j] == gb[j]) continue;
      const int g = slot == 0 ? ga[j] : gb[j];
      int64_t halves = 0;
#pragma unroll
      for (int j2 = 0; j2 < 3; ++j2) {
        if (j2 >= c.s || zj[j2] != zj[j]) continue;
        if (ga[j2] == gb[j2]) halves += ga[j2] == g ? 2 * wj[j2] : 0;
        else halves += (ga[j2] == g || gb[j2] == g) ? wj[j2] : 0;
      }
      if (halves * D > 2 * (slot == 0 ? av_a[j] : av_b[j])) mask |= 2u;
    }
    if (ga[j] != gb[j] && D % 2 != 0) mask |= 2u;  // D replicas cannot be halved
    if (tpj[j] > nd_a[j] || tpj[j] > nd_b[j]) mask |= 8u;
  }
  double max_t = 0.0, t_sync = 0.0, t_upd = 0.0;
  uint32_t oom = 0;
  for (int i = lane; i < P; i += 64) {
    const int seg = i < c.k1 ? 0 : (i < c.k2 ? 1 : 2);
    const int xg = at3(xs, seg), g = xg & 255, g2 = xg >> 8, z = at3(zj, seg);
    const int k = at3(c.tp, seg);
    const int64_t tp = at3(tpj, seg);
    // the zones of the neighbouring stages (the stage's own where there is none)
    const int sn = (i + 1) < c.k1 ? 0 : ((i + 1) < c.k2 ? 1 : 2);
    const int sp = (i - 1) < c.k1 ? 0 : ((i - 1) < c.k2 ? 1 : 2);
    const int zn = i < P - 1 ? at3(zj, sn) : z, zp = i > 0 ? at3(zj, sp) : z;
    // everything the stage reads from memory, requested together
    const size_t si = (size_t)rs + i;
    const uint64_t params = pl.st_params[si];
    const int32_t layers = pl.st_n[si];
    const uint64_t act = pl.act[c.mb * TP + k];
    const uint64_t res1 = pl.res[g], res2 = pl.res[g2], cap1 = pl.cap[g], cap2 = pl.cap[g2];
    const double c1 = pl.st_c[((si * G + g) * MB + c.mb) * TP + k];
    const double c2 = pl.st_c[((si * G + g2) * MB + c.mb) * TP + k];
    const double u1 = pl.st_u[(si * G + g) * TP + k], u2 = pl.st_u[(si * G + g2) * TP + k];
    const double price1 = pl.price[g], price2 = pl.price[g2];
    const double bw_n = bwp[z * Z + zn], bw_p = bwp[z * Z + zp];
    const double eg = pl.egress ? pl.egress[z * Z + zn] + pl.egress[zn * Z + z] : 0.0;
    const uint64_t bytes_i = stage_bytes_of(params, layers, pl.bpp, i, P, (int)tp, nb, act);
    const uint64_t m = bytes_i + res1, m2 = bytes_i + res2;  // both replica types
    if (m > cap1 || m2 > cap2) oom = 1u;
    peak = m > peak ? m : peak;
    peak = m2 > peak ? m2 : peak;
    double x = 0.0, comm = 0.0;
    if (i < P - 1) {
      x += p2p / bw_n;
      if (pl.egress && zn != z) comm = (double)nb * (double)D * p2p * eg;
    }
    if (i > 0) x += p2p / bw_p;
    // the slower replica type sets the stage's pace (straggler, Sec. 4.3)
    const double t = fmax(c1, c2) + x;
    max_t = fmax(max_t, t);
    if (D > 1) {
      const uint64_t shard = (params + (uint64_t)tp - 1) / (uint64_t)tp;
      const double bytes = (double)shard * (double)pl.gb;
      const double sync = 2.0 * (double)(D - 1) / (double)D * bytes / link_bw(pl, z, z, bytes);
      t_sync = fmax(t_sync, sync);
    }
    t_upd = fmax(t_upd, u1);
    t_upd = fmax(t_upd, u2);
    lds.t[i] = t;
    lds.dol[i] = g == g2 ? (double)(D * tp) * price1 : (double)(D * tp) * (0.5 * (price1 + price2));
    lds.comm[i] = comm;
  }
  if (__builtin_amdgcn_ballot_w64(oom != 0) != 0) mask |= 1u;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint64_t o = __shfl_xor((unsigned long long)peak, off);
    peak = o > peak ? o : peak;
  }
  max_t = wave_max_f64(max_t);
  t_sync = wave_max_f64(t_sync);
  t_upd = wave_max_f64(t_upd);
  // LDS operations of one wave complete in order; the fence keeps the compiler from
  // moving the reads above the writes
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  double sum_t = 0.0, dollars = 0.0, comm = 0.0;
#pragma unroll 8
  for (int i = 0; i < P; ++i) {  // (unrolled so that the LDS reads run ahead of the additions)
    sum_t += lds.t[i];
    dollars += lds.dol[i];
    comm += lds.comm[i];
  }
  T = (sum_t + (double)(nb - 1) * max_t) + t_sync + t_upd;
  C = dollars / 3600.0 * T + comm;
  if (has_bound) {
    if (objective == 0) { if (C > bound) mask |= 32u; }
    else if (1.0 / T < bound) mask |= 32u;
  }
  __builtin_amdgcn_wave_barrier();  // the staging arrays are reused by the next candidate
}

struct RefineArgs {
  const SurvRec *surv;
  uint32_t surv_cap;
  uint32_t *counters;
  const uint32_t *tau_src;  // NULL: take every survivor
  float band;
  RefRec *ref;
  uint32_t ref_cap;
  int objective, has_bound;
  double bound;
};

// One wave per survivor.
__global__ __launch_bounds__(kRefineWaves * 64) void k_refine(DevPlan pl, RefineArgs a) {
  __shared__ RefineLds lds[kRefineWaves];
  const uint32_t wave = blockIdx.x * kRefineWaves + (threadIdx.x >> 6);
  const uint32_t n_waves = gridDim.x * kRefineWaves;
  // the wave's first record is requested together with the count (the buffer holds surv_cap
  // records, so the address is valid whatever the count turns out to be)
  SurvRec first{};
  if (wave < a.surv_cap) first = a.surv[wave];
  const uint32_t n = min(a.counters[CNT_SURV], a.surv_cap);
  const float tau = a.tau_src ? __uint_as_float(*a.tau_src) * a.band : kPosInf;
  for (uint32_t i = wave; i < n; i += n_waves) {
    const SurvRec sv = i == wave ? first : a.surv[i];
    if (!(sv.key_loose <= tau)) continue;
    Cand c;
    decode_in_shape(pl, sv.shape, sv.idx, c);
    RefRec r;
    r.idx = sv.idx;
    r.pad = 0;
    eval_exact_wave(pl, c, a.objective, a.has_bound, a.bound, lds[threadIdx.x >> 6], r.T, r.C,
                    r.mem, r.mask);
    if ((threadIdx.x & 63) == 0) {
      const uint32_t slot = atomicAdd(&a.counters[CNT_REF], 1u);
      if (slot < a.ref_cap) {  // (a record that does not fit is counted in CNT_REF only: the
        a.ref[slot] = r;       // host reports the overflow, the ranking sees what was stored)
        if (r.mask == 0) atomicAdd(&a.counters[CNT_FEAS], 1u);
      }
    }
  }
}

__device__ __forceinline__ bool lex_less(double ka, uint64_t ia, double kb, uint64_t ib) {
  return ka < kb || (ka == kb && ia < ib);
}

// The host waits for the results by polling hdr->seq in host-mapped memory, which saves the
// few microseconds between a kernel's last store and the completion of its dispatch; the
// sequence number is therefore stored last, behind a system-scope fence.
__device__ __forceinline__ void publish(ResultHeader *hdr, uint32_t seq) {
  __threadfence_system();
  __hip_atomic_store(&hdr->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Best plan: minimum fp64 key over valid candidates, then the lowest index within the
// tie tolerance of it.  One workgroup; results go to host-mapped memory.
__global__ __launch_bounds__(1024) void k_pick_best(const RefRec *ref, uint32_t ref_cap,
                                                    const uint32_t *counters,
                                                    uint32_t *next_counters, int objective,
                                                    ResultHeader *hdr, RefRec *out, uint32_t seq) {
  __shared__ double s_key[16];
  __shared__ unsigned long long s_idx[16];
  __shared__ uint32_t s_pos[16];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  // a thread's first record is requested together with the counters (the buffer holds
  // ref_cap records, so the address is valid whatever the count turns out to be)
  RefRec mine{};
  if ((uint32_t)t < ref_cap) mine = ref[t];
  const uint32_t n_ref = counters[CNT_REF], n_surv = counters[CNT_SURV],
                 n_feas = counters[CNT_FEAS], gmin = counters[CNT_GMIN];
  const uint32_t n = min(n_ref, ref_cap);
  if (t < CNT_COUNT) next_counters[t] = counter_reset_value(t);  // for the next call
  double best = __builtin_huge_val();
  if ((uint32_t)t < n && mine.mask == 0) best = objective == 0 ? mine.T : mine.C;
  for (uint32_t i = t + blockDim.x; i < n; i += blockDim.x)
    if (ref[i].mask == 0) best = fmin(best, objective == 0 ? ref[i].T : ref[i].C);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) best = fmin(best, __shfl_xor(best, off));
  if (lane == 0) s_key[wv] = best;
  __syncthreads();
  best = s_key[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) best = fmin(best, s_key[w]);
  const double limit = best * (1.0 + kTieTol);
  unsigned long long bi = ~0ull;
  uint32_t bp = 0;
  if ((uint32_t)t < n && mine.mask == 0 && (objective == 0 ? mine.T : mine.C) <= limit) {
    bi = mine.idx;
    bp = t;
  }
  for (uint32_t i = t + blockDim.x; i < n; i += blockDim.x) {
    const double key = objective == 0 ? ref[i].T : ref[i].C;
    if (ref[i].mask == 0 && key <= limit && ref[i].idx < bi) { bi = ref[i].idx; bp = i; }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long oi = __shfl_xor(bi, off);
    const uint32_t op = __shfl_xor(bp, off);
    if (oi < bi) { bi = oi; bp = op; }
  }
  if (lane == 0) { s_idx[wv] = bi; s_pos[wv] = bp; }
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 16; ++w)
      if (s_idx[w] < bi) { bi = s_idx[w]; bp = s_pos[w]; }
    const bool found = bi != ~0ull;
    if (found) {
      if (bp == 0) out[0] = mine;  // (thread 0 holds record 0)
      else out[0] = ref[bp];
    }
    hdr->n_found = found ? 1u : 0u;
    hdr->surv_count = n_surv;
    hdr->ref_count = n_ref;
    hdr->feasible_count = n_feas;
    hdr->gmin_bits = gmin;
    publish(hdr, seq);
  }
}

constexpr uint32_t kRankLds = 1024;  // records the one-workgroup form of k_rank_topk takes

// Top-k: the rank of every valid re-evaluated candidate in ascending (key, index) order.
// Launched as one workgroup of kRankLds threads when few records are expected (small k):
// keys and indices go to LDS, the threads share out the counting of each record's
// predecessors, and the k first are copied to host-mapped memory in rank order.  Otherwise (several workgroups,
// or more than kRankLds records) one wave per candidate: its lanes count, in strides over
// the list, the entries that precede it; ranks below k go to a device-side list, which the
// workgroup that finishes last copies to host-mapped memory in one coalesced pass
// (scattered 40-byte stores over the bus, each behind its own fence, cost 20 us for 500
// records).
__global__ __launch_bounds__(kRankLds) void k_rank_topk(const RefRec *ref, uint32_t ref_cap,
                                                        const uint32_t *counters,
                                                        uint32_t *next_counters, int objective,
                                                        uint32_t k, ResultHeader *hdr, RefRec *out,
                                                        RefRec *staged, uint32_t *done,
                                                        uint32_t seq) {
  __shared__ uint32_t s_last;
  __shared__ double s_key[kRankLds];
  __shared__ unsigned long long s_idx[kRankLds];
  __shared__ uint16_t s_opos[kRankLds];
  __shared__ uint32_t s_before[kRankLds];
  // (one-workgroup form) a thread's record is requested together with the count: the
  // buffer holds ref_cap records, so the address is valid whatever the count turns out to be
  RefRec mine{};
  if (gridDim.x == 1 && threadIdx.x < ref_cap) mine = ref[threadIdx.x];
  const uint32_t n_ref = counters[CNT_REF];
  const uint32_t n = min(n_ref, ref_cap);
  const uint32_t f = counters[CNT_FEAS];  // valid stored records (requested with the count)
  const bool overflow = n_ref > ref_cap;  // uniform: the list is incomplete, nothing is ranked
  if (blockIdx.x == 0 && threadIdx.x < CNT_COUNT)
    next_counters[threadIdx.x] = counter_reset_value(threadIdx.x);  // for the next call
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    hdr->n_found = overflow ? 0u : (f < k ? f : k);
    hdr->surv_count = counters[CNT_SURV];
    hdr->ref_count = n_ref;
    hdr->feasible_count = f;
    hdr->gmin_bits = counters[CNT_GMIN];
  }
  if (overflow) {  // the host turns ref_count > ref_cap into SAILOR_ENOMEM
    if (gridDim.x == 1) {
      if (threadIdx.x == 0) publish(hdr, seq);
      return;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      __threadfence_system();
      s_last = atomicAdd(done, 1u) == gridDim.x - 1 ? 1u : 0u;
      if (s_last) publish(hdr, seq);
    }
    return;
  }
  if (gridDim.x == 1 && n <= kRankLds) {  // uniform
    const uint32_t t = threadIdx.x;
    if (t < n) {
      const bool ok = mine.mask == 0;
      s_key[t] = ok ? (objective == 0 ? mine.T : mine.C) : __builtin_huge_val();
      s_idx[t] = ok ? mine.idx : ~0ull;
    }
    s_before[t] = 0;
    __syncthreads();
    // the workgroup's threads form rows of np >= n threads (a power of two); row r counts,
    // for record q, the predecessors among records r, r + rows, ...
    uint32_t np = 64;
    while (np < n) np <<= 1;
    const uint32_t q = t & (np - 1), row = t / np, rows = kRankLds / np;
    if (q < n && s_idx[q] != ~0ull) {
      const double mk = s_key[q];
      const unsigned long long mi = s_idx[q];
      uint32_t before = 0;
#pragma unroll 4
      for (uint32_t j = row; j < n; j += rows) before += lex_less(s_key[j], s_idx[j], mk, mi) ? 1u : 0u;
      if (before) atomicAdd(&s_before[q], before);
    }
    __syncthreads();
    if (t < n && s_idx[t] != ~0ull && s_before[t] < k) s_opos[s_before[t]] = (uint16_t)t;
    __syncthreads();
    const uint32_t n_out = f < k ? f : k;  // n_out <= n
    constexpr uint32_t kWords = sizeof(RefRec) / 8;
    for (uint32_t w = threadIdx.x; w < n_out * kWords; w += blockDim.x)
      reinterpret_cast<unsigned long long *>(out)[w] =
          reinterpret_cast<const unsigned long long *>(ref + s_opos[w / kWords])[w % kWords];
    // One system-scope fence for the workgroup (each costs a fraction of a microsecond per
    // wave that executes it): the stores above are ordered before thread 0's fence by a
    // workgroup-scope release and the barrier.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0) publish(hdr, seq);
    return;
  }
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const uint32_t n_waves = gridDim.x * (blockDim.x >> 6);
  bool wrote = false;
  for (uint32_t i = wave; i < n; i += n_waves) {
    const RefRec r = ref[i];
    if (r.mask != 0) continue;  // uniform over the wave
    const double mk = objective == 0 ? r.T : r.C;
    uint32_t before = 0;
    for (uint32_t j = lane; j < n; j += 64) {
      const RefRec &o = ref[j];
      if (o.mask == 0 && lex_less(objective == 0 ? o.T : o.C, o.idx, mk, r.idx)) ++before;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) before += __shfl_xor(before, off);
    if (lane == 0 && before < k) {
      staged[before] = r;
      wrote = true;
    }
  }
  if (wrote) __threadfence();  // visible to the other workgroups before this one counts as done
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence_system();  // (workgroup 0: the header fields above are on their way)
    s_last = atomicAdd(done, 1u) == gridDim.x - 1 ? 1u : 0u;
  }
  __syncthreads();
  if (!s_last) return;  // uniform
  __threadfence();      // the last workgroup: see what the others staged
  const uint32_t n_out = f < k ? f : k;
  const unsigned long long *src = reinterpret_cast<const unsigned long long *>(staged);
  unsigned long long *dst = reinterpret_cast<unsigned long long *>(out);
  for (uint32_t i = threadIdx.x; i < n_out * (uint32_t)(sizeof(RefRec) / 8); i += blockDim.x)
    dst[i] = __builtin_nontemporal_load(src + i);
  __threadfence_system();
  __syncthreads();
  if (threadIdx.x == 0) publish(hdr, seq);
}

// ------------------------------------------------------------------ event-by-event 1F1B

struct SimArgs {
  uint64_t count;
  const uint64_t *indices;
  double *t_event, *t_closed;  // either may be NULL
  double *rings;               // NULL: the rings live in LDS; else [count][2][P_max][ring] doubles
  int ring;                    // slots per stage, a power of two > P_max
  int p_max;
};

// The op a stage runs at position pos of its 1F1B order: warm-up forwards, then one forward
// and one backward in turn, then the remaining backwards.  Returns true for a backward.
__device__ __forceinline__ bool sim_op_at(int P, int M, int i, int pos, int &m) {
  const int w = min(P - 1 - i, M);
  if (pos < w) { m = pos; return false; }
  const int q = pos - w;
  if (q < 2 * (M - w)) {
    m = (q & 1) ? (q >> 1) : w + (q >> 1);
    return (q & 1) != 0;
  }
  m = (M - w) + (q - 2 * (M - w));
  return true;
}

// The 1F1B schedule of one pipeline of a plan, op by op (warm-up, steady and cool-down phases,
// Sec. 4.3), beside the closed form of Sec. 4.2.2 on the same stage times.  One workgroup per
// candidate, one thread per stage.  A forward of stage i takes its layers' forward time plus the
// transfer to stage i + 1, a backward its backward time plus the transfer to stage i - 1; a
// forward waits for the previous stage's forward of the same microbatch, a backward for the next
// stage's backward.  The schedule advances in rounds: in a round every stage runs its next op if
// what it waits for was finished in an earlier round.  End times travel between neighbouring
// stages through rings indexed by microbatch; a producer is never more than P ops ahead of its
// consumer, so `ring` > P slots per stage suffice.  At most 2 (N_b + P) rounds are needed.
__global__ __launch_bounds__(256) void k_sim_1f1b(DevPlan pl, SimArgs a) {
  extern __shared__ double sim_lds[];
  __shared__ double s_t[kMaxStages];
  __shared__ int s_fc[kMaxStages], s_bc[kMaxStages];  // forwards / backwards a stage has finished
  __shared__ double s_red[4];
  const uint64_t ci = blockIdx.x;
  if (ci >= a.count) return;
  const int i = threadIdx.x;
  const uint64_t idx = a.indices[ci];
  Cand c;
  if (!decode_index(pl, idx, c)) {  // uniform over the workgroup
    if (i == 0) {
      if (a.t_event) a.t_event[ci] = __builtin_nan("");
      if (a.t_closed) a.t_closed[ci] = __builtin_nan("");
    }
    return;
  }
  const int P = c.P, G = pl.G, GX = pl.GX, Z = pl.Z, MB = pl.MB, TP = pl.TP;
  const int M = pl.nb[c.mb * pl.DP + c.dp];
  if (M == 0) {  // the batch does not divide
    if (i == 0) {
      if (a.t_event) a.t_event[ci] = __builtin_huge_val();
      if (a.t_closed) a.t_closed[ci] = __builtin_huge_val();
    }
    return;
  }
  const ShapeRec sh = pl.shapes[c.shape];
  const bool mine = i < P;
  double fdur = 0.0, bdur = 0.0;
  if (mine) {
    const int seg = i < c.k1 ? 0 : (i < c.k2 ? 1 : 2);
    const int xg = pl.xt[at3(c.a, seg) % GX], g = xg & 255, g2 = xg >> 8, z = at3(c.a, seg) / GX, k = at3(c.tp, seg);
    const size_t at = (((size_t)(sh.row_stage + i) * G + g) * MB + c.mb) * TP + k;
    const size_t at2 = (((size_t)(sh.row_stage + i) * G + g2) * MB + c.mb) * TP + k;
    const double p2p = (double)pl.p2p[c.mb];
    const double *bwp = pl.bwp + c.mb * Z * Z;
    double send_f = 0.0, send_b = 0.0;
    if (i < P - 1) {
      const int sn = (i + 1) < c.k1 ? 0 : ((i + 1) < c.k2 ? 1 : 2);
      send_f = p2p / bwp[z * Z + at3(c.a, sn) / GX];
    }
    if (i > 0) {
      const int sp = (i - 1) < c.k1 ? 0 : ((i - 1) < c.k2 ? 1 : 2);
      send_b = p2p / bwp[z * Z + at3(c.a, sp) / GX];
    }
    double f = pl.st_f[at], b = pl.st_b[at];
    if (g2 != g && pl.st_f[at2] + pl.st_b[at2] > f + b) {  // the pipeline through the slower type
      f = pl.st_f[at2];
      b = pl.st_b[at2];
    }
    fdur = f + send_f;
    bdur = b + send_b;
    s_t[i] = f + b + (send_f + send_b);
    s_fc[i] = 0;
    s_bc[i] = 0;
  }
  __syncthreads();
  if (i == 0 && a.t_closed) {  // sums in stage order
    double sum_t = 0.0, max_t = 0.0;
    for (int j = 0; j < P; ++j) {
      sum_t += s_t[j];
      max_t = fmax(max_t, s_t[j]);
    }
    a.t_closed[ci] = sum_t + (double)(M - 1) * max_t;
  }
  double *ring_f = a.rings ? a.rings + ci * 2 * (size_t)a.p_max * a.ring : sim_lds;
  double *ring_b = ring_f + (size_t)a.p_max * a.ring;
  const int rmask = a.ring - 1;
  int pos = 0;
  double free_at = 0.0;
  for (int round = 0; round < 2 * (M + P) + 4; ++round) {  // the bound is never reached
    bool ready = false, bwd = false;
    int m = 0;
    double dep = 0.0;
    if (mine && pos < 2 * M) {
      bwd = sim_op_at(P, M, i, pos, m);
      if (!bwd) {
        if (i == 0) ready = true;
        else if (s_fc[i - 1] > m) { ready = true; dep = ring_f[(size_t)(i - 1) * a.ring + (m & rmask)]; }
      } else {
        if (i == P - 1) { ready = true; dep = ring_f[(size_t)i * a.ring + (m & rmask)]; }
        else if (s_bc[i + 1] > m) { ready = true; dep = ring_b[(size_t)(i + 1) * a.ring + (m & rmask)]; }
      }
    }
    __syncthreads();  // every stage has read before any stage writes
    if (ready) {
      const double start = fmax(free_at, dep);
      free_at = start + (bwd ? bdur : fdur);
      if (bwd) { ring_b[(size_t)i * a.ring + (m & rmask)] = free_at; s_bc[i] += 1; }
      else { ring_f[(size_t)i * a.ring + (m & rmask)] = free_at; s_fc[i] += 1; }
      pos += 1;
    }
    if (!__syncthreads_or(ready ? 1 : 0)) break;  // nothing moved: every stage is done
  }
  // makespan: the latest stage
  double end = mine ? free_at : 0.0;
  end = wave_max_f64(end);
  if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = end;
  __syncthreads();
  if (i == 0 && a.t_event) {
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) end = fmax(end, s_red[w]);
    a.t_event[ci] = end;
  }
}

// ------------------------------------------------------------------ eval_batch

// "iterations per second below the floor", decided the same way by both evaluation kernels
// (a product instead of a division; the two differ only for values within rounding of the
// floor)
__device__ __forceinline__ bool throughput_below(float T, float floor_) { return T * floor_ > 1.0f; }

struct EvalArgs {
  uint64_t first, count;
  const uint64_t *indices;
  float *time, *cost;
  uint64_t *mem;
  uint32_t *mask;
  int objective, has_bound;
  float bound;
};

template <int S>
__device__ __forceinline__ void eval_direct_s(const DevPlan &pl, const Cand &c, const ShapeRec &sh,
                                              const LaneC &lc, float &T, float &C, uint64_t &peak,
                                              uint32_t &mask) {
  const int GX = pl.GX, Z = pl.Z, MB = pl.MB, DP = pl.DP;
  const int64_t D = pl.vals[c.dp];
  const float *ts = pl.tsec_f + c.mb * Z * Z;  // transfer seconds of this microbatch size
  Acc acc;
  int w[3] = {0, 0, 0};
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int p = c.a[j], gx = p % GX, z = p / GX;
    const int ga = pl.xt[gx] & 255, gb = pl.xt[gx] >> 8;
    const int tpv = pl.vals[pl.DP + c.tp[j]];
    const size_t sl = agg_slot(pl, c.shape, c.tp[j], j);
    const Rec r = make_rec(pl.ta[(sl * GX + gx) * MB + c.mb], pl.syncz[sl * Z + z], pl.upd[sl * GX + gx],
                           pl.price_f[gx], ts[z * Z + z], sh.n[j], tpv, 0u);
    const uint64_t need = pl.need[(sl * MB + c.mb) * DP + c.dp];
    const uint64_t m = need + pl.res[ga], m2 = need + pl.res[gb];
    if (m > pl.cap[ga] || m2 > pl.cap[gb]) mask |= 1u;
    peak = m > peak ? m : peak;
    peak = m2 > peak ? m2 : peak;
    w[j] = sh.n[j] * tpv;  // GPUs of one replica on this pool
    if (!((pl.qw[(size_t)w[j] * pl.ZG + p] >> c.dp) & 1u)) mask |= 2u;
    if (tpv > pl.node[ga] || tpv > pl.node[gb]) mask |= 8u;
    if (j == 0) {
      acc = acc_begin(r);
    } else {
      const int zp = c.a[j - 1] / GX;
      acc = acc_cross(acc, r, ts[zp * Z + z], ts[z * Z + zp],
                      pl.egs_f[zp * Z + z], sh.n[j - 1] == 1, j == 1);
    }
  }
  // segments that draw on one real pool together
  if (pl.mixed) {
    if (S >= 2 && !((joint_quota_bits(pl, S, c.a[0], c.a[1], c.a[2], w[0], w[1], w[2]) >> c.dp) & 1u))
      mask |= 2u;
  } else if (S == 3 && c.a[0] == c.a[2]) {
    if ((int64_t)(w[0] + w[2]) * D > (int64_t)pl.avail[c.a[0]]) mask |= 2u;
  }
  acc_finish(acc, lc, T, C);
}

// One lane per candidate; reads the segment aggregates straight from global memory.
__global__ __launch_bounds__(256) void k_eval_direct(DevPlan pl, EvalArgs a) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.count) return;
  const uint64_t idx = a.indices ? a.indices[i] : a.first + i;
  float T = kPosInf, C = kPosInf;
  uint64_t peak = 0;
  uint32_t mask = 0xFFFFFFFFu;
  Cand c;
  if (decode_index(pl, idx, c)) {
    mask = 0;
    const int nb = pl.nb[c.mb * pl.DP + c.dp];
    if (nb == 0) {
      mask = 4u;
    } else {
      const ShapeRec sh = pl.shapes[c.shape];
      LaneC lc;
      lc.nbm1 = pl.nbm1_f[c.mb * pl.DP + c.dp];
      lc.cd = pl.cd_f[c.dp];
      lc.dph = pl.dph_f[c.dp];
      lc.xb = pl.xb_f[c.mb];
      if (c.s == 1) eval_direct_s<1>(pl, c, sh, lc, T, C, peak, mask);
      else if (c.s == 2) eval_direct_s<2>(pl, c, sh, lc, T, C, peak, mask);
      else eval_direct_s<3>(pl, c, sh, lc, T, C, peak, mask);
      if (a.has_bound) {
        if (a.objective == 0) { if (C > a.bound) mask |= 32u; }
        else if (throughput_below(T, a.bound)) mask |= 32u;
      }
    }
  }
  if (a.time) a.time[i] = T;
  if (a.cost) a.cost[i] = C;
  if (a.mem) a.mem[i] = peak;
  if (a.mask) a.mask[i] = mask;
}

// Range form of sailor_eval_batch.  One workgroup per EvalUnit: the records of the unit's
// shape for every tp are staged in LDS.  A lane keeps its inner digits (mb, tp, dp, pool 1)
// while the unit's outer digits advance, and consecutive lanes hold consecutive
// candidate indices, so every store instruction writes 64 consecutive elements.
struct PoolInfo {   // per pool, staged in LDS (a pair of types: the tighter of the two)
  uint64_t res;     // reserved bytes (the larger)
  int64_t room;     // capacity - reserved (the smaller; negative when nothing fits)
  int32_t avail;    // GPUs available (plain types only)
  uint32_t meta;    // zone | (bit 8 + k: tp k exceeds the node size) (H1)
  uint64_t pad;     // (32 bytes: the index is a shift)
};
static_assert(sizeof(PoolInfo) == 32, "one pool per 32 bytes of LDS");

// 24-bit multiply (full rate, unlike the 32-bit one): every product below is a table offset
__device__ __forceinline__ uint32_t mul24(uint32_t a, uint32_t b) { return __umul24(a, b); }

// A segment record of the range evaluation, kept in LDS as two 16-byte halves in arrays of
// their own: the records a wave reads together then lie 16 bytes apart, not 32, and collide
// on half as many banks.
__device__ __forceinline__ Rec rec_of(const float4 *lo, const float4 *hi, uint32_t i) {
  const float4 a = lo[i], b = hi[i];
  Rec r;
  r.sumT = a.x; r.tF = a.y; r.tL = a.z; r.tI = a.w;
  r.syncb = b.x; r.upd = b.y; r.pricen = b.z;
  r.bits = 0u;  // validity comes from the masks here
  return r;
}

template <int S, bool PST, bool MIXED>
__device__ __forceinline__ void eval_rows_body(const DevPlan &pl, const EvalArgs &a,
                                               const EvalUnit &u, const ShapeRec &sh,
                                               const float4 *rec_lo, const float4 *rec_hi,
                                               const float4 *pair, const uint32_t *qm,
                                               const uint64_t *need, const PoolInfo *pinfo,
                                               const uint32_t *odec, const int32_t *vals,
                                               const uint64_t *isect) {
  const uint32_t ZG = pl.ZG, MB = pl.MB, TP = pl.TP, DP = pl.DP, Z = pl.Z;
  const uint32_t inner = pl.inner;
  const uint64_t last = a.first + a.count;
  const bool single0 = sh.n[0] == 1, single1 = sh.n[1] == 1;
  // the unit's outputs start here; lanes add a 32-bit offset (a unit that begins before the
  // range only stores where idx >= first, so the wrapped pointer is never used below it)
  const int64_t ubase = (int64_t)(u.idx_lo - a.first);
  float *const o_time = a.time ? a.time + ubase : nullptr;
  float *const o_cost = a.cost ? a.cost + ubase : nullptr;
  uint64_t *const o_mem = a.mem ? a.mem + ubase : nullptr;
  uint32_t *const o_mask = a.mask ? a.mask + ubase : nullptr;
  const bool whole = u.idx_lo >= a.first && u.idx_lo + (uint64_t)u.o_cnt * inner <= last;  // uniform
  const uint32_t tp_rec = mul24(ZG, MB) + 1u;  // records per (segment, tp) slice, one unused
  const uint32_t seg_rec = mul24(TP, tp_rec), seg_need = mul24(mul24(TP, MB), DP),
                 seg_qm = mul24(TP, ZG);
  for (uint32_t in = threadIdx.x; in < inner; in += blockDim.x) {
    const uint32_t a1 = fast_div(in, pl.mg_mbtpdp), rem = in - mul24(a1, MB * TP * DP);
    const uint32_t dp = fast_div(rem, pl.mg_mbtp), rem2 = rem - mul24(dp, MB * TP);
    const uint32_t tp = fast_div(rem2, pl.mg_mb), mb = rem2 - mul24(tp, MB);
    const bool divisible = pl.nb[mb * DP + dp] != 0;
    LaneC lc;
    lc.nbm1 = pl.nbm1_f[mb * DP + dp];
    lc.cd = pl.cd_f[dp];
    lc.dph = pl.dph_f[dp];
    lc.xb = pl.xb_f[mb];
    // this lane's slices of the staged tables; segment j with tp index k on pool p:
    const float4 *recl_lo = rec_lo + mb, *recl_hi = rec_hi + mb;  // [(j * TP + k) * tp_rec + p * MB]
    const uint64_t *needl = need + mul24(mb, DP) + dp;  // [(j * TP + k) * MB * DP]
    const float4 *pairm = pair + mul24(mb, Z * Z);   // transfers of this microbatch size
    // with one tp per plan the later segments use this lane's tp: their slices are fixed
    const uint32_t tpo_rec = mul24(tp, tp_rec), tpo_need = mul24(mul24(tp, MB), DP),
                   tpo_qm = mul24(tp, ZG);
    // segment 1 does not change while the outer digits advance
    const uint32_t p0 = a1;
    const Rec r0 = rec_of(recl_lo, recl_hi, tpo_rec + mul24(p0, MB));
    const Acc A0 = acc_begin(r0);
    const PoolInfo i0 = pinfo[p0];
    const uint64_t need0 = needl[tpo_need], mem0 = need0 + i0.res;
    uint32_t mask0 = 0;
    if ((int64_t)need0 > i0.room) mask0 |= 1u;
    if (i0.meta & (1u << (8 + tp))) mask0 |= 8u;
    const bool q0 = (qm[tpo_qm + p0] >> dp) & 1u;
    const uint32_t z0 = i0.meta & 0xFFu;
    const int64_t D = vals[dp];  // value lists staged in LDS: [DP] dp, then [TP] tp
    const int64_t gpus0 = (int64_t)sh.n[0] * vals[DP + tp];
    // with one tp per plan the bytes segments 2 and 3 need do not change with the outer digits
    const uint64_t need1_lane = (!PST && S >= 2) ? needl[seg_need + tpo_need] : 0;
    const uint64_t need2_lane = (!PST && S == 3) ? needl[2 * seg_need + tpo_need] : 0;
    uint32_t off = in;           // o * inner + in
    for (uint32_t o = 0; o < u.o_cnt; ++o, off += inner) {
      if (!whole) {
        const uint64_t idx = u.idx_lo + off;
        if (idx < a.first || idx >= last) continue;
      }
      const uint32_t od = odec[o];  // outer digits (uniform)
      float T = kPosInf, C = kPosInf;
      uint64_t peak = 0;
      uint32_t mask = 4u;
      if (divisible) {
        mask = mask0;
        peak = mem0;
        Acc acc = A0;
        bool quota_ok = q0;
        if (S >= 2) {
          const uint32_t r2 = od & 127u;
          const uint32_t t1 = PST ? ((od >> 7) & 7u) : tp;
          uint32_t p1 = p0 + 1 + r2;
          if (p1 >= ZG) p1 -= ZG;
          // uniform offsets when the segment has its own tp digit, this lane's otherwise
          const uint32_t o_rec = seg_rec + (PST ? mul24(t1, tp_rec) : tpo_rec);
          const uint32_t o_need = seg_need + (PST ? mul24(mul24(t1, MB), DP) : tpo_need);
          const uint32_t o_qm = seg_qm + (PST ? mul24(t1, ZG) : tpo_qm);
          const Rec r1 = rec_of(recl_lo, recl_hi, o_rec + mul24(p1, MB));
          const PoolInfo i1 = pinfo[p1];
          const uint32_t z1 = i1.meta & 0xFFu;
          const uint64_t need1 = PST ? needl[o_need] : need1_lane, mem1 = need1 + i1.res;
          if ((int64_t)need1 > i1.room) mask |= 1u;
          if (i1.meta & (1u << (8 + t1))) mask |= 8u;
          peak = mem1 > peak ? mem1 : peak;
          const bool q1 = (qm[o_qm + p1] >> dp) & 1u;
          quota_ok = quota_ok && q1;
          if (S == 2 && MIXED && quota_ok && pool_bit(isect, (int)p0, (int)p1))
            quota_ok = (joint_quota_bits(pl, 2, (int)p0, (int)p1, 0, (int)gpus0,
                                         sh.n[1] * vals[DP + t1], 0) >> dp) & 1u;
          const float4 pr = pairm[mul24(z0, Z) + z1];
          acc = acc_cross(acc, r1, pr.x, pr.y, pr.z, single0, true);
          if (S == 3) {
            const uint32_t r3 = (od >> 10) & 127u;
            const uint32_t t2 = PST ? (od >> 17) : tp;
            uint32_t p2 = p1 + 1 + r3;
            if (p2 >= ZG) p2 -= ZG;
            const uint32_t o_rec2 = 2 * seg_rec + (PST ? mul24(t2, tp_rec) : tpo_rec);
            const uint32_t o_need2 = 2 * seg_need + (PST ? mul24(mul24(t2, MB), DP) : tpo_need);
            const uint32_t o_qm2 = 2 * seg_qm + (PST ? mul24(t2, ZG) : tpo_qm);
            const Rec r2r = rec_of(recl_lo, recl_hi, o_rec2 + mul24(p2, MB));
            const PoolInfo i2 = pinfo[p2];
            const uint64_t need2 = PST ? needl[o_need2] : need2_lane, mem2 = need2 + i2.res;
            if ((int64_t)need2 > i2.room) mask |= 1u;
            if (i2.meta & (1u << (8 + t2))) mask |= 8u;
            peak = mem2 > peak ? mem2 : peak;
            if (MIXED) {  // pools that draw on one real pool together get the joint check
              quota_ok = quota_ok && ((qm[o_qm2 + p2] >> dp) & 1u);
              if (quota_ok && (pool_bit(isect, (int)p0, (int)p1) || pool_bit(isect, (int)p1, (int)p2) ||
                               pool_bit(isect, (int)p0, (int)p2)))
                quota_ok = (joint_quota_bits(pl, 3, (int)p0, (int)p1, (int)p2, (int)gpus0,
                                             sh.n[1] * vals[DP + t1], sh.n[2] * vals[DP + t2]) >> dp) & 1u;
            } else if (p2 == p0) {  // segments 1 and 3 share one pool's quota
              const int64_t gpus = gpus0 + (int64_t)sh.n[2] * vals[DP + t2];
              quota_ok = q1 && gpus * D <= (int64_t)i0.avail;
            } else {
              quota_ok = quota_ok && ((qm[o_qm2 + p2] >> dp) & 1u);
            }
            const float4 pr2 = pairm[mul24(z1, Z) + (i2.meta & 0xFFu)];
            acc = acc_cross(acc, r2r, pr2.x, pr2.y, pr2.z, single1, false);
          }
        }
        if (!quota_ok) mask |= 2u;
        acc_finish(acc, lc, T, C);
        if (a.has_bound) {
          if (a.objective == 0) { if (C > a.bound) mask |= 32u; }
          else if (throughput_below(T, a.bound)) mask |= 32u;
        }
      }
      if (o_time) o_time[off] = T;
      if (o_cost) o_cost[off] = C;
      if (o_mem) o_mem[off] = peak;
      if (o_mask) o_mask[off] = mask;
    }
  }
}

template <bool MIXED>
__global__ __launch_bounds__(512) void k_eval_rows(DevPlan pl, EvalArgs a, const EvalUnit *units,
                                                   uint32_t unit0) {
  extern __shared__ uint4 lds_raw[];
  const EvalUnit u = units[unit0 + blockIdx.x];
  const ShapeRec sh = pl.shapes[u.shape];
  const int ZG = pl.ZG, G = pl.GX, MB = pl.MB, TP = pl.TP, DP = pl.DP, Z = pl.Z, S = sh.s;
  // [3][TP][ZG * MB + 1]: a (segment, tp) slice is one record longer than its contents, so
  // that the slices of the tp values a wave reads together do not start on the same LDS banks
  float4 *rec_lo = reinterpret_cast<float4 *>(lds_raw);  // the records' two halves (see rec_of)
  float4 *rec_hi = rec_lo + 3 * TP * (ZG * MB + 1);
  float4 *pair = rec_hi + 3 * TP * (ZG * MB + 1);         // [MB][Z][Z]
  PoolInfo *pinfo = reinterpret_cast<PoolInfo *>(pair + MB * Z * Z);     // [ZG]
  uint64_t *need = reinterpret_cast<uint64_t *>(pinfo + ZG);             // [3][TP][MB][DP]
  uint64_t *isect = need + 3 * TP * MB * DP;                             // [ZG][2]
  uint32_t *qm = reinterpret_cast<uint32_t *>(isect + 2 * ZG);           // [3][TP][ZG]
  uint32_t *odec = qm + 3 * TP * ZG;  // [o_cnt] the outer digits of the unit, unpacked:
  int32_t *vals = reinterpret_cast<int32_t *>(odec + kEvalUnitMaxOuter);  // [DP] dp, [TP] tp
  const int t = threadIdx.x;          // r2 | tp2 << 7 | r3 << 10 | tp3 << 17
  if (t < DP) vals[t] = pl.dpv[t];
  else if (t < DP + TP) vals[t] = pl.tpv[t - DP];
  __syncthreads();
  if (S >= 2)
    for (uint32_t o = t; o < u.o_cnt; o += blockDim.x) {
      uint32_t oa = u.o_lo + o;
      uint32_t d = oa % (uint32_t)(ZG - 1);
      oa /= (uint32_t)(ZG - 1);
      if (pl.pst) { d |= (oa % (uint32_t)TP) << 7; oa /= (uint32_t)TP; }
      if (S == 3) {
        d |= (oa % (uint32_t)(ZG - 1)) << 10;
        oa /= (uint32_t)(ZG - 1);
        if (pl.pst) d |= oa << 17;
      }
      odec[o] = d;
    }
  else
    for (uint32_t o = t; o < u.o_cnt; o += blockDim.x) odec[o] = 0;
  for (int i = t; i < S * TP * ZG; i += blockDim.x) {
    const int p = i % ZG, k = (i / ZG) % TP, seg = i / (ZG * TP);
    const int n = seg == 0 ? sh.n[0] : (seg == 1 ? sh.n[1] : sh.n[2]);
    qm[i] = pl.qw[(size_t)(n * vals[DP + k]) * ZG + p];
  }
  for (int p = t; p < ZG; p += blockDim.x) {
    const int x = pl.xt[p % G], ga = x & 255, gb = x >> 8;
    PoolInfo pi;
    pi.res = max(pl.res[ga], pl.res[gb]);
    pi.room = min((int64_t)pl.cap[ga] - (int64_t)pl.res[ga], (int64_t)pl.cap[gb] - (int64_t)pl.res[gb]);
    pi.avail = pl.mixed ? 0 : pl.avail[p];
    pi.meta = (uint32_t)(p / G) | (pl.h1m[p] << 8);
    pi.pad = 0;
    pinfo[p] = pi;
    isect[2 * p] = pl.isect[2 * p];
    isect[2 * p + 1] = pl.isect[2 * p + 1];
  }
  for (int i = t; i < MB * Z * Z; i += blockDim.x) {  // per mb: transfer a -> b, b -> a, egress
    const int m = i / (Z * Z), ab = i - m * Z * Z, za = ab / Z, zb = ab % Z;
    pair[i] = make_float4(pl.tsec_f[i], pl.tsec_f[(m * Z + zb) * Z + za], pl.egs_f[ab], 0.f);
  }
  for (int i = t; i < S * TP * MB * DP; i += blockDim.x) {
    const int md = i % (MB * DP), k = (i / (MB * DP)) % TP, seg = i / (MB * DP * TP);
    need[i] = pl.need[agg_slot(pl, u.shape, k, seg) * MB * DP + md];
  }
  for (int i = t; i < S * TP * ZG * MB; i += blockDim.x) {
    const int mb = i % MB, p = (i / MB) % ZG, k = (i / (MB * ZG)) % TP, seg = i / (MB * ZG * TP);
    const int g = p % G, z = p / G;
    const size_t sl = agg_slot(pl, u.shape, k, seg);
    const Rec r =
        make_rec(pl.ta[(sl * G + g) * MB + mb], pl.syncz[sl * Z + z], pl.upd[sl * G + g],
                 pl.price_f[g], pl.tsec_f[(mb * Z + z) * Z + z],
                 seg == 0 ? sh.n[0] : (seg == 1 ? sh.n[1] : sh.n[2]), vals[DP + k], 0u);
    const int at = i + seg * TP + k;  // (one unused record behind every slice)
    rec_lo[at] = make_float4(r.sumT, r.tF, r.tL, r.tI);
    rec_hi[at] = make_float4(r.syncb, r.upd, r.pricen, 0.f);
  }
  __syncthreads();
#define SAILOR_ROWS(S_, PST_) \
  eval_rows_body<S_, PST_, MIXED>(pl, a, u, sh, rec_lo, rec_hi, pair, qm, need, pinfo, odec, vals, isect)
  if (S == 1) SAILOR_ROWS(1, false);
  else if (!pl.pst) { if (S == 2) SAILOR_ROWS(2, false); else SAILOR_ROWS(3, false); }
  else { if (S == 2) SAILOR_ROWS(2, true); else SAILOR_ROWS(3, true); }
#undef SAILOR_ROWS
}

}  // namespace sailor
