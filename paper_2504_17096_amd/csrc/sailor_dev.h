// Device-side data layout of a plan, shared by the host code and the kernels.
//
// A candidate plan (Sailor, Sec. 4.2) is a point of a flat index space; see
// include/sailor.h for the numbering.  Candidates that share the pipeline depth, the
// layer split and the cut points form a "shape": all per-stage work of the simulator
// (Sec. 4.3) that does not depend on which pool a segment runs on is folded, once per
// plan, into per-shape segment aggregates.  The scan kernel then evaluates a candidate
// from a few aggregates instead of a loop over its stages.
#pragma once

#include <stdint.h>

namespace sailor {

constexpr int kMaxMB = 8, kMaxTP = 8, kMaxDP = 24, kMaxPools = 128, kMaxZones = 16,
              kMaxTypes = 16, kMaxStages = 256;
constexpr int kEvalUnitMaxOuter = 1024;  // most outer-digit values one range-evaluation unit spans
constexpr int kMaxUnitThreads = 512;  // scan workgroups use 2..8 waves, chosen per plan
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kPosInf = __builtin_huge_valf();

// relative error budget of an fp32 key against its exact value, used to widen the
// bands inside which candidates are re-evaluated in fp64
constexpr float kEvalEps = 2.0e-6f;
constexpr double kTieTol = 1.0e-5;

struct ShapeRec {
  uint64_t base;       // first candidate index of the shape
  uint32_t row_stage;  // first entry of the shape's partition row in the stage tables
  uint32_t pp_idx, q;
  uint16_t P, s;
  uint16_t n[3];       // stages per segment (0 = absent)
  uint16_t lo[3];      // first stage of each segment
  uint16_t k1, k2;     // cut points (P when unused)
};

struct BlockRec {       // all candidates with one (pp index, segment count)
  uint64_t off, size;
  uint64_t shape_size;  // candidates per shape
  uint32_t first_shape, n_shapes;
  uint32_t pp_idx, s, P, pad;
};

struct UnitRec {        // work of one workgroup of the scan: one shape, one tp per segment
  uint64_t base;        // (all equal unless segments carry their own tp digit), a range
  uint32_t shape;       // [o_lo, o_lo + o_cnt) of segment 2's pool.  base = first index of
  uint8_t tp[3], s;     // the shape + the offset of the unit's tp digits of segments 2, 3;
  uint16_t o_lo, o_cnt; // n = stages per segment (copied from the shape, so that a
  uint16_t n[3];        // workgroup needs one record to start).  A unit found to run long is
  uint8_t part, n_parts;  // cut into n_parts records: record `part` takes every n_parts-th
  uint32_t pad2;          // share of the lane space (the (mb, dp, pool 1) triples)
};
static_assert(sizeof(UnitRec) == 32, "one unit record per 32 bytes");

struct EvalUnit {       // work of one workgroup of the range evaluation: one shape, all tp,
  uint64_t idx_lo;      // a contiguous index range = a range of the outer pool digits
  uint32_t shape;
  uint32_t o_lo, o_cnt;
  uint32_t pad;
};

struct SurvRec {        // candidate kept for the fp64 re-evaluation
  uint64_t idx;
  float key;            // fp32 key; +inf when only loosely inside the constraint
  float key_loose;      // fp32 key
  uint32_t shape;       // the candidate's shape, known to the pass that kept it
  uint32_t pad;
};

struct RefRec {         // fp64 re-evaluation of one candidate
  uint64_t idx, mem;
  double T, C;
  uint32_t mask, pad;
};

struct ResultHeader {   // written by the final kernel into host-mapped memory
  uint32_t n_found, surv_count, ref_count, feasible_count;
  uint32_t gmin_bits;  // smallest strict fp32 key of the scan
  uint32_t seq;        // the call's sequence number, written last: the results are complete
  uint32_t pad[2];
};

struct DevPlan {
  // G real GPU types; GX types a segment can choose (G, or G + G (G - 1) / 2 with the pairs
  // of mixed replicas); ZG = Z * GX pools of the candidate space; ZGr = Z * G real pools
  int G, GX, Z, ZG, ZGr, MB, TP, DP;
  int mixed;               // 1: pairs of types exist
  int n_blocks, n_shapes, n_units, n_row_stages, P_max;
  int pst;                 // 1: segments 2 and 3 carry their own tp digit
  int otp;                 // radix of those digits: TP, or 1 when all segments share one tp
  int W_max;               // most GPUs one replica can take from a pool: P_max * largest tp
  uint32_t inner;          // MB*TP*DP*ZG candidates per (shape, outer digits)
  uint64_t stride3;        // index stride of segment 3's relative pool: inner*(ZG-1)*otp
  uint32_t bpp, gb;
  // ceil(2^32 / d) for d = MB, GX, MB*TP, MB*TP*DP, MB*ZG, MB*(ZG-1) (0 encodes d = 1)
  uint32_t mg_mb, mg_g, mg_mbtp, mg_mbtpdp, mg_mbzg, mg_mbzg1;
  int64_t B;
  uint64_t N;
  int mbv[kMaxMB], tpv[kMaxTP], dpv[kMaxDP];
  const int32_t *vals;         // the same lists in device memory, for lane-dependent indices:
                               // [DP] dp, then [TP] tp
  // inputs
  const int32_t *avail;        // [ZG]
  const uint64_t *cap, *res;   // [G]
  const int32_t *node;         // [G]
  const double *price;         // [G]
  const double *bw, *egress;   // [Z][Z]
  const uint64_t *act;         // [MB][TP]
  const uint64_t *p2p;         // [MB]
  // derived small tables
  uint32_t *qw;                // [W_max + 1][ZG] bit d: dpv[d] replicas of w GPUs fit the pool
                               // (a pair: half of them on each type, dpv[d] even)
  uint32_t *qh;                // [2 W_max + 1][ZGr] bit d: dpv[d] * x half-GPUs fit the real pool
  uint32_t *row_gen;           // [1] availability generation at which an entry of qh last changed
  uint32_t *h1m;               // [ZG] bit k: tpv[k] exceeds the node size of the pool's type(s) (H1)
  const uint16_t *xt;          // [GX] the two real types of an extended type: a | b << 8
  uint64_t *isect;             // [ZG][2] bit q: pools p and q draw on a common real pool
  int n_bw_coef;               // 0: constant link bandwidth
  const double *bw_poly;       // [Z][Z][n_bw_coef] bandwidth over log2(message bytes)
  double *bwp;                 // [MB][Z][Z] bandwidth seen by one activation transfer
  float *tsec_f;               // [MB][Z][Z] seconds of one activation transfer a -> b
  float *egs_f;                // [Z][Z] egress both ways
  float *price_f;              // [GX] (a pair: the mean)
  float *xb_f;                 // [MB] (B/mb) * p2p bytes
  float *cd_f;                 // [DP] 2 (D-1) / D
  float *nbm1_f;               // [MB][DP] microbatches per pipeline - 1
  float *dph_f;                // [DP] D / 3600
  int32_t *nb;                 // [MB][DP] microbatches per pipeline, 0 if B % (D mb) != 0
  uint32_t *divis;             // [MB] bit d set when nb[mb][d] > 0
  // per-stage tables, one entry per stage of every partition row
  const int32_t *st_n;         // layers
  const int32_t *st_first;     // first layer
  uint64_t *st_params;         // parameters incl. embedding / head
  double *st_c;                // [rs][G][MB][TP] sum of fwd + bwd layer times
  double *st_f, *st_b;         // [rs][G][MB][TP] the two sums apart (event-by-event schedule)
  double *st_u;                // [rs][G][TP] sum of update times
  // candidate space
  const ShapeRec *shapes;
  const BlockRec *blocks;
  const UnitRec *units;
  // per-shape segment aggregates, [shape][TP][3]...  (a pair of types: every stage at the
  // pace of its slower type, memory on both)
  float4 *ta;                  // [..][GX][MB] {sum, first, last, max interior} of stage compute
  uint32_t *memok;             // [..][GX][MB] bit d: no stage of the segment runs out of memory
  uint64_t *need;              // [..][MB][DP] max over stages of model + activation bytes
  float *syncz;                // [..][Z] slowest stage: gradient bytes / intra-zone bandwidth
  float *upd;                  // [..][GX] slowest stage update
};

}  // namespace sailor
