// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) is cut into work items.  Item sizes are counted in
// quarter units: the sequence's pages make U = ceil(4 * pages / ppi) units; the last n_small of
// them (a host choice, possibly none) become SMALL items of one unit, the others are dealt to
// BIG items of four units (about ppi pages; the last big item may be shorter).  The grid lists
// every big item of the launch before any small one, so the small items start last and can
// level the end of a launch that runs several rounds of workgroups.  An item takes the
// same fraction [u0 / U, u1 / U) of each of the three per-type page lists, so items of one
// sequence cost the same per unit whatever the precision mix.  ppi is chosen on the host so
// that the big items fill the machine a whole number of times; item counts are derived on the
// device from the page counts, identically in the attention and merge kernels.  Each item
// writes, per query head, a partial (m, l, acc[D]): running maximum of the scaled scores in the
// log2 domain, sum of 2^(score - m), and the unnormalised weighted value sum.
#pragma once
#include "common.h"

namespace thinkv {

struct DecodeArgs {
  const void* q;
  void* out;
  float* lse;
  const int32_t* seq_ids;
  const int32_t* q_pos;
  float* partial;       // [B][Hq][max_split][D + 2]
  int layer, B, window, q_dtype, out_dtype;
  int ppi;              // pages per big item
  int n_small;          // small items wanted per (query, kv-head)
  int max_big, max_small;   // grid extents (>= the counts of any sequence)
  int max_split;        // max_big + max_small: partial rows per (query, head)
  float scale_log2e;    // softmax_scale * log2(e)
  // sparsity statistic (null / 0 on plain attention calls)
  float* stat;          // [B][n_kv_heads][stat_stride] pooled scores, 16 per page in page-list order (types 0, 1, 2)
  int64_t stat_stride;  // floats per (query, kv-head): 16 * max_ctx_pages
  float* sparsity;      // [B]
};

struct ItemPlan {
  int n_big, n_small, units;
};

__host__ __device__ inline ItemPlan plan_items(int ppi, int n_small_wanted, int max_big, int max_small, int np_total) {
  ItemPlan p;
  p.units = (int)(((int64_t)np_total * 4 + ppi - 1) / ppi);
  p.n_small = p.units < n_small_wanted ? p.units : n_small_wanted;
  p.n_big = (p.units - p.n_small + 3) / 4;
  if (p.n_big > max_big) p.n_big = max_big;           // never on a launch sized by the host's bound
  if (p.n_small > max_small) p.n_small = max_small;
  return p;
}

// item i of the plan covers units [u0, u1) of p.units; items 0 .. n_big-1 are the big ones
__device__ inline void item_units(const ItemPlan& p, int i, int* u0, int* u1) {
  const int big_units = p.units - p.n_small;
  if (i < p.n_big) {
    *u0 = 4 * i;
    *u1 = 4 * i + 4 < big_units ? 4 * i + 4 : big_units;
  } else {
    *u0 = big_units + (i - p.n_big);
    *u1 = *u0 + 1;
  }
}

// Which (query, kv-head, item) workgroup `id` of the 1-D grid works on: all big items of the
// launch come first, then all small ones.  `j` is the item's index among the big (or small)
// items of its (query, kv-head); the caller checks it against the sequence's plan.
// Workgroup id -> (query, kv-head, item).  Big items come first, item-major: ids [j * heads,
// (j + 1) * heads) are item j of every head, and head h's item j sits at offset (h + j) mod heads
// of that run.  Two things follow.  The hardware starts workgroups in id order and a SIMD favours
// its oldest wave, so the workgroups of the first third of a chip-filling launch run visibly faster
// than those of the last third: item-major order gives every head workgroups of every age.  And
// ids go round the XCDs (id mod 8), so the shift by j puts the items of a head on different XCDs.
__device__ inline void locate_workgroup(const DecodeArgs& a, int n_kv_heads, int id, int* b, int* hkv, int* j, bool* small) {
  const int heads = n_kv_heads * a.B;
  const int n_big_total = a.max_big * heads;
  *small = id >= n_big_total;
  if (*small) id -= n_big_total;
  *j = id / heads;
  int rest = id % heads - *j % heads;
  if (rest < 0) rest += heads;
  *hkv = rest % n_kv_heads;
  *b = rest / n_kv_heads;
}

__device__ inline int64_t partial_index(const DecodeArgs& a, int Hq, int D, int b, int hq, int split) {
  return (((int64_t)b * Hq + hq) * a.max_split + split) * (D + 2);
}

}  // namespace thinkv
