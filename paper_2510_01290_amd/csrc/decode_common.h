// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) is cut into work items.  Item sizes are counted in
// quarter units: the sequence's pages make U = ceil(4 * pages / ppi) units, dealt four at a time
// to ceil(U / 4) items (about ppi pages each; the last item may be shorter).  An item takes the
// same fraction [u0 / U, u1 / U) of each of the three per-type page lists, so items of one
// sequence cost the same per unit whatever the precision mix.  (On full-attention layers the
// fast kernel only uses the item count: there the workgroups of a (query, kv-head) draw their
// pages from shared queues.)  ppi is chosen on the host; item counts are derived on the device
// from the page counts, identically in the attention and merge kernels.  Each item writes, per
// query head, a partial (m, l, acc[D]): running maximum of the scaled scores in the log2
// domain, sum of 2^(score - m), and the unnormalised weighted value sum.
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
  int ppi;              // pages per item
  int max_split;        // grid extent: items, hence partial rows, per (query, head) (>= the count of any sequence)
  float scale_log2e;    // softmax_scale * log2(e)
  // sparsity statistic (null / 0 on plain attention calls)
  float* stat;          // [B][n_kv_heads][stat_stride] pooled scores, 16 per page in page-list order (types 0, 1, 2)
  int64_t stat_stride;  // floats per (query, kv-head): 16 * max_ctx_pages
  float* sparsity;      // [B]
  int direct;           // 1: every query has a single item (max_split == 1) and the attention kernel writes out / lse itself
};

struct ItemPlan {
  int n_items, units;
};

__host__ __device__ inline ItemPlan plan_items(int ppi, int max_items, int np_total) {
  ItemPlan p;
  p.units = (int)(((int64_t)np_total * 4 + ppi - 1) / ppi);
  p.n_items = (p.units + 3) / 4;
  if (p.n_items > max_items) p.n_items = max_items;   // never on a launch sized by the host's bound
  return p;
}

// item i of the plan covers units [u0, u1) of p.units
__device__ inline void item_units(const ItemPlan& p, int i, int* u0, int* u1) {
  *u0 = 4 * i;
  *u1 = 4 * i + 4 < p.units ? 4 * i + 4 : p.units;
}

// Workgroup id -> (query, kv-head, item j), item-major: ids [j * heads, (j + 1) * heads) are item
// j of every head, and head h's item j sits at offset (h + j) mod heads of that run; the caller
// checks j against the sequence's plan.  Two things follow.  The hardware starts workgroups in id order and a SIMD favours
// its oldest wave, so the workgroups of the first third of a chip-filling launch run visibly faster
// than those of the last third: item-major order gives every head workgroups of every age.  And
// ids go round the XCDs (id mod 8), so the shift by j puts the items of a head on different XCDs.
__device__ inline void locate_workgroup(const DecodeArgs& a, int n_kv_heads, int id, int* b, int* hkv, int* j) {
  const int heads = n_kv_heads * a.B;
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
