// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) is cut into n_split work items.  Item s takes, from each
// of the three per-type page lists, the pages [s*np_c/n_split, (s+1)*np_c/n_split), so every
// item gets the same share of every precision and therefore about the same bytes.  n_split is
// derived on the device from the page counts, identically in the attention and merge kernels.
// Each item writes, per query head, a partial (m, l, acc[D]): running maximum of the scaled
// scores in the log2 domain, sum of 2^(score - m), and the unnormalised weighted value sum.
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
  int max_split;        // grid extent in the split dimension
  int pages_per_item;   // target pages per work item
  float scale_log2e;    // softmax_scale * log2(e)
};

__device__ inline int n_split_of(int np_total, int pages_per_item, int max_split) {
  int s = (np_total + pages_per_item - 1) / pages_per_item;
  s = s < 1 ? 1 : s;
  return s > max_split ? max_split : s;
}

__device__ inline int64_t partial_index(const DecodeArgs& a, int Hq, int D, int b, int hq, int split) {
  return (((int64_t)b * Hq + hq) * a.max_split + split) * (D + 2);
}

}  // namespace thinkv
