// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) is cut into n = ceil(pages / ppi) work items.  Item s
// takes, from each of the three per-type page lists, the pages [s*np_c/n, (s+1)*np_c/n), so
// every item gets the same share of every precision and items of one sequence cost the same.
// ppi (pages per item) is chosen on the host so that a launch fills the machine a whole
// number of times; n is derived on the device from the page counts, identically in the
// attention and merge kernels.  Each item writes, per query head, a partial (m, l, acc[D]):
// running maximum of the scaled scores in the log2 domain, sum of 2^(score - m), and the
// unnormalised weighted value sum.
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
  int max_split;        // grid extent of the split dimension (>= items of any sequence)
  float scale_log2e;    // softmax_scale * log2(e)
};

__device__ inline int n_items_of(const DecodeArgs& a, int np_total) {
  const int s = (np_total + a.ppi - 1) / a.ppi;
  return s < a.max_split ? s : a.max_split;
}

__device__ inline int64_t partial_index(const DecodeArgs& a, int Hq, int D, int b, int hq, int split) {
  return (((int64_t)b * Hq + hq) * a.max_split + split) * (D + 2);
}

}  // namespace thinkv
