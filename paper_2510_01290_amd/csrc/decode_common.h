// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) is cut into work items class by class: the page list of
// thought type c is cut into ceil(np_c / ppi_c) items of about ppi_c pages, ppi_c chosen by
// the bit width so that items of all classes move about the same bytes.  An item therefore
// holds pages of ONE bit width, which is a compile-time constant of the kernel body it runs.
// A sequence's items are numbered class after class (class 0 first); the split dimension of
// the grid is sized on the host for the worst class mix of max_ctx_pages pages; item counts
// are derived on the device from the page counts, identically in the attention and merge
// kernels.  Each item writes, per query head,
// a partial (m, l, acc[D]): running maximum of the scaled scores in the log2 domain, sum of
// 2^(score - m), and the unnormalised weighted value sum.
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
  int ppi[3];           // pages per item of each class
  int max_split;        // grid extent of the split dimension (>= items of any sequence)
  float scale_log2e;    // softmax_scale * log2(e)
};

__host__ __device__ inline int pages_per_item_for_bits(int bits) { return bits == 8 ? 64 : (bits == 4 ? 128 : 192); }

__device__ inline int n_items_of(int np, int ppi) { return (np + ppi - 1) / ppi; }

// which class and item a split index names; false if the sequence has no such item
__device__ inline bool locate_item(const DecodeArgs& a, const int np[3], int split, int* cls, int* item, int* n_items) {
  int s = split;
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const int ns = n_items_of(np[c], a.ppi[c]);
    if (s < ns) {
      *cls = c;
      *item = s;
      *n_items = ns;
      return split < a.max_split;
    }
    s -= ns;
  }
  return false;
}

__device__ inline int64_t partial_index(const DecodeArgs& a, int Hq, int D, int b, int hq, int split) {
  return (((int64_t)b * Hq + hq) * a.max_split + split) * (D + 2);
}

}  // namespace thinkv
