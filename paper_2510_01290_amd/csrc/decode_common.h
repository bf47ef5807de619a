// Split-K bookkeeping shared by the decode-attention kernels and the merge kernel.
//
// The context of one (query, kv-head) -- a "head" below -- is worked on by several items; each
// item leaves, per query head of the group, one partial row (acc[D], m, l, two words of padding):
// the unnormalised weighted value sum, the running maximum of the scaled scores in the log2
// domain, and the sum of 2^(score - m).  The merge kernel folds the rows of a head.
//
// How many items a head gets is decided on the device from its page count, identically by every
// kernel of a call: an item per `ppi` pages, at most `per_head` (both chosen by the host); the items
// of a head that is short do not exist (their waves leave at once).  On full-attention layers the
// fast kernel's items do not own pages: the items of a head draw page pairs from shared queues, so
// an item is a worker and its count a share of the machine.  Elsewhere item j of n takes the same
// fraction [j/n, (j+1)/n) of each of the three per-type lists.
#pragma once
#include "common.h"

// waves per SIMD the fast kernel is built for (its register budget: 256 registers a lane at head_dim 128, where a
// pair of 8-bit pages alone takes 48 and two pairs are held; half the tiles and half the page bytes at head_dim 64
// leave room for a third wave); the host sizes launches with the same numbers
#ifndef TKV_WAVES_128
#define TKV_WAVES_128 2
#endif
#ifndef TKV_WAVES_64
#define TKV_WAVES_64 3
#endif
__host__ __device__ constexpr int decode_waves_per_simd(int head_dim) { return head_dim == 64 ? TKV_WAVES_64 : TKV_WAVES_128; }

namespace thinkv {

struct DecodeArgs {
  const void* q;
  void* out;
  float* lse;
  const int32_t* seq_ids;
  const int32_t* q_pos;
  float* partial;       // [n_rows][G][D + 4]
  int32_t* alloc;       // [B * n_kv_heads][2]: first row and number of rows of each head, written by its item 0
  int layer, B, window, q_dtype, out_dtype;
  int n_rows;           // items (grid extent of the fast kernel, in waves), = per_head * B * n_kv_heads
  int per_head;         // the most items a head can have
  int ppi;              // pages per item
  float scale_log2e;    // softmax_scale * log2(e)
  // sparsity statistic (null / 0 on plain attention calls)
  float* stat;          // [B][n_kv_heads][stat_stride] pooled scores, 16 per page in page-list order (types 0, 1, 2)
  int64_t stat_stride;  // floats per (query, kv-head): 16 * max_ctx_pages
  float* sparsity;      // [B]
  int direct;           // 1: every head has a single item and the attention kernel writes out / lse itself
};

constexpr int kMaxRowsPerHead = 1024;

struct ItemLoc {
  int b, hkv;   // the head
  int j, n;     // item j of n
  int row0;     // the head's first partial row
};

__device__ inline int seq_pages(const thinkv_view& v, int layer, int seq, int* np) {
  const thinkv_config& c = v.cfg;
  int tot = 0;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    np[k] = (seq >= 0 && seq < c.max_seqs) ? v.n_pages[npages_index(c, seq, layer, k)] : 0;
    tot += np[k];
  }
  return tot;
}

// Item id -> head, item number, item count, first row.  Item-major: ids [j * heads, (j + 1) * heads) are item j of every
// head (the hardware starts workgroups in id order and a SIMD favours its oldest wave: every head gets workers of every
// age), shifted by j so that the items of a head land on different XCDs (ids go round the XCDs).
__device__ inline ItemLoc locate_item(const thinkv_view& v, const DecodeArgs& a, int id) {
  const thinkv_config& c = v.cfg;
  const int H = c.n_kv_heads, heads = H * a.B;
  ItemLoc it;
  it.j = id / heads;
  int rest = id % heads - it.j % heads;
  if (rest < 0) rest += heads;
  it.hkv = rest % H;
  it.b = rest / H;
  int np[3];
  const int tot = seq_pages(v, a.layer, a.seq_ids[it.b], np);
  int n = (int)(((int64_t)tot + a.ppi - 1) / a.ppi);
  n = n < 1 ? 1 : (n > a.per_head ? a.per_head : n);
  it.n = n;
  it.row0 = rest * a.per_head;
  return it;
}

constexpr int kRowPad = 4;   // a partial row: acc[D], m, l, two unused words (rows stay 16-byte aligned)

__device__ inline float* partial_row(const DecodeArgs& a, int G, int D, int row, int g) {
  return a.partial + ((int64_t)row * G + g) * (D + kRowPad);
}

}  // namespace thinkv
