// Quantise-and-append: slot selection with in-place reuse of evicted slots, group
// quantisation of the new K/V rows, packing into the page layout, table updates.
//
// The result must equal a one-token-at-a-time loop (first reclaimable slot in list order,
// else the tail of the last page, else a new page popped in token order).  Because eviction
// never interleaves with an append call, that loop has a closed form per (sequence, type):
// the k-th token of the type (k counted inside the call) takes
//     k < R            the k-th reclaimable slot in (page, slot) order        (R = #reclaimable)
//     k < R + tail     slot filled + (k - R) of the last page                  (tail = 16 - filled)
//     otherwise        slot (k-R-tail) % 16 of the (k-R-tail)/16-th new page
// and new pages are granted to sequences in ascending sequence id, which is token order.
// Three steps in two kernels, both on the caller's stream:
//   plan   (block per sequence)  token ranks per type, prefix popcounts of the reclaimable bits,
//                                pages needed
//   place  (block per token)     slot lookup, quantisation, packing, slot_pos, handle
//   commit (block per sequence)  masks, fill counts, page lists, counters
// The commit of a sequence changes tables that the place blocks of the sequence's tokens read
// (masks, fill counts, page list), and reads nothing that they write.  So it needs no kernel of
// its own, only to come after those reads: every place block, once its slot is settled, bumps
// an arrival counter of its sequence (view->append_counters), and the block that completes the
// count commits the sequence before it goes on to quantise its own token.  Reads-before-writes
// is all that has to hold, so no fence is involved (a release fence costs an L2 write-back here).
// A call of more than 64 tokens (a prefill, a refill: hundreds of blocks would bump one sequence's
// counter) keeps a commit kernel of its own and places its tokens sixteen to a block (see
// append_place_bulk_kernel).
// The grant of new pages (exclusive sum of the needs of the sequences before s, against what the
// pool held when the call began) is a sum over at most max_seqs small numbers: every block that
// wants it works it out for itself rather than waiting for a kernel of its own.  A decode step
// appends one token per sequence, so the call is a chain of short dependent launches and one
// launch less is a good part of its time.
#include "common.h"
#include "formats_dev.h"

namespace thinkv {

struct SeqPlan {
  int lo, hi;        // token range of the sequence inside the call
  int n[3];          // tokens per type
  int R[3];          // reclaimable slots per type before the call
  int tail[3];       // never-used slots in the last page
  int np_old[3];
  int need[3];       // new pages wanted (already limited by the page-list capacity)
  int grant[3];      // new pages granted
  int base[3];       // offset of the first granted page in pop order
  int pad;
};
static_assert(sizeof(SeqPlan) == 24 * 4, "SeqPlan layout");

constexpr int kBulkFrom = 64;   // calls of more tokens take the bulk kernels

struct AppendWs {
  SeqPlan* plan;     // [max_seqs]
  int* avail_old;    // [4]
  int* tok_rank;     // [n_tok]
  int* pre;          // [max_seqs][3][max_pages]
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t append_ws_bytes(const thinkv_config& c, int n_tok) {
  return align256((size_t)c.max_seqs * sizeof(SeqPlan)) + 256 + align256((size_t)(n_tok > 0 ? n_tok : 1) * 4) +
         align256((size_t)c.max_seqs * 3 * c.max_pages * 4);
}

static AppendWs carve(const thinkv_config& c, int n_tok, void* ws) {
  char* p = (char*)ws;
  AppendWs w;
  w.plan = (SeqPlan*)p;
  p += align256((size_t)c.max_seqs * sizeof(SeqPlan));
  w.avail_old = (int*)p;
  p += 256;
  w.tok_rank = (int*)p;
  p += align256((size_t)(n_tok > 0 ? n_tok : 1) * 4);
  w.pre = (int*)p;
  return w;
}

// Sum over a 256-thread block (every thread gets it).
__device__ inline int block_sum(int v, int* lds /*[5]*/) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
  __syncthreads();
  return lds[0] + lds[1] + lds[2] + lds[3];
}

// exclusive scan of one int per thread over a 256-thread block; returns the block total
__device__ inline int block_excl_scan(int v, int* excl, int* lds /*[5]*/) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int o = __shfl_up(inc, d, 64);
    if (lane >= d) inc += o;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    int t = lds[w];
    if (w < wave) off += t;
    tot += t;
  }
  *excl = off + inc - v;
  return tot;
}

__global__ __launch_bounds__(256) void append_plan_kernel(thinkv_view v, int layer, const int32_t* __restrict__ tok_seq,
                                                          const uint8_t* __restrict__ tok_class, int n_tok, AppendWs ws,
                                                          const int32_t* __restrict__ ev_seq, const int32_t* __restrict__ ev_handle,
                                                          int n_ev) {
  __shared__ int s_rng[2];
  __shared__ int s_scan[5];
  const thinkv_config& c = v.cfg;
  const int s = blockIdx.x, tid = threadIdx.x;
  // Evictions that come with the call (thinkv_evict_append): an eviction touches the tables of its
  // own sequence only, and so does the plan of a sequence, so the block of sequence s applies the
  // handles of sequence s and goes on; no block waits for another.
  if (n_ev > 0) {
    for (int i = tid; i < n_ev; i += 256) {
      const int es = ev_seq[i];
      if (es == s) evict_one(v, layer, s, ev_handle[i]);
      else if (s == 0 && (es < 0 || es >= c.max_seqs)) atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
    }
    __threadfence_block();
    __syncthreads();
  }
  if (n_tok <= kBulkFrom) {
    // small call (decode-style): every thread looks at a few tokens and the two that see the
    // sequence's first and last token publish the range
    if (tid == 0) s_rng[0] = s_rng[1] = 0;
    __syncthreads();
    for (int i = tid; i < n_tok; i += 256) {
      if (tok_seq[i] != s) continue;
      if (i == 0 || tok_seq[i - 1] != s) s_rng[0] = i;
      if (i == n_tok - 1 || tok_seq[i + 1] != s) s_rng[1] = i + 1;
    }
  } else if (tid == 0) {
    int lo = 0, hi = n_tok;  // lower_bound(s)
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (tok_seq[mid] < s) lo = mid + 1; else hi = mid;
    }
    int lo2 = lo, hi2 = n_tok;  // upper_bound(s)
    while (lo2 < hi2) {
      int mid = (lo2 + hi2) >> 1;
      if (tok_seq[mid] <= s) lo2 = mid + 1; else hi2 = mid;
    }
    s_rng[0] = lo;
    s_rng[1] = lo2;
  }
  __syncthreads();
  // page counts and never-used slots in the last page of every type: three lanes walk the three
  // dependent load chains (page count -> last page id -> fill count) side by side
  __shared__ int s_np[3], s_tail[3];
  if (tid < 3) {
    const int npk = v.n_pages[npages_index(c, s, layer, tid)];
    s_np[tid] = npk;
    s_tail[tid] = npk > 0 ? kPage - (int)v.page_filled[tid][v.block_table[table_base(c, s, layer, tid) + npk - 1]] : 0;
  }
  __syncthreads();
  const int lo = s_rng[0], hi = s_rng[1];
  SeqPlan pl;
  pl.lo = lo;
  pl.hi = hi;
  pl.pad = 0;
  for (int k = 0; k < 3; ++k) {
    pl.n[k] = pl.R[k] = pl.tail[k] = pl.need[k] = pl.grant[k] = pl.base[k] = 0;
    pl.np_old[k] = 0;
  }
  if (lo < hi) {
    // rank of every token among the call's tokens of its type: the three types' 0/1 flags are
    // scanned together, ten bits each (a chunk holds at most 256 tokens)
    int running[3] = {0, 0, 0};
    for (int b0 = lo; b0 < hi; b0 += 256) {
      const int i = b0 + tid;
      const int cl = i < hi ? (int)tok_class[i] : 3;
      const int flag = cl < 3 ? 1 << (10 * cl) : 0;
      int ex;
      const int tot = block_excl_scan(flag, &ex, s_scan);
      if (cl < 3) ws.tok_rank[i] = running[cl] + ((ex >> (10 * cl)) & 1023);
      for (int k = 0; k < 3; ++k) running[k] += (tot >> (10 * k)) & 1023;
    }
    // exclusive prefix of the reclaimable-slot counts over each page list: every thread takes a
    // contiguous run of pages of every type (all masks are requested before the first scan), so
    // one block scan per type suffices
    int mine[3], q0[3], q1[3];
    for (int k = 0; k < 3; ++k) {
      const uint32_t* msk = v.slot_mask + table_base(c, s, layer, k);
      const int np = s_np[k], per = (np + 255) / 256;
      q0[k] = tid * per;
      q1[k] = q0[k] + per < np ? q0[k] + per : np;
      mine[k] = 0;
      for (int pi = q0[k]; pi < q1[k]; ++pi) mine[k] += __popc(msk[pi] >> 16);
    }
    for (int k = 0; k < 3; ++k) {
      const uint32_t* msk = v.slot_mask + table_base(c, s, layer, k);
      int* pre = ws.pre + ((int64_t)s * 3 + k) * c.max_pages;
      const int np = s_np[k];
      int ex;
      const int runR = block_excl_scan(mine[k], &ex, s_scan);
      for (int pi = q0[k]; pi < q1[k]; ++pi) {
        pre[pi] = ex;
        ex += __popc(msk[pi] >> 16);
      }
      const int tail = s_tail[k];
      int need = running[k] - runR - tail;
      need = need > 0 ? (need + kPage - 1) / kPage : 0;
      const int room = c.max_pages - np;
      need = need < room ? need : room;
      pl.n[k] = running[k];
      pl.R[k] = runR;
      pl.tail[k] = tail;
      pl.np_old[k] = np;
      pl.need[k] = need;
    }
  }
  if (tid == 0) ws.plan[s] = pl;
  if (s == 0 && tid < 3) ws.avail_old[tid] = v.free_top[tid];   // the pools as the call finds them
}

// New pages of type k granted to sequence s: base = pages wanted by the sequences before s
// (pop order), grant = what the pool (avail pages when the call began) still covers of s's own
// need.  Called by every thread of the block.
__device__ inline void grant_of(const AppendWs& ws, int s, int k, int* base, int* grant, int* lds /*[5]*/) {
  const int avail = ws.avail_old[k];
  int before = 0;
  for (int t = threadIdx.x; t < s; t += 256) before += ws.plan[t].need[k];
  before = block_sum(before, lds);
  const int need = ws.plan[s].need[k];
  const int left = avail - before;
  *base = before < avail ? before : avail;
  *grant = left < 0 ? 0 : (left < need ? left : need);
}

__device__ void update_pools(const thinkv_view& v, const AppendWs& ws, int* s_scan);
__device__ void commit_sequence(const thinkv_view& v, int layer, const AppendWs& ws, int s, int* s_scan);

// ---------------------------------------------------------------------------------------------
// place: one block per (token, share of the kv-heads); every block of a token derives the same
// slot, block 0 records it.
template <int D>
__global__ __launch_bounds__(256) void append_place_kernel(thinkv_view v, int layer, const void* __restrict__ k_new,
                                                           const void* __restrict__ v_new, const int32_t* __restrict__ tok_seq,
                                                           const int32_t* __restrict__ tok_pos, const uint8_t* __restrict__ tok_class,
                                                           int32_t* __restrict__ tok_handle, int n_tok, int in_dtype, AppendWs ws,
                                                           int heads_per_block, int commit_here) {
  constexpr int NG = D / kGroup;        // groups per row
  constexpr int NM = D / 16;            // 16-channel blocks per row
  constexpr int HP = 256 / (2 * D);     // heads handled per pass
  __shared__ int s_place[7];            // type, page id, slot, ok, index in the page list, arrivals wanted, last to arrive
  __shared__ uint8_t s_codes[HP][2][D];
  __shared__ uint32_t s_meta[HP][2][NG];
  __shared__ uint8_t s_scale8[HP][2][D / kGroupFp];   // THINKV_FMT_FP: the E4M3 scale codes of the row's groups of 16
  const thinkv_config& c = v.cfg;
  const int i = blockIdx.x, tid = threadIdx.x;
  // the first input value of this thread is requested before the slot is settled: the slot takes a
  // chain of dependent loads, and a decode-style call is nothing but latency
  const int hs = tid / (2 * D), r = tid % (2 * D), kind = r / D, ch = r % D;
  const int h_first = blockIdx.y * heads_per_block + hs;
  const int h_end = (int)(blockIdx.y + 1) * heads_per_block < c.n_kv_heads ? (int)(blockIdx.y + 1) * heads_per_block : c.n_kv_heads;
  float x_first = 0.f;
  if (h_first < h_end) x_first = load_as_f32(kind ? v_new : k_new, ((int64_t)i * c.n_kv_heads + h_first) * D + ch, in_dtype);
  // slot selection.  Thread 0 settles every case that is a closed form; the page of the k-th
  // reclaimable slot (k < R) is found by all threads, each testing a stride of the page list.
  __shared__ int s_find[4];   // 1 = search wanted / 2 = grant wanted, sequence, type, rank
  __shared__ int s_scan[5];
  if (tid == 0) {
    int ok = 0, cls = 0, pid = 0, slot = 0, pi = 0, find = 0, k = 0, target = 0;
    const int s = tok_seq[i];
    if (s < 0 || s >= c.max_seqs) {
      atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
    } else {
      cls = tok_class[i];
      const SeqPlan& pl = ws.plan[s];
      // every block of every token inside the sequence's range reports to the sequence
      if (i >= pl.lo && i < pl.hi) target = (pl.hi - pl.lo) * (int)gridDim.y;
      if (cls > 2) {
        atomicOr(&v.dev_status[sl_index(c, s, layer)], THINKV_ST_BAD_CLASS);
      } else if (i >= pl.lo && i < pl.hi) {
        k = ws.tok_rank[i];
        const int32_t* tab = v.block_table + table_base(c, s, layer, cls);
        const int R = pl.R[cls], tail = pl.tail[cls], np = pl.np_old[cls];
        if (k < R) {
          find = 1;
        } else if (k < R + tail) {
          pi = np - 1;
          pid = tab[pi];
          slot = (int)v.page_filled[cls][pid] + (k - R);
          ok = 1;
        } else {
          find = 2;   // a new page: which one depends on the grant, worked out by the whole block
        }
      }
    }
    s_find[0] = find; s_find[1] = s; s_find[2] = cls; s_find[3] = k;
    s_place[0] = cls; s_place[1] = pid; s_place[2] = slot; s_place[3] = ok; s_place[4] = pi; s_place[5] = target;
  }
  __syncthreads();
  if (s_find[0] == 1) {
    const int s = s_find[1], cls = s_find[2], k = s_find[3];
    const int np = ws.plan[s].np_old[cls];
    const int64_t tb = table_base(c, s, layer, cls);
    const int* pre = ws.pre + ((int64_t)s * 3 + cls) * c.max_pages;
    for (int pi = tid; pi < np; pi += 256) {
      uint32_t e = v.slot_mask[tb + pi] >> 16;
      const int first = pre[pi];
      if (k >= first && k < first + (int)__popc(e)) {   // exactly one page of the list
        for (int j = k - first; j > 0; --j) e &= e - 1;
        s_place[1] = v.block_table[tb + pi];
        s_place[2] = __ffs(e) - 1;
        s_place[3] = 1;
        s_place[4] = pi;
      }
    }
    __syncthreads();
  }
  if (s_find[0] == 2) {
    const int s = s_find[1], cls = s_find[2], k = s_find[3];
    int base, grant;
    grant_of(ws, s, cls, &base, &grant, s_scan);
    if (tid == 0) {
      const SeqPlan& pl = ws.plan[s];
      const int kk = k - pl.R[cls] - pl.tail[cls], npi = kk >> 4;
      if (npi < grant) {
        s_place[1] = v.free_stack[cls][ws.avail_old[cls] - 1 - (base + npi)];
        s_place[2] = kk & 15;
        s_place[3] = 1;
        s_place[4] = pl.np_old[cls] + npi;
      }
    }
    __syncthreads();
  }
  if (tid == 0 && blockIdx.y == 0) {
    const int cls = s_place[0], pid = s_place[1], slot = s_place[2], ok = s_place[3], pi = s_place[4];
    if (ok) {
      v.slot_pos[cls][(int64_t)pid * kPage + slot] = tok_pos[i];
      atomicMax(&v.page_pos_max[cls][pid], tok_pos[i]);
    }
    if (tok_handle) tok_handle[i] = ok ? THINKV_HANDLE(cls, pi, slot) : -1;
  }
  __syncthreads();
  // Everything this block reads of the sequence's tables has been read.  Report; the block that
  // completes the sequence's count commits it (and puts the counter back to zero).
  if (tid == 0) {
    const int target = s_place[5], s = s_find[1];
    int last = 0;
    if (target > 0 && commit_here) {
      last = atomicAdd(&v.append_counters[s], 1u) == (uint32_t)target - 1u;
      if (last) v.append_counters[s] = 0u;
    }
    s_place[6] = last;
  }
  __syncthreads();
  if (s_place[6]) commit_sequence(v, layer, ws, s_find[1], s_scan);
  if (commit_here && blockIdx.x == 0 && blockIdx.y == 0) update_pools(v, ws, s_scan);
  __syncthreads();
  if (!s_place[3]) return;
  const int cls = s_place[0], pid = s_place[1], t = s_place[2];
  const int bits = c.bits_of_class[cls];
  const bool fp = c.format == THINKV_FMT_FP;
  const BlockGeom g = block_geom(bits, D, c.format);
  const int H = c.n_kv_heads;
  const float qmax = (float)((1 << bits) - 1);
  uint8_t* page = v.arena[cls] + (int64_t)pid * H * g.block_bytes;
  const int CB = g.chunk_bytes, FPH = 16 / bits, CPB = 8 / bits;  // codes per byte

  for (int h0 = blockIdx.y * heads_per_block; h0 < h_end; h0 += HP) {
    const int h = h0 + hs;
    if (h < h_end) {
      const void* src = kind ? v_new : k_new;
      const float x = h == h_first ? x_first : load_as_f32(src, ((int64_t)i * H + h) * D + ch, in_dtype);
      if (fp) {
        // the paper's formats: the ratio to the scale in binary64, as the formats are defined
        uint32_t code;
        if (bits == 8) {
          code = e4m3_encode((double)x / (double)c.fp8_scale[kind]);
        } else {
          float amax = fabsf(x);
#pragma unroll
          for (int d = 8; d >= 1; d >>= 1) amax = fmaxf(amax, __shfl_xor(amax, d, 64));
          const uint32_t sc8 = e4m3_code_up((double)amax / (bits == 4 ? 6.0 : 1.0));
          const double sd = (double)e4m3_value(sc8);
          const double r = sd > 0.0 ? (double)x / sd : 0.0;
          code = bits == 4 ? e2m1_encode(r) : ternary_encode(r);
          if ((ch & 15) == 0) s_scale8[hs][kind][ch >> 4] = (uint8_t)sc8;
        }
        s_codes[hs][kind][ch] = (uint8_t)code;
      } else {
      float mn = x, mx = x;
#pragma unroll
      for (int d = 16; d >= 1; d >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, d, 64));
        mx = fmaxf(mx, __shfl_xor(mx, d, 64));
      }
      const _Float16 zp = (_Float16)(mn + 0.0f);
      const float s32 = (mx - mn) / qmax;
      _Float16 sc = (_Float16)s32;
      if ((float)sc < s32) {
        uint16_t u = __builtin_bit_cast(uint16_t, sc);
        sc = __builtin_bit_cast(_Float16, (uint16_t)(u + 1));
      }
      const float sf = (float)sc, zf = (float)zp;
      float code = 0.0f;
      if (sf > 0.0f) {
        code = rintf((x - zf) / sf);
        code = fminf(fmaxf(code, 0.0f), qmax);
      }
      s_codes[hs][kind][ch] = (uint8_t)(int)code;
      if ((ch & 31) == 0)
        s_meta[hs][kind][ch >> 5] = (uint32_t)__builtin_bit_cast(uint16_t, sc) | ((uint32_t)__builtin_bit_cast(uint16_t, zp) << 16);
      }
    }
    __syncthreads();
    // pack: every destination byte the slot owns is assembled by one thread
    const int per_head = 8 * CB;  // 4*CB bytes of K codes + 4*CB bytes of V codes
    const int ph = tid / per_head, pr = tid % per_head;
    if (ph < HP && h0 + ph < H) {
      uint8_t* blk = page + (int64_t)(h0 + ph) * g.block_bytes;
      uint32_t byte = 0;
      if (pr < 4 * CB) {  // K: chunk 16*j + t, byte ob
        const int j = pr / CB, ob = pr % CB;
        const int w = ob >> 2, bo = (ob & 3) * 8, hh = bo >> 4, lf = (bo & 15) / bits;
        for (int q = 0; q < CPB; ++q) {
          const int f = w * FPH + lf + q;
          const int chn = 32 * (f >> 2) + 8 * j + 2 * (f & 3) + hh;
          byte |= (uint32_t)s_codes[ph][0][chn] << (q * bits);
        }
        blk[g.k_codes + (16 * j + t) * CB + ob] = (uint8_t)byte;
      } else {            // V: chunk 16*(t/4) + m, fields u*NM .. u*NM+NM-1 of half t%2
        const int vb = pr - 4 * CB, OB = CB / 4;
        const int m = vb / OB, kk = vb % OB;
        const int u = (t >> 1) & 1, hh = t & 1;
        const int f0 = u * NM + kk * CPB;
        const int off = 4 * (f0 / FPH) + 2 * hh + (bits * (f0 % FPH)) / 8;
        for (int q = 0; q < CPB; ++q) {
          const int mb = kk * CPB + q;
          byte |= (uint32_t)s_codes[ph][1][16 * mb + m] << (q * bits);
        }
        blk[g.v_codes + (16 * (t >> 2) + m) * CB + off] = (uint8_t)byte;
      }
    }
    if (fp) {
      constexpr int NG16 = D / kGroupFp;
      if (bits != 8 && tid < HP * 2 * NG16) {
        const int mh = tid / (2 * NG16), mr = tid % (2 * NG16), mk = mr / NG16, mg = mr % NG16;
        if (h0 + mh < H) (page + (int64_t)(h0 + mh) * g.block_bytes)[(mk ? g.v_meta : g.k_meta) + mg * kPage + t] = s_scale8[mh][mk][mg];
      }
    } else if (tid < HP * 2 * NG) {
      const int mh = tid / (2 * NG), mr = tid % (2 * NG), mk = mr / NG, mg = mr % NG;
      if (h0 + mh < H) {
        uint8_t* blk = page + (int64_t)(h0 + mh) * g.block_bytes;
        const uint32_t md = s_meta[mh][mk][mg];
        uint16_t* meta = (uint16_t*)(blk + (mk ? g.v_meta : g.k_meta));
        meta[meta_index(t, mg)] = (uint16_t)(md & 0xFFFFu);
        meta[meta_index(t, mg) + 4] = (uint16_t)(md >> 16);
      }
    }
    __syncthreads();
  }
}

// The pools after the call: what all sequences together were granted is gone.  (One block;
// nothing in the call reads free_top after the plan kernel's snapshot.)
__device__ void update_pools(const thinkv_view& v, const AppendWs& ws, int* s_scan /*[5]*/) {
  const int tid = threadIdx.x;
  for (int k = 0; k < 3; ++k) {
    int want = 0;
    for (int t = tid; t < v.cfg.max_seqs; t += 256) want += ws.plan[t].need[k];
    want = block_sum(want, s_scan);
    const int avail = ws.avail_old[k];
    if (tid == 0) v.free_top[k] = avail - (want < avail ? want : avail);
  }
}

// One block: masks, fill counts, page lists and counters of sequence s, once every place block
// of the sequence has settled its slot.
__device__ void commit_sequence(const thinkv_view& v, int layer, const AppendWs& ws, int s, int* s_scan /*[5]*/) {
  const thinkv_config& c = v.cfg;
  const int tid = threadIdx.x;
  const SeqPlan pl = ws.plan[s];
  if (pl.lo >= pl.hi) return;
  int placed_all = 0, short_any = 0;
  for (int k = 0; k < 3; ++k) {
    const int n = pl.n[k], R = pl.R[k], tail = pl.tail[k], np = pl.np_old[k];
    if (n == 0) continue;
    int base = 0, grant = 0;
    if (pl.need[k] > 0) grant_of(ws, s, k, &base, &grant, s_scan);
    int32_t* tab = v.block_table + table_base(c, s, layer, k);
    uint32_t* msk = v.slot_mask + table_base(c, s, layer, k);
    const int* pre = ws.pre + ((int64_t)s * 3 + k) * c.max_pages;
    for (int pi = tid; pi < np; pi += 256) {
      uint32_t m = msk[pi];
      uint32_t e = m >> 16;
      int take = n - pre[pi];
      const int have = __popc(e);
      take = take < 0 ? 0 : (take > have ? have : take);
      uint32_t bits = 0;
      for (int j = 0; j < take; ++j) {
        uint32_t b = e & (0u - e);
        bits |= b;
        e ^= b;
      }
      m = (m | bits) & ~(bits << 16);
      if (pi == np - 1 && tail > 0 && n > R) {
        const int add = (n - R) < tail ? (n - R) : tail;
        const int pid = tab[pi];
        const int f = v.page_filled[k][pid];
        m |= ((1u << add) - 1u) << f;
        v.page_filled[k][pid] = (uint8_t)(f + add);
      }
      msk[pi] = m;
    }
    for (int i = tid; i < grant; i += 256) {
      const int pid = v.free_stack[k][ws.avail_old[k] - 1 - (base + i)];
      int cnt = n - R - tail - kPage * i;
      cnt = cnt > kPage ? kPage : cnt;
      tab[np + i] = pid;
      v.page_filled[k][pid] = (uint8_t)cnt;
      msk[np + i] = (1u << cnt) - 1u;
      for (int sl = cnt; sl < kPage; ++sl) v.slot_pos[k][(int64_t)pid * kPage + sl] = -1;
    }
    const int cap = R + tail + kPage * grant;
    placed_all += n < cap ? n : cap;
    if (n > cap) short_any = 1;
    if (tid == 0) v.n_pages[npages_index(c, s, layer, k)] = np + grant;
  }
  if (tid == 0) {
    v.n_live[sl_index(c, s, layer)] += placed_all;
    if (short_any) atomicOr(&v.dev_status[sl_index(c, s, layer)], THINKV_ST_NOPAGES);
  }
}

// ---------------------------------------------------------------------------------------------
// Bulk calls (prefill-style: thousands of tokens).  One block per token pays the slot selection and
// eight short load-quantise-store passes for every token; here a block takes sixteen consecutive
// tokens of the call: sixteen threads settle their slots side by side, then every pass quantises
// one (kv-head, K or V) row of all sixteen tokens, eight channels per thread (one 16-byte load).
// K codes go straight from registers to the page: the eight channels of a thread are the fields
// of one 8-channel piece of a group, which the layout keeps together (8, 4 or 2 x 1 bytes).  V
// codes are transposed through LDS (a V chunk holds channels 16 apart).  The grants of new pages
// are worked out once, by a small kernel between plan and place.
__global__ __launch_bounds__(256) void append_grant_kernel(thinkv_view v, AppendWs ws) {
  __shared__ int s_scan[5];
  const int S = v.cfg.max_seqs, tid = threadIdx.x;
  for (int k = 0; k < 3; ++k) {
    const int avail = ws.avail_old[k];
    int run = 0;
    for (int s0 = 0; s0 < S; s0 += 256) {
      const int s = s0 + tid;
      const int need = s < S ? ws.plan[s].need[k] : 0;
      int ex;
      const int tot = block_excl_scan(need, &ex, s_scan);
      if (s < S) {
        const int before = run + ex, left = avail - before;
        ws.plan[s].base[k] = before < avail ? before : avail;
        ws.plan[s].grant[k] = left < 0 ? 0 : (left < need ? left : need);
      }
      run += tot;
    }
  }
}

constexpr int kBulkTokens = 16;   // tokens per block of the bulk place kernel

template <int D, bool F32>
__global__ __launch_bounds__(256) void append_place_bulk_kernel(thinkv_view v, int layer, const void* __restrict__ k_new,
                                                                const void* __restrict__ v_new, const int32_t* __restrict__ tok_seq,
                                                                const int32_t* __restrict__ tok_pos,
                                                                const uint8_t* __restrict__ tok_class, int32_t* __restrict__ tok_handle,
                                                                int n_tok, int in_dtype, AppendWs ws, int heads_per_block) {
  constexpr int NM = D / 16;            // 16-channel blocks per row
  constexpr int TPR = D / 8;            // threads per row
  constexpr int RPP = 256 / TPR;        // rows per pass: 16 (one (head, K or V) of all tokens) or 32 (one head, K and V)
  __shared__ int s_cls[kBulkTokens], s_pid[kBulkTokens], s_slot[kBulkTokens], s_ok[kBulkTokens], s_pi[kBulkTokens];
  __shared__ int s_find[kBulkTokens], s_seq[kBulkTokens], s_rank[kBulkTokens];
  __shared__ __attribute__((aligned(8))) uint8_t s_codes[2][kBulkTokens][D];
  const thinkv_config& c = v.cfg;
  const int tid = threadIdx.x, i0 = blockIdx.x * kBulkTokens;
  // this block's share of the kv-heads; the first input rows are requested before the slots are settled
  const int H = c.n_kv_heads;
  const int h_lo = blockIdx.y * heads_per_block, h_hi = h_lo + heads_per_block < H ? h_lo + heads_per_block : H;
  const int rsub = tid / TPR, cpiece = tid % TPR;          // row inside the pass, 8-channel piece of the row
  const int grp = cpiece >> 2, j = cpiece & 3;             // group of the piece, piece inside the group
  const int n_pass = (2 * (h_hi - h_lo) * kBulkTokens) / RPP;
  // row of this thread in pass p: always the same token (a pass holds whole runs of sixteen rows);
  // head and K or V change from pass to pass
  const int t = rsub % kBulkTokens;
  auto row_of = [&](int p, int* h, int* kind) {
    const int hk = (p * RPP + rsub) / kBulkTokens;
    *h = h_lo + (hk >> 1);
    *kind = hk & 1;
  };
  // the eight input values of this thread in pass p (16-bit inputs: one 16-byte word, binary32: two)
  const int64_t row_at = (int64_t)(i0 + t) * H * D + 8 * cpiece;
  constexpr int kW = F32 ? 2 : 1;
  struct Raw {
    uint4 w[kW];
  };
  auto fetch = [&](int p, Raw* r) {
    int h, kind;
    row_of(p, &h, &kind);
    if (p >= n_pass || i0 + t >= n_tok) return;   // (a token without a slot is loaded too: its slot is not known yet at the first call)
    const int64_t at = row_at + h * D;
    const void* src = kind ? v_new : k_new;
    if (F32) {
      r->w[0] = *(const uint4*)((const float*)src + at);
      r->w[kW - 1] = *(const uint4*)((const float*)src + at + 4);
    } else {
      r->w[0] = *(const uint4*)((const uint16_t*)src + at);
    }
  };
  // four passes are requested ahead: a pass is short, and one pass is not enough to cover a load
  constexpr int kAhead = 4;
  Raw cur[kAhead], nxt[kAhead];
#pragma unroll
  for (int q = 0; q < kAhead; ++q) {
#pragma unroll
    for (int i = 0; i < kW; ++i) cur[q].w[i] = nxt[q].w[i] = uint4{0u, 0u, 0u, 0u};
    fetch(q, &cur[q]);
  }
  // ---- slots: every case that is a closed form is settled by the token's own thread
  if (tid < kBulkTokens) {
    const int i = i0 + tid;
    int ok = 0, cls = 0, pid = 0, slot = 0, pi = 0, find = 0, k = 0, s = -1;
    if (i < n_tok) {
      s = tok_seq[i];
      if (s < 0 || s >= c.max_seqs) {
        atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
      } else {
        cls = tok_class[i];
        const SeqPlan& pl = ws.plan[s];
        if (cls > 2) {
          atomicOr(&v.dev_status[sl_index(c, s, layer)], THINKV_ST_BAD_CLASS);
        } else if (i >= pl.lo && i < pl.hi) {
          k = ws.tok_rank[i];
          const int32_t* tab = v.block_table + table_base(c, s, layer, cls);
          const int R = pl.R[cls], tail = pl.tail[cls], np = pl.np_old[cls];
          if (k < R) {
            find = 1;   // the k-th reclaimable slot: searched by the whole block below
          } else if (k < R + tail) {
            pi = np - 1;
            pid = tab[pi];
            slot = (int)v.page_filled[cls][pid] + (k - R);
            ok = 1;
          } else {
            const int kk = k - R - tail, npi = kk >> 4;
            if (npi < pl.grant[cls]) {
              pid = v.free_stack[cls][ws.avail_old[cls] - 1 - (pl.base[cls] + npi)];
              slot = kk & 15;
              pi = np + npi;
              ok = 1;
            }
          }
        }
      }
    }
    s_cls[tid] = cls; s_pid[tid] = pid; s_slot[tid] = slot; s_ok[tid] = ok; s_pi[tid] = pi;
    s_find[tid] = find; s_seq[tid] = s; s_rank[tid] = k;
  }
  __syncthreads();
  for (int t = 0; t < kBulkTokens; ++t) {
    if (s_find[t] != 1) continue;   // the same for all threads
    const int s = s_seq[t], cls = s_cls[t], k = s_rank[t];
    const int np = ws.plan[s].np_old[cls];
    const int64_t tb = table_base(c, s, layer, cls);
    const int* pre = ws.pre + ((int64_t)s * 3 + cls) * c.max_pages;
    for (int pi = tid; pi < np; pi += 256) {
      uint32_t e = v.slot_mask[tb + pi] >> 16;
      const int first = pre[pi];
      if (k >= first && k < first + (int)__popc(e)) {   // exactly one page of the list
        for (int j = k - first; j > 0; --j) e &= e - 1;
        s_pid[t] = v.block_table[tb + pi];
        s_slot[t] = __ffs(e) - 1;
        s_ok[t] = 1;
        s_pi[t] = pi;
      }
    }
  }
  __syncthreads();
  if (tid < kBulkTokens && i0 + tid < n_tok && blockIdx.y == 0) {
    const int i = i0 + tid, cls = s_cls[tid], pid = s_pid[tid], slot = s_slot[tid], ok = s_ok[tid];
    if (ok) {
      v.slot_pos[cls][(int64_t)pid * kPage + slot] = tok_pos[i];
      atomicMax(&v.page_pos_max[cls][pid], tok_pos[i]);
    }
    if (tok_handle) tok_handle[i] = ok ? THINKV_HANDLE(cls, s_pi[tid], slot) : -1;
  }
  // ---- quantise and store
  // what does not change from pass to pass: this thread's token as a quantiser thread ...
  const bool ok = s_ok[t] != 0;
  const int slot = s_slot[t];
  const int bits = c.bits_of_class[s_cls[t]];
  const bool fp = c.format == THINKV_FMT_FP;
  const BlockGeom gm = block_geom(bits, D, c.format);
  uint8_t* const page = v.arena[s_cls[t]] + (int64_t)s_pid[t] * H * gm.block_bytes;
  const float qmax = (float)((1 << bits) - 1);
  // ... and its (token, chunk) as a thread that packs V codes
  const int tv = tid >> 4, m = tid & 15;
  const bool v_ok = s_ok[tv] != 0;
  const int bv = c.bits_of_class[s_cls[tv]], slv = s_slot[tv];
  const BlockGeom gv = block_geom(bv, D, c.format);
  uint8_t* const v_chunk = v.arena[s_cls[tv]] + (int64_t)s_pid[tv] * H * gv.block_bytes + gv.v_codes +
                           (16 * (slv >> 2) + m) * gv.chunk_bytes + 2 * (slv & 1);
  const int v_u = (slv >> 1) & 1;
  auto pass = [&](int p, const Raw& raw) {
    int h, kind;
    row_of(p, &h, &kind);
    const bool has_v = RPP > kBulkTokens || (p & 1);       // some rows of this pass are V rows (the same for all threads)
    const int buf = (RPP > kBulkTokens ? p : p >> 1) & 1;
    uint8_t* blk = page + h * gm.block_bytes;
    if (ok) {
      float x[8];
      const uint4 r0 = raw.w[0], r1 = raw.w[kW - 1];
      const uint32_t w[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
      if (F32) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __builtin_bit_cast(float, w[e]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint16_t u = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
          x[e] = in_dtype == THINKV_F16 ? (float)__builtin_bit_cast(_Float16, u) : __builtin_bit_cast(float, (uint32_t)u << 16);
        }
      }
      uint32_t code[8];
      if (fp) {
        // the paper's formats: the eight channels of a thread lie in one group of 16 (number 2 grp + j / 2), which two
        // neighbour threads share; ratios to the scale in binary64, as the formats are defined
        double sd = (double)c.fp8_scale[kind];
        if (bits != 8) {
          float amax = fabsf(x[0]);
#pragma unroll
          for (int e = 1; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
          amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
          const uint32_t sc8 = e4m3_code_up((double)amax / (bits == 4 ? 6.0 : 1.0));
          sd = (double)e4m3_value(sc8);
          if ((j & 1) == 0) (blk + (kind ? gm.v_meta : gm.k_meta))[(2 * grp + (j >> 1)) * kPage + slot] = (uint8_t)sc8;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const double r = sd > 0.0 ? (double)x[e] / sd : 0.0;
          code[e] = bits == 8 ? e4m3_encode(r) : (bits == 4 ? e2m1_encode(r) : ternary_encode(r));
        }
      } else {
      float mn = x[0], mx = x[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) {
        mn = fminf(mn, x[e]);
        mx = fmaxf(mx, x[e]);
      }
#pragma unroll
      for (int d = 1; d <= 2; d <<= 1) {   // the four threads of a group are neighbours
        mn = fminf(mn, __shfl_xor(mn, d, 64));
        mx = fmaxf(mx, __shfl_xor(mx, d, 64));
      }
      const _Float16 zp = (_Float16)(mn + 0.0f);
      const float s32 = (mx - mn) / qmax;
      _Float16 sc = (_Float16)s32;
      if ((float)sc < s32) {
        uint16_t u = __builtin_bit_cast(uint16_t, sc);
        sc = __builtin_bit_cast(_Float16, (uint16_t)(u + 1));
      }
      const float sf = (float)sc, zf = (float)zp;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float q = 0.0f;
        if (sf > 0.0f) {
          q = rintf((x[e] - zf) / sf);
          q = fminf(fmaxf(q, 0.0f), qmax);
        }
        code[e] = (uint32_t)(int)q;
      }
      if (j == 0) {
        uint16_t* meta = (uint16_t*)(blk + (kind ? gm.v_meta : gm.k_meta));
        meta[meta_index(slot, grp)] = __builtin_bit_cast(uint16_t, sc);
        meta[meta_index(slot, grp) + 4] = __builtin_bit_cast(uint16_t, zp);
      }
      }
      if (!kind) {
        // K: channel 32 grp + 8 j + e is field 4 grp + e / 2, half e % 2, of chunk 16 j + slot
        uint8_t* chunk = blk + gm.k_codes + (16 * j + slot) * gm.chunk_bytes;
        if (bits == 8) {          // fields 4 grp .. + 3 are words 2 grp and 2 grp + 1
          uint32_t w0 = 0, w1 = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            w0 |= code[e] << (16 * (e & 1) + 8 * (e >> 1));
            w1 |= code[4 + e] << (16 * (e & 1) + 8 * (e >> 1));
          }
          *(uint2*)(chunk + 8 * grp) = uint2{w0, w1};
        } else if (bits == 4) {   // word grp
          uint32_t w0 = 0;
#pragma unroll
          for (int e = 0; e < 8; ++e) w0 |= code[e] << (16 * (e & 1) + 4 * (e >> 1));
          *(uint32_t*)(chunk + 4 * grp) = w0;
        } else {                  // a quarter of each half of word grp / 2
          uint32_t lo = 0, hi = 0;
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            lo |= code[e] << e;
            hi |= code[e + 1] << e;
          }
          chunk[4 * (grp >> 1) + (grp & 1)] = (uint8_t)lo;
          chunk[4 * (grp >> 1) + 2 + (grp & 1)] = (uint8_t)hi;
        }
      } else {
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          w0 |= code[e] << (8 * e);
          w1 |= code[4 + e] << (8 * e);
        }
        *(uint2*)&s_codes[buf][t][8 * cpiece] = uint2{w0, w1};
      }
    }
    if (has_v) {
      __syncthreads();
      // V: chunk 16 (slot / 4) + m holds channels m, m + 16, ... of four slots.  Thread (token, m)
      // packs the token's NM codes of the chunk: field u NM + mb of half hh (u, hh from the slot), i.e.
      // whole 16-bit halves of consecutive words, or one byte when a row has fewer fields than a half.
      const int hv = h_lo + (RPP > kBulkTokens ? p : p >> 1);   // the head whose V rows were just staged
      if (v_ok) {
        uint32_t cd[NM];
#pragma unroll
        for (int mb = 0; mb < NM; ++mb) cd[mb] = s_codes[buf][tv][16 * mb + m];
        uint8_t* chunk = v_chunk + hv * gv.block_bytes;        // already at the half word of the slot
        if (bv == 8) {
#pragma unroll
          for (int w = 0; w < NM / 2; ++w) *(uint16_t*)(chunk + 4 * (v_u * (NM / 2) + w)) = (uint16_t)(cd[2 * w] | cd[2 * w + 1] << 8);
        } else if (bv == 4) {
#pragma unroll
          for (int w = 0; w < NM / 4; ++w)
            *(uint16_t*)(chunk + 4 * (v_u * (NM / 4) + w)) =
                (uint16_t)(cd[4 * w] | cd[4 * w + 1] << 4 | cd[4 * w + 2] << 8 | cd[4 * w + 3] << 12);
        } else {
          uint32_t val = 0;
#pragma unroll
          for (int mb = 0; mb < NM; ++mb) val |= cd[mb] << (2 * mb);
          if (NM == 8)
            *(uint16_t*)(chunk + 4 * v_u) = (uint16_t)val;
          else
            chunk[v_u] = (uint8_t)val;
        }
      }
    }
  };
  for (int p0 = 0; p0 < n_pass; p0 += kAhead) {
#pragma unroll
    for (int q = 0; q < kAhead; ++q) fetch(p0 + kAhead + q, &nxt[q]);
#pragma unroll
    for (int q = 0; q < kAhead; ++q)
      if (p0 + q < n_pass) pass(p0 + q, cur[q]);
#pragma unroll
    for (int q = 0; q < kAhead; ++q) cur[q] = nxt[q];
  }
}

// bulk calls: one block per sequence after the place kernel
__global__ __launch_bounds__(256) void append_commit_kernel(thinkv_view v, int layer, AppendWs ws) {
  __shared__ int s_scan[5];
  if (blockIdx.x == 0) update_pools(v, ws, s_scan);
  commit_sequence(v, layer, ws, blockIdx.x, s_scan);
}

int launch_append(const thinkv_view& v, int layer, const void* k_new, const void* v_new, const int32_t* tok_seq,
                  const int32_t* tok_pos, const uint8_t* tok_class, int32_t* tok_handle, int n_tok, int in_dtype,
                  void* workspace, hipStream_t st, const int32_t* ev_seq, const int32_t* ev_handle, int n_ev) {
  AppendWs ws = carve(v.cfg, n_tok, workspace);
  const int S = v.cfg.max_seqs;
  hipLaunchKernelGGL(append_plan_kernel, dim3(S), dim3(256), 0, st, v, layer, tok_seq, tok_class, n_tok, ws, ev_seq, ev_handle, n_ev);
  const int commit_here = n_tok <= kBulkFrom;   // else thousands of blocks would bump one sequence's counter
  const bool aligned = (((uintptr_t)k_new | (uintptr_t)v_new) & 15) == 0;
  if (!commit_here && aligned) {
    hipLaunchKernelGGL(append_grant_kernel, dim3(1), dim3(256), 0, st, v, ws);
    // enough blocks to fill the chip: a mid-sized call spreads the kv-heads of its token groups over blocks
    const int H = v.cfg.n_kv_heads, groups = (n_tok + kBulkTokens - 1) / kBulkTokens;
    int hpb = (int)(((int64_t)H * groups + 4095) / 4096);
    hpb = hpb < 1 ? 1 : (hpb > H ? H : hpb);
    const dim3 grid(groups, (H + hpb - 1) / hpb);
    const bool f32 = in_dtype == THINKV_F32;
#define THINKV_BULK(DD, FF)                                                                                                   \
  hipLaunchKernelGGL((append_place_bulk_kernel<DD, FF>), grid, dim3(256), 0, st, v, layer, k_new, v_new, tok_seq, tok_pos, \
                     tok_class, tok_handle, n_tok, in_dtype, ws, hpb)
    if (v.cfg.head_dim == 128) {
      if (f32) THINKV_BULK(128, true); else THINKV_BULK(128, false);
    } else {
      if (f32) THINKV_BULK(64, true); else THINKV_BULK(64, false);
    }
#undef THINKV_BULK
  } else {
    // A decode-style call (few tokens) spreads the kv-heads of a token over several workgroups so
    // that their load-quantise-store chains run side by side; a bulk call whose rows are not
    // 16-byte aligned keeps one workgroup per token.
    const int H = v.cfg.n_kv_heads, hp = v.cfg.head_dim == 128 ? 1 : 2;
    const int hpb = commit_here ? hp : ((H + hp - 1) / hp) * hp;
    const dim3 grid(n_tok, (H + hpb - 1) / hpb);
    if (v.cfg.head_dim == 128)
      hipLaunchKernelGGL(append_place_kernel<128>, grid, dim3(256), 0, st, v, layer, k_new, v_new, tok_seq, tok_pos,
                         tok_class, tok_handle, n_tok, in_dtype, ws, hpb, commit_here);
    else
      hipLaunchKernelGGL(append_place_kernel<64>, grid, dim3(256), 0, st, v, layer, k_new, v_new, tok_seq, tok_pos,
                         tok_class, tok_handle, n_tok, in_dtype, ws, hpb, commit_here);
  }
  if (!commit_here) hipLaunchKernelGGL(append_commit_kernel, dim3(S), dim3(256), 0, st, v, layer, ws);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
