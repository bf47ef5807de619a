// Thought-adaptive eviction: which tokens of a thought segment survive (Sec. 4.3 of the paper,
// "Think Before you Evict"; appendix "TBE Eviction Policy").  A segment picked for eviction is
// cut down to K = min(|segment|, R_n) tokens by K-means over its post-RoPE keys: one
// representative key-value pair per cluster survives, the member nearest the centroid.
//
// The paper names K-means and nothing else.  What is built:
//   points     the token's stored keys, dequantised in binary32 (fmaf(code, scale, zp)), all
//              kv-heads concatenated (eviction is per token, so one clustering serves all heads)
//   K >= N     everything survives
//   init       centroid j = point floor(j * N / K)
//   Lloyd      nearest centroid by squared distance (ties -> lowest cluster); stop when no
//              assignment changed or after max_iters assignments; else centroids move to the
//              means of their points (an emptied cluster keeps its centroid)
//   survivors  per non-empty cluster the member nearest the centroid (ties -> lowest index; of
//              two members the earlier one: both are equally near their mean)
//
// Two kernels.  gather: one workgroup per token writes its key row [Hkv * D] into the workspace.
// kmeans: one workgroup of 256 threads per segment (segments hold at most 256 live tokens, the
// schedule keeps at most 64): lane L of every wave owns points L, L + 64, ..., wave w clusters
// 16w .. 16w + 15, so all threads are busy whatever the segment's size; the N x K distances are
// accumulated tile by tile (32 channels of all points and all centroids staged in LDS, up to 64
// accumulators per thread), the update sums the members of a cluster in index order (fixed summation order, so
// the result is the same on every run), and the survivor of a cluster is found with a 64-bit
// LDS minimum over (distance bits, index).  Plain binary32 FMAs on the vector ALU: the event is
// rare (segments are annealed when a transition thought ends or the budget is exceeded).
#include "common.h"

namespace thinkv {

constexpr int kTbeMaxTokens = THINKV_TBE_MAX_SEGMENT;   // live tokens of one segment
constexpr int kTbeMaxKeep = THINKV_TBE_MAX_KEEP;        // largest retention level
constexpr int kTile = 32;                               // channels per LDS tile
constexpr int kPad = 36;                                // row stride of a tile in floats (odd multiple of 16 bytes)

struct TbeArgs {
  const int32_t* tok_seq;
  const int32_t* tok_handle;
  const int32_t* seg_offset;
  const int32_t* seg_keep;
  int32_t* ev_handle;
  float* x;      // [n_tok][dim]
  float* cent;   // [n_seg][kTbeMaxKeep][dim]
  int layer, n_seg, n_tok, max_iters, dim;
};

size_t tbe_ws_bytes(const thinkv_config& c, int n_tok, int n_seg) {
  const size_t dim = (size_t)c.n_kv_heads * c.head_dim;
  return ((size_t)(n_tok > 0 ? n_tok : 1) * dim + (size_t)(n_seg > 0 ? n_seg : 1) * kTbeMaxKeep * dim) * sizeof(float) + 256;
}

// ---- gather: x[i][hd * D + ch] = the stored key of token i
__global__ __launch_bounds__(256) void tbe_gather_kernel(thinkv_view v, TbeArgs a) {
  const thinkv_config& c = v.cfg;
  const int i = blockIdx.x, tid = threadIdx.x;
  const int D = c.head_dim, H = c.n_kv_heads;
  float* row = a.x + (int64_t)i * a.dim;
  const int s = a.tok_seq[i];
  const uint32_t uh = (uint32_t)a.tok_handle[i];
  const int cls = uh >> 28, pi = (uh >> 4) & 0xFFFFFF, slot = uh & 15;
  bool ok = s >= 0 && s < c.max_seqs;
  if (!ok && tid == 0) atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
  if (ok && (a.tok_handle[i] < 0 || cls > 2 || pi >= v.n_pages[npages_index(c, s, a.layer, cls)])) {
    ok = false;
    if (tid == 0) atomicOr(&v.dev_status[sl_index(c, s, a.layer)], THINKV_ST_BAD_SLOT);
  }
  if (!ok) {   // a token that does not exist clusters as the origin and is never evicted
    for (int idx = tid; idx < a.dim; idx += 256) row[idx] = 0.f;
    return;
  }
  const int bits = c.bits_of_class[cls], FPH = 16 / bits;
  const uint32_t mask = (1u << bits) - 1u;
  const BlockGeom g = block_geom(bits, D);
  const int pid = v.block_table[table_base(c, s, a.layer, cls) + pi];
  const uint8_t* page = v.arena[cls] + (int64_t)pid * H * g.block_bytes;
  for (int idx = tid; idx < a.dim; idx += 256) {
    const int hd = idx / D, ch = idx % D;
    const uint8_t* blk = page + (int64_t)hd * g.block_bytes;
    const int grp = ch >> 5, chunk = 16 * ((ch & 31) >> 3) + slot;
    const int f = 4 * grp + ((ch & 7) >> 1), bit = 32 * (f / FPH) + 16 * (ch & 1) + bits * (f % FPH);
    const uint32_t word = ((const uint32_t*)(blk + g.k_codes + chunk * g.chunk_bytes))[bit >> 5];
    const float code = (float)((word >> (bit & 31)) & mask);
    const _Float16* meta = (const _Float16*)(blk + g.k_meta);
    row[idx] = fmaf(code, (float)meta[meta_index(slot, grp)], (float)meta[meta_index(slot, grp) + 4]);
  }
}

// ---- kmeans
constexpr int kPT = kTbeMaxTokens / 64;   // points per thread at most: lane L owns points L, L + 64, ...
constexpr int kKT = kTbeMaxKeep / 4;      // clusters per thread: wave w owns clusters kKT*w .. kKT*w + kKT-1

// Squared distances of this lane's points to this wave's clusters, accumulated over the channels.
// A wave reads the centroid rows as LDS broadcasts (all its lanes want the same cluster) and every
// lane its own point rows; pt = ceil(n / 64) points per lane are live.
__device__ inline void distances(const float* __restrict__ x, const float* __restrict__ cent, int n, int k, int dim, int pt,
                                 float (*xs)[kPad], float (*cs)[kPad], float (*acc)[kKT]) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int q = 0; q < kPT; ++q)
#pragma unroll
    for (int j = 0; j < kKT; ++j) acc[q][j] = 0.f;
  for (int d0 = 0; d0 < dim; d0 += kTile) {
    __syncthreads();
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int idx = tid; idx < 64 * pt * (kTile / 4); idx += 256) {
      const int r = idx / (kTile / 4), c4 = idx % (kTile / 4);
      *(float4*)&xs[r][4 * c4] = r < n ? *(const float4*)&x[(int64_t)r * dim + d0 + 4 * c4] : zero4;
    }
    for (int idx = tid; idx < kTbeMaxKeep * (kTile / 4); idx += 256) {
      const int r = idx / (kTile / 4), c4 = idx % (kTile / 4);
      *(float4*)&cs[r][4 * c4] = r < k ? *(const float4*)&cent[(int64_t)r * dim + d0 + 4 * c4] : zero4;
    }
    __syncthreads();
#pragma unroll 2
    for (int c4 = 0; c4 < kTile / 4; ++c4) {
      float4 xv[kPT];
#pragma unroll
      for (int q = 0; q < kPT; ++q)
        if (q < pt) xv[q] = *(const float4*)&xs[lane + 64 * q][4 * c4];
#pragma unroll
      for (int j = 0; j < kKT; ++j) {
        const float4 cv = *(const float4*)&cs[kKT * wave + j][4 * c4];
#pragma unroll
        for (int q = 0; q < kPT; ++q)
          if (q < pt) {
            const float e0 = xv[q].x - cv.x, e1 = xv[q].y - cv.y, e2 = xv[q].z - cv.z, e3 = xv[q].w - cv.w;
            acc[q][j] = fmaf(e3, e3, fmaf(e2, e2, fmaf(e1, e1, fmaf(e0, e0, acc[q][j]))));
          }
      }
    }
  }
}

__global__ __launch_bounds__(256) void tbe_kmeans_kernel(thinkv_view v, TbeArgs a) {
  const thinkv_config& c = v.cfg;
  const int seg = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = a.seg_offset[seg], hi = a.seg_offset[seg + 1];
  const int n = hi - lo, want = a.seg_keep[seg];
  if (n <= 0) return;
  if (n > kTbeMaxTokens || want > kTbeMaxKeep || want < 1 || lo < 0 || hi > a.n_tok) {
    // outside what this kernel covers: nothing is evicted, and the caller is told
    if (tid == 0) atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEGMENT);
    for (int i = tid; i < n && lo >= 0 && lo + i < a.n_tok; i += 256) a.ev_handle[lo + i] = -1;
    return;
  }
  if (want >= n) {
    for (int i = tid; i < n; i += 256) a.ev_handle[lo + i] = -1;
    return;
  }
  const int k = want, dim = a.dim, pt = (n + 63) / 64;
  const float* x = a.x + (int64_t)lo * dim;
  float* cent = a.cent + (int64_t)seg * kTbeMaxKeep * dim;
  __shared__ __attribute__((aligned(16))) float xs[kTbeMaxTokens][kPad];
  __shared__ __attribute__((aligned(16))) float cs[kTbeMaxKeep][kPad];
  __shared__ float s_bd[4][kTbeMaxTokens];   // per wave (cluster quarter): best distance of every point ...
  __shared__ int s_bj[4][kTbeMaxTokens];     // ... and the cluster it belongs to
  __shared__ int s_assign[kTbeMaxTokens], s_order[kTbeMaxTokens];
  __shared__ int s_cnt[kTbeMaxKeep], s_start[kTbeMaxKeep];
  __shared__ unsigned long long s_best[kTbeMaxKeep];
  // initial centroids: evenly spaced points
  for (int idx = tid; idx < k * dim; idx += 256) {
    const int j = idx / dim, d = idx % dim;
    cent[idx] = x[(int64_t)((j * n) / k) * dim + d];
  }
  float acc[kPT][kKT];
  int mine[kPT];
#pragma unroll
  for (int q = 0; q < kPT; ++q) mine[q] = -1;
  // nearest cluster of this lane's points: best of this wave's quarter, then best of the four quarters
  // (ties go to the lowest cluster: quarters and clusters are scanned in ascending order)
  auto assign = [&](int* out) {
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      float bd = INFINITY;
      int bj = 0;
#pragma unroll
      for (int j = 0; j < kKT; ++j)
        if (kKT * wave + j < k && acc[q][j] < bd) {
          bd = acc[q][j];
          bj = kKT * wave + j;
        }
      s_bd[wave][lane + 64 * q] = bd;
      s_bj[wave][lane + 64 * q] = bj;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      float bd = s_bd[0][lane + 64 * q];
      int bj = s_bj[0][lane + 64 * q];
#pragma unroll
      for (int w = 1; w < 4; ++w)
        if (s_bd[w][lane + 64 * q] < bd) {
          bd = s_bd[w][lane + 64 * q];
          bj = s_bj[w][lane + 64 * q];
        }
      out[q] = bj;
    }
  };
  for (int it = 0; it < a.max_iters; ++it) {
    distances(x, cent, n, k, dim, pt, xs, cs, acc);
    int now[kPT];
    assign(now);
    int changed = 0;
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      changed |= (lane + 64 * q < n) && now[q] != mine[q];
      mine[q] = now[q];
    }
    if (!__syncthreads_or(changed)) break;
    // ---- update: members of every cluster in index order
    if (tid < kTbeMaxKeep) s_cnt[tid] = 0;
    if (wave == 0) {
#pragma unroll
      for (int q = 0; q < kPT; ++q)
        if (lane + 64 * q < n) s_assign[lane + 64 * q] = mine[q];
    }
    __syncthreads();
    if (tid < n) {
      const int cl = s_assign[tid];
      int rank = 0;
      for (int i = 0; i < tid; ++i) rank += s_assign[i] == cl;
      atomicAdd(&s_cnt[cl], 1);
      s_order[tid] = rank;   // position among the cluster's members, for now
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int j = 0; j < k; ++j) {
        s_start[j] = run;
        run += s_cnt[j];
      }
    }
    __syncthreads();
    int slot = -1;
    if (tid < n) slot = s_start[s_assign[tid]] + s_order[tid];
    __syncthreads();
    if (tid < n) s_order[slot] = tid;
    __syncthreads();
    for (int j = 0; j < k; ++j) {
      const int m = s_cnt[j];
      if (m == 0) continue;
      const float inv = 1.0f / (float)m;
      for (int d = tid; d < dim; d += 256) {
        float sum = 0.f;
        for (int r = 0; r < m; ++r) sum += x[(int64_t)s_order[s_start[j] + r] * dim + d];
        cent[(int64_t)j * dim + d] = sum * inv;
      }
    }
    __syncthreads();
  }
  // ---- survivors: nearest member of every cluster under the final centroids
  distances(x, cent, n, k, dim, pt, xs, cs, acc);
  if (tid < kTbeMaxKeep) {
    s_cnt[tid] = 0;
    s_start[tid] = kTbeMaxTokens;   // here: lowest index among the cluster's members
    s_best[tid] = ~0ull;
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kPT; ++q) {
    const int p = lane + 64 * q;
    if (p < n && mine[q] / kKT == wave) {   // the wave that holds the distance to the point's own cluster
      float own = 0.f;
#pragma unroll
      for (int j = 0; j < kKT; ++j)
        if (j == mine[q] % kKT) own = acc[q][j];
      atomicAdd(&s_cnt[mine[q]], 1);
      atomicMin(&s_start[mine[q]], p);
      // distances are not negative, so their bit patterns order like the numbers; the index breaks ties
      atomicMin(&s_best[mine[q]], ((unsigned long long)__builtin_bit_cast(uint32_t, own) << 32) | (unsigned)p);
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      const int p = lane + 64 * q;
      if (p < n) {
        // two members are equally near their mean whatever the rounding says: the earlier one stays
        const bool keep = s_cnt[mine[q]] <= 2 ? p == s_start[mine[q]] : (int)(s_best[mine[q]] & 0xFFFFFFFFull) == p;
        a.ev_handle[lo + p] = keep ? -1 : a.tok_handle[lo + p];
      }
    }
  }
}

int launch_tbe_select(const thinkv_view& v, int layer, const int32_t* tok_seq, const int32_t* tok_handle, const int32_t* seg_offset,
                      const int32_t* seg_keep, int n_seg, int n_tok, int max_iters, int32_t* ev_handle, void* workspace,
                      hipStream_t st) {
  TbeArgs a;
  a.tok_seq = tok_seq;
  a.tok_handle = tok_handle;
  a.seg_offset = seg_offset;
  a.seg_keep = seg_keep;
  a.ev_handle = ev_handle;
  a.dim = v.cfg.n_kv_heads * v.cfg.head_dim;
  a.x = (float*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.cent = a.x + (size_t)n_tok * a.dim;
  a.layer = layer;
  a.n_seg = n_seg;
  a.n_tok = n_tok;
  a.max_iters = max_iters;
  hipLaunchKernelGGL(tbe_gather_kernel, dim3(n_tok), dim3(256), 0, st, v, a);
  hipLaunchKernelGGL(tbe_kmeans_kernel, dim3(n_seg), dim3(256), 0, st, v, a);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

// ---------------------------------------------------------------------------------------------
// The plan: which segments of which sequences are cut, and to how many tokens (Sec. 4.3: Case 1,
// every preceding segment goes down one retention level when a transition segment has ended;
// Case 2, while the sequence holds more live tokens than the budget, the oldest segment of the
// least important type that can still shrink goes down one level).  A segment is cut at most
// once per call (one K-means per segment and call); its level follows from its live size: it is
// cut to the largest retention value below that size.  The open (last) segment is never touched.
// A live token belongs to the segment whose start is the largest one not above its position
// (the block table's start-index column, Sec. 5.2).
//
// Four kernels.  count (one workgroup per examined sequence): live tokens per segment (every
// thread takes pages of the sequence's three lists and reads a page's sixteen positions as four
// vectors; binary search of each live slot's position in the segment starts, held in LDS), then
// one thread walks the plan and leaves the sequence's cuts in a staging area.  offsets (one
// workgroup): every sequence's place in the dense output lists; a sequence whose cuts no longer
// all fit the caller's buffers keeps the leading ones that do (the rest waits for the next call).
// fill (one workgroup per sequence): list offsets of the sequence's cuts by a prefix sum, then its
// live tokens are dealt to their lists.  sort (one wave per cut): each list is put in ascending
// position by a rank sort in LDS, so the output does not depend on the order in which threads
// got there.
constexpr int kMaxSegs = THINKV_TBE_MAX_SEGS;
constexpr int kRetention[5] = {64, 32, 16, 8, 4};
constexpr int kPlanThreads = 1024;

struct PlanArgs {
  const int32_t* seq_ids;
  const int32_t* seg_start;
  const uint8_t* seg_type;
  const int32_t* n_segs;
  const uint8_t* transition_ended;
  int32_t* tok_seq;
  int32_t* tok_handle;
  int32_t* seg_offset;
  int32_t* seg_keep;
  int32_t* counts;
  // staging: per examined sequence max_cuts entries of (segment, keep, live tokens); the number of
  // cuts and of their tokens; the sequence's first cut / first token in the dense lists; per cut of
  // the dense lists the sequence it belongs to
  int32_t* st_seg;
  int32_t* st_keep;
  int32_t* st_cnt;
  int32_t* st_ncuts;
  int32_t* st_total;
  int32_t* st_seg_base;
  int32_t* st_tok_base;
  int32_t* st_cut_seq;
  int layer, B, max_segs, budget, max_cuts, cap_seg, cap_tok;
};

size_t tbe_plan_ws_bytes(int B, int max_cuts) {
  return ((size_t)(B > 0 ? B : 1) * (4 * (size_t)max_cuts + 4)) * sizeof(int32_t) + 256;
}

__device__ inline int next_level(int size) {
#pragma unroll
  for (int i = 0; i < 5; ++i)
    if (kRetention[i] < size) return kRetention[i];
  return 0;
}

// segment of position pos: index of the last start <= pos, -1 if there is none
__device__ inline int segment_of(const int* starts, int n, int pos) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (starts[mid] <= pos) lo = mid + 1; else hi = mid;
  }
  return lo - 1;
}

// calls f(segment, position, handle) for every live token of the sequence; every thread takes pages
template <typename F>
__device__ inline void for_live_tokens(const thinkv_view& v, int seq, int layer, const int* s_start, int ns, F f) {
  const thinkv_config& c = v.cfg;
  for (int k = 0; k < 3; ++k) {
    const int np = v.n_pages[npages_index(c, seq, layer, k)];
    const int64_t tb = table_base(c, seq, layer, k);
    for (int pi = threadIdx.x; pi < np; pi += blockDim.x) {
      const uint32_t m = v.slot_mask[tb + pi] & 0xFFFFu;
      if (!m) continue;
      const int pid = v.block_table[tb + pi];
      const int4* sp = (const int4*)(v.slot_pos[k] + (int64_t)pid * kPage);
      int pos[kPage];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int4 w = sp[q];
        pos[4 * q] = w.x; pos[4 * q + 1] = w.y; pos[4 * q + 2] = w.z; pos[4 * q + 3] = w.w;
      }
#pragma unroll
      for (int slot = 0; slot < kPage; ++slot) {
        if (!(m >> slot & 1)) continue;
        const int sg = segment_of(s_start, ns, pos[slot]);
        if (sg >= 0) f(sg, pos[slot], THINKV_HANDLE(k, pi, slot));
      }
    }
  }
}

__global__ __launch_bounds__(kPlanThreads) void tbe_count_plan_kernel(thinkv_view v, PlanArgs a) {
  const thinkv_config& c = v.cfg;
  const int b = blockIdx.x, tid = threadIdx.x;
  __shared__ int s_start[kMaxSegs];
  __shared__ int s_cnt[kMaxSegs];
  __shared__ uint8_t s_type[kMaxSegs];
  const int seq = a.seq_ids[b];
  if (seq < 0 || seq >= c.max_seqs) {
    if (tid == 0) {
      atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
      a.st_ncuts[b] = 0;
      a.st_total[b] = 0;
    }
    return;
  }
  int ns = a.n_segs[seq];
  ns = ns < 0 ? 0 : (ns > a.max_segs ? a.max_segs : ns);
  const int32_t* starts = a.seg_start + (int64_t)seq * a.max_segs;
  const uint8_t* types = a.seg_type + (int64_t)seq * a.max_segs;
  for (int i = tid; i < ns; i += kPlanThreads) {
    s_start[i] = starts[i];
    s_type[i] = types[i];
    s_cnt[i] = 0;
  }
  __syncthreads();
  for_live_tokens(v, seq, a.layer, s_start, ns, [&](int sg, int, int) { atomicAdd(&s_cnt[sg], 1); });
  __syncthreads();
  if (tid != 0) return;
  int total = v.n_live[sl_index(c, seq, a.layer)];
  int n_cuts = 0, listed = 0;
  bool oversize = false;
  int32_t* o_seg = a.st_seg + (int64_t)b * a.max_cuts;
  int32_t* o_keep = a.st_keep + (int64_t)b * a.max_cuts;
  int32_t* o_cnt = a.st_cnt + (int64_t)b * a.max_cuts;
  auto cut = [&](int i, int r) {
    o_seg[n_cuts] = i;
    o_keep[n_cuts] = r;
    o_cnt[n_cuts] = s_cnt[i];
    ++n_cuts;
    listed += s_cnt[i];
    total -= s_cnt[i] - r;
    s_cnt[i] = -r;          // negative: cut in this call, now holding r tokens
  };
  const int last = ns - 1;
  if (a.transition_ended && a.transition_ended[b]) {
    for (int i = 0; i < last && n_cuts < a.max_cuts; ++i) {
      const int r = next_level(s_cnt[i]);
      if (!r) continue;
      if (s_cnt[i] > kTbeMaxTokens) {
        oversize = true;
        continue;
      }
      cut(i, r);
    }
  }
  // Case 2.  A segment that cannot be cut now cannot be cut later in this call either (one cut per
  // segment and call), so "the oldest segment of the least important type that can still shrink",
  // asked again after every cut, is one walk over the types in order of importance and over the
  // segments of each from the oldest on.
  for (int t = 0; t < 3; ++t)
    for (int i = 0; i < last && total > a.budget && n_cuts < a.max_cuts; ++i) {
      if (s_type[i] != t || s_cnt[i] < 0) continue;
      const int r = next_level(s_cnt[i]);
      if (!r) continue;
      if (s_cnt[i] > kTbeMaxTokens) {
        oversize = true;
        continue;
      }
      cut(i, r);
    }
  a.st_ncuts[b] = n_cuts;
  a.st_total[b] = listed;
  if (oversize) atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEGMENT);
}

// exclusive prefix sum over one value per lane of wave 0 times four (values [4 * lane, 4 * lane + 4) of a
// list of at most 256); returns the four exclusive sums through ex[] and the total
__device__ inline int wave_scan4(const int* val, int* ex) {
  const int lane = threadIdx.x & 63;
  int inc = val[0] + val[1] + val[2] + val[3];
  const int mine = inc;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d, 64);
    if (lane >= d) inc += o;
  }
  const int total = __shfl(inc, 63, 64);
  int run = inc - mine;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    ex[q] = run;
    run += val[q];
  }
  return total;
}

__global__ __launch_bounds__(64) void tbe_offsets_kernel(PlanArgs a) {
  // one wave: sequences in order (their number is that of a decode batch); a sequence whose cuts all
  // fit is placed from its two totals, only one that does not is looked at cut by cut
  const int lane = threadIdx.x;
  int n_seg = 0, n_tok = 0;
  for (int b = 0; b < a.B; ++b) {
    const int nc = a.st_ncuts[b], tot = a.st_total[b];
    int kept = nc, kept_tok = tot;
    if (n_seg + nc > a.cap_seg || (int64_t)n_tok + tot > a.cap_tok) {
      // leading cuts that still fit (the lists only grow, so the first that does not fit ends them)
      int val[4], ex[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) val[q] = 4 * lane + q < nc ? a.st_cnt[(int64_t)b * a.max_cuts + 4 * lane + q] : 0;
      wave_scan4(val, ex);
      int fits = 0, fits_tok = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = 4 * lane + q;
        if (i < nc && n_seg + i < a.cap_seg && (int64_t)n_tok + ex[q] + val[q] <= a.cap_tok) {
          ++fits;
          fits_tok += val[q];
        }
      }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        fits += __shfl_xor(fits, d, 64);
        fits_tok += __shfl_xor(fits_tok, d, 64);
      }
      kept = fits;
      kept_tok = fits_tok;
    }
    if (lane == 0) {
      a.st_seg_base[b] = n_seg;
      a.st_tok_base[b] = n_tok;
      a.st_ncuts[b] = kept;
    }
    n_seg += kept;
    n_tok += kept_tok;
  }
  if (lane == 0) {
    a.seg_offset[n_seg] = n_tok;
    a.counts[0] = n_seg;
    a.counts[1] = n_tok;
  }
}

__global__ __launch_bounds__(kPlanThreads) void tbe_fill_kernel(thinkv_view v, PlanArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int n_cuts = a.st_ncuts[b];
  if (n_cuts == 0) return;
  __shared__ int s_start[kMaxSegs];
  __shared__ int s_cut[kMaxSegs];                 // cut number of a segment, -1 = not cut
  __shared__ int s_fill[kTbeMaxTokens];           // tokens dealt to a cut so far (cuts per sequence <= 256, checked on the host)
  __shared__ int s_off[kTbeMaxTokens];            // first token of a cut's list
  const int seq = a.seq_ids[b];
  int ns = a.n_segs[seq];
  ns = ns < 0 ? 0 : (ns > a.max_segs ? a.max_segs : ns);
  const int32_t* starts = a.seg_start + (int64_t)seq * a.max_segs;
  for (int i = tid; i < ns; i += kPlanThreads) {
    s_start[i] = starts[i];
    s_cut[i] = -1;
  }
  const int seg_base = a.st_seg_base[b], tok_base = a.st_tok_base[b];
  if (tid < 64) {
    int val[4], ex[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) val[q] = 4 * tid + q < n_cuts ? a.st_cnt[(int64_t)b * a.max_cuts + 4 * tid + q] : 0;
    wave_scan4(val, ex);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = 4 * tid + q;
      if (i < n_cuts) {
        s_off[i] = tok_base + ex[q];
        s_fill[i] = 0;
        a.seg_offset[seg_base + i] = tok_base + ex[q];
        a.seg_keep[seg_base + i] = a.st_keep[(int64_t)b * a.max_cuts + i];
        a.st_cut_seq[seg_base + i] = seq;
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < n_cuts; i += kPlanThreads) s_cut[a.st_seg[(int64_t)b * a.max_cuts + i]] = i;
  __syncthreads();
  // deal the tokens: position into tok_seq for now, handle into tok_handle
  for_live_tokens(v, seq, a.layer, s_start, ns, [&](int sg, int pos, int h) {
    const int cu = s_cut[sg];
    if (cu < 0) return;
    const int at = s_off[cu] + atomicAdd(&s_fill[cu], 1);
    a.tok_seq[at] = pos;
    a.tok_handle[at] = h;
  });
}

// one wave per cut of the dense lists: ascending position inside the list
__global__ __launch_bounds__(256) void tbe_sort_kernel(PlanArgs a) {
  __shared__ int s_pos[4][kTbeMaxTokens];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cu = blockIdx.x * 4 + wave;
  const bool live = cu < a.counts[0];
  int lo = 0, n = 0, pos[kPT], h[kPT];
  if (live) {
    lo = a.seg_offset[cu];
    n = a.seg_offset[cu + 1] - lo;   // at most kTbeMaxTokens: larger segments are never cut
#pragma unroll
    for (int q = 0; q < kPT; ++q)
      if (lane + 64 * q < n) {
        pos[q] = a.tok_seq[lo + lane + 64 * q];
        h[q] = a.tok_handle[lo + lane + 64 * q];
        s_pos[wave][lane + 64 * q] = pos[q];
      }
  }
  __syncthreads();
  if (!live) return;
  const int seq = a.st_cut_seq[cu];
  int rank[kPT];
#pragma unroll
  for (int q = 0; q < kPT; ++q) rank[q] = 0;
  for (int i = 0; i < n; ++i) {
    const int other = s_pos[wave][i];
#pragma unroll
    for (int q = 0; q < kPT; ++q) rank[q] += other < pos[q] || (other == pos[q] && i < lane + 64 * q);
  }
#pragma unroll
  for (int q = 0; q < kPT; ++q)
    if (lane + 64 * q < n) {
      a.tok_handle[lo + rank[q]] = h[q];
      a.tok_seq[lo + rank[q]] = seq;
    }
}

int launch_tbe_plan(const thinkv_view& v, int layer, const int32_t* seq_ids, const int32_t* seg_start, const uint8_t* seg_type,
                    const int32_t* n_segs, const uint8_t* transition_ended, int B, int max_segs, int budget, int max_cuts,
                    int cap_seg, int cap_tok, int32_t* tok_seq, int32_t* tok_handle, int32_t* seg_offset, int32_t* seg_keep,
                    int32_t* counts, void* workspace, hipStream_t st) {
  PlanArgs a;
  a.seq_ids = seq_ids;
  a.seg_start = seg_start;
  a.seg_type = seg_type;
  a.n_segs = n_segs;
  a.transition_ended = transition_ended;
  a.tok_seq = tok_seq;
  a.tok_handle = tok_handle;
  a.seg_offset = seg_offset;
  a.seg_keep = seg_keep;
  a.counts = counts;
  int32_t* w = (int32_t*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  a.st_seg = w;
  a.st_keep = w + (size_t)B * max_cuts;
  a.st_cnt = w + 2 * (size_t)B * max_cuts;
  a.st_cut_seq = w + 3 * (size_t)B * max_cuts;
  a.st_ncuts = w + 4 * (size_t)B * max_cuts;
  a.st_total = a.st_ncuts + B;
  a.st_seg_base = a.st_total + B;
  a.st_tok_base = a.st_seg_base + B;
  a.layer = layer;
  a.B = B;
  a.max_segs = max_segs;
  a.budget = budget;
  a.max_cuts = max_cuts;
  a.cap_seg = cap_seg;
  a.cap_tok = cap_tok;
  if (B > 0) hipLaunchKernelGGL(tbe_count_plan_kernel, dim3(B), dim3(kPlanThreads), 0, st, v, a);
  hipLaunchKernelGGL(tbe_offsets_kernel, dim3(1), dim3(64), 0, st, a);
  if (B > 0) hipLaunchKernelGGL(tbe_fill_kernel, dim3(B), dim3(kPlanThreads), 0, st, v, a);
  const int64_t most = (int64_t)B * max_cuts < cap_seg ? (int64_t)B * max_cuts : cap_seg;
  if (most > 0) hipLaunchKernelGGL(tbe_sort_kernel, dim3((unsigned)((most + 3) / 4)), dim3(256), 0, st, a);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
