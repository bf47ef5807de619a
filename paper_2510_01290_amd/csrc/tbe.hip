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
// kmeans: one workgroup of sixteen waves per segment (segments hold at most 256 live tokens, the
// schedule keeps at most 64).  Squared distances are taken as |x|^2 - 2 x.c + |c|^2 with the
// products x.c of all points with all centroids on the matrix cores; a dequantised key does not
// fit binary16 and the binary32 matrix instruction is slow, so every number enters as the sum of
// two binary16 parts (22 significant bits) and a product is three binary16 MFMAs.  The error of
// all this is of the order of 1e-6 of |x|^2, far below the gaps that separate genuine decisions;
// an assignment only needs |c|^2 - 2 x.c.  The channels go through LDS 64 at a time, the centroid
// update is folded into the next pass over the channels (a cluster's members are summed from the
// point tile that is in LDS anyway, in index order, so the result is the same on every run), and
// the survivor of a cluster is found with a 64-bit LDS minimum over (distance bits, index).
#include "common.h"

namespace thinkv {

constexpr int kTbeMaxTokens = THINKV_TBE_MAX_SEGMENT;   // live tokens of one segment
constexpr int kTbeMaxKeep = THINKV_TBE_MAX_KEEP;        // largest retention level
constexpr int kTile = 64;                               // channels per LDS tile

struct TbeArgs {
  const int32_t* tok_seq;
  const int32_t* tok_handle;
  const int32_t* seg_offset;
  const int32_t* seg_keep;
  int32_t* ev_handle;
  float* x;      // [n_tok][dim]
  float* cent;   // [n_seg][kTbeMaxKeep][dim]
  int32_t* assign;   // [n_tok] cluster of every token at the last assignment (-1: its segment was not clustered)
  int layer, n_seg, n_tok, max_iters, dim;
};

size_t tbe_ws_bytes(const thinkv_config& c, int n_tok, int n_seg) {
  const size_t dim = (size_t)c.n_kv_heads * c.head_dim;
  return ((size_t)(n_tok > 0 ? n_tok : 1) * dim + (size_t)(n_seg > 0 ? n_seg : 1) * kTbeMaxKeep * dim) * sizeof(float) +
         (size_t)(n_tok > 0 ? n_tok : 1) * sizeof(int32_t) + 256;
}

// ---- gather: x[i][hd * D + ch] = the stored key of token i.  A workgroup takes kGatherTokens tokens:
// one thread per token walks the chain handle -> page list -> page, then all threads extract codes.
constexpr int kGatherTokens = 8;

__global__ __launch_bounds__(256) void tbe_gather_kernel(thinkv_view v, TbeArgs a) {
  const thinkv_config& c = v.cfg;
  const int tid = threadIdx.x, i0 = blockIdx.x * kGatherTokens;
  const int D = c.head_dim, H = c.n_kv_heads, ld = D == 128 ? 7 : 6;
  __shared__ int s_ok[kGatherTokens], s_cls[kGatherTokens], s_slot[kGatherTokens], s_pid[kGatherTokens];
  if (tid < kGatherTokens) {
    const int i = i0 + tid;
    int ok = 0, cls = 0, slot = 0, pid = 0;
    if (i < a.n_tok) {
      const int s = a.tok_seq[i];
      const int32_t h = a.tok_handle[i];
      const uint32_t uh = (uint32_t)h;
      cls = uh >> 28;
      slot = uh & 15;
      const int pi = (uh >> 4) & 0xFFFFFF;
      if (s < 0 || s >= c.max_seqs) {
        atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
      } else if (h < 0 || cls > 2 || pi >= v.n_pages[npages_index(c, s, a.layer, cls)]) {
        atomicOr(&v.dev_status[sl_index(c, s, a.layer)], THINKV_ST_BAD_SLOT);
      } else {
        pid = v.block_table[table_base(c, s, a.layer, cls) + pi];
        ok = 1;
      }
    }
    s_ok[tid] = ok; s_cls[tid] = cls; s_slot[tid] = slot; s_pid[tid] = pid;
  }
  __syncthreads();
  for (int t = 0; t < kGatherTokens && i0 + t < a.n_tok; ++t) {
    float* row = a.x + (int64_t)(i0 + t) * a.dim;
    if (!s_ok[t]) {   // a token that does not exist clusters as the origin and is never evicted
      for (int idx = tid; idx < a.dim; idx += 256) row[idx] = 0.f;
      continue;
    }
    const int cls = s_cls[t], slot = s_slot[t];
    const int bits = c.bits_of_class[cls];
    const int lb = bits == 8 ? 3 : (bits == 4 ? 2 : 1), lf = 4 - lb;   // log2 of the bits per code and of the fields per half word
    const uint32_t mask = (1u << bits) - 1u;
    const bool fp = c.format == THINKV_FMT_FP;
    const BlockGeom g = block_geom(bits, D, c.format);
    const uint8_t* page = v.arena[cls] + (int64_t)s_pid[t] * H * g.block_bytes;
    for (int idx = tid; idx < a.dim; idx += 256) {
      const int hd = idx >> ld, ch = idx & (D - 1);
      const uint8_t* blk = page + (int64_t)hd * g.block_bytes;
      const int grp = ch >> 5, chunk = 16 * ((ch & 31) >> 3) + slot;
      const int f = 4 * grp + ((ch & 7) >> 1), bit = 32 * (f >> lf) + 16 * (ch & 1) + ((f & ((1 << lf) - 1)) << lb);
      const uint32_t word = ((const uint32_t*)(blk + g.k_codes + chunk * g.chunk_bytes))[bit >> 5];
      const uint32_t raw = (word >> (bit & 31)) & mask;
      if (fp) {   // the paper's formats: value of the code times the tensor's scale or the E4M3 scale of the channel's group of 16
        const float sc = bits == 8 ? c.fp8_scale[0] : e4m3_value(blk[g.k_meta + (ch >> 4) * kPage + slot]);
        row[idx] = fp_code_value(raw, bits) * sc;
        continue;
      }
      const float code = (float)raw;
      const _Float16* meta = (const _Float16*)(blk + g.k_meta);
      row[idx] = fmaf(code, (float)meta[meta_index(slot, grp)], (float)meta[meta_index(slot, grp) + 4]);
    }
  }
}

// ---- kmeans
constexpr int kPT = kTbeMaxTokens / 64;   // points per lane at most: lane L looks after points L, L + 64, ...
constexpr int kRB = kTbeMaxTokens / 16;   // 16-point row blocks of the distance matrix at most
constexpr int kKmThreads = 1024;          // sixteen waves, four per SIMD: the staging of a tile is mostly waiting
constexpr int kRowSplit = kKmThreads / 256;   // waves that share a cluster quarter and split the row blocks
constexpr int kRBW = kRB / kRowSplit;     // row blocks per wave: wave w takes blocks kRowSplit t + w / 4
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
constexpr int kPadH = 2 * kTile + 8;   // binary16 numbers per tile row: high parts, low parts, padding (an odd multiple of 16 bytes)

struct KmScratch {
  _Float16 xs[kTbeMaxTokens][kPadH];   // one tile: 64 channels of every point, each as high + low binary16 part ...
  _Float16 cs[kTbeMaxKeep][kPadH];     // ... and of every centroid
  float xx[kTbeMaxTokens];             // squared norms of the points
  float cc[kTbeMaxKeep];               // squared norms of the centroids
  int cnt[kTbeMaxKeep];                // members of every cluster,
  int start[kTbeMaxKeep];              // where its members begin in order[],
  int order[kTbeMaxTokens];            // and the points cluster by cluster, in index order inside a cluster
};

// four channels into a tile row: x = hi + lo with hi = binary16(x), lo = binary16(x - hi), 22 significant bits
__device__ inline void store_split(_Float16* row, int c, float4 v) {
  const f16x4 hi = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
  const f16x4 lo = {(_Float16)(v.x - (float)hi[0]), (_Float16)(v.y - (float)hi[1]), (_Float16)(v.z - (float)hi[2]),
                    (_Float16)(v.w - (float)hi[3])};
  *(f16x4*)&row[c] = hi;
  *(f16x4*)&row[kTile + c] = lo;
}

// eight channels of a tile row back as binary32 (hi + lo)
__device__ inline void load_joined(const _Float16* row, int c, float* out) {
  const f16x8 hi = *(const f16x8*)&row[c], lo = *(const f16x8*)&row[kTile + c];
#pragma unroll
  for (int e = 0; e < 8; ++e) out[e] = (float)hi[e] + (float)lo[e];
}

// One pass over the channels, 64 at a time through LDS (the loads of the next tile are in flight
// while the current one is worked on):
//   update  the centroid of every cluster that has members moves to their mean (sum from zero in
//           index order, times 1 / count), tile by tile, from the point tile that is in LDS anyway;
//           the moved rows go back to cent[] so that a cluster that later loses all its members
//           still finds its centroid there
//   dots    dot[p][j] of all points with all centroids on the matrix cores.  The binary32 matrix
//           instruction is slow (a sixteenth of the binary16 rate), and binary16 alone cannot hold a
//           dequantised key, so every number enters as the sum of two binary16 parts and a product
//           is taken as hi.hi + hi.lo + lo.hi on v_mfma_f32_16x16x32_f16 (exact products, binary32
//           sums; what is dropped is of the order of 2^-22 of |x||c|).  Wave w owns clusters
//           16 (w % 4) .. + 15 and every fourth row block of 16 points (blocks 4 t + w / 4); after
//           the call lane l holds, in acc[t][i], the product of point 16 (4 t + w / 4) + 4 (l / 16) + i
//           with cluster 16 (w % 4) + l % 16
//   norms   squared norms of the centroids, and of the points when first is set (they do not move)
__device__ inline void pass_over_channels(const float* __restrict__ x, float* __restrict__ cent, int n, int k, int dim, bool first,
                                          bool update, KmScratch& sm, f32x4 (&acc)[kRBW]) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int rbs = (n + 15) >> 4;
  constexpr int kC4 = kTile / 4;                          // float4 per tile row
  const int xq = (rbs * 16 * kC4 + kKmThreads - 1) / kKmThreads;   // float4 loads per thread for the points' tile
  constexpr int kXQ = kTbeMaxTokens * kC4 / kKmThreads;
  constexpr int kCQ = kTbeMaxKeep * kC4 / kKmThreads;
  const int cb = wave & 3, half = wave >> 2;
#pragma unroll
  for (int t = 0; t < kRBW; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float nx = 0.f, nc = 0.f;
  float4 px[kXQ], pc[kCQ];
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  auto fetch = [&](int d0) {
#pragma unroll
    for (int q = 0; q < kXQ; ++q)
      if (q < xq) {
        const int idx = tid + kKmThreads * q, row = idx / kC4, c4 = idx % kC4;
        px[q] = row < n ? *(const float4*)&x[(int64_t)row * dim + d0 + 4 * c4] : zero4;
      }
#pragma unroll
    for (int q = 0; q < kCQ; ++q) {
      const int idx = tid + kKmThreads * q, row = idx / kC4, c4 = idx % kC4;
      pc[q] = row < k ? *(const float4*)&cent[(int64_t)row * dim + d0 + 4 * c4] : zero4;
    }
  };
  // the update: thread (cluster tid / 8, part tid % 8) owns 8 channels of the cluster's row
  const int uj = tid >> 3, upart = tid & 7;
  const int um = update && uj < k ? sm.cnt[uj] : 0, ust = uj < k ? sm.start[uj] : 0;
  const float uinv = um > 0 ? 1.0f / (float)um : 0.f;
  fetch(0);
  for (int d0 = 0; d0 < dim; d0 += kTile) {
    __syncthreads();   // the previous tile has been used
#pragma unroll
    for (int q = 0; q < kXQ; ++q)
      if (q < xq) {
        const int idx = tid + kKmThreads * q;
        store_split(sm.xs[idx / kC4], 4 * (idx % kC4), px[q]);
      }
#pragma unroll
    for (int q = 0; q < kCQ; ++q) {
      const int idx = tid + kKmThreads * q;
      store_split(sm.cs[idx / kC4], 4 * (idx % kC4), pc[q]);
    }
    __syncthreads();
    if (d0 + kTile < dim) fetch(d0 + kTile);
    if (update) {
      if (um > 0) {
        float sum[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) sum[e] = 0.f;
        for (int i = 0; i < um; ++i) {
          float t[8];
          load_joined(sm.xs[sm.order[ust + i]], 8 * upart, t);
#pragma unroll
          for (int e = 0; e < 8; ++e) sum[e] += t[e];
        }
        const float4 m0 = make_float4(sum[0] * uinv, sum[1] * uinv, sum[2] * uinv, sum[3] * uinv);
        const float4 m1 = make_float4(sum[4] * uinv, sum[5] * uinv, sum[6] * uinv, sum[7] * uinv);
        store_split(sm.cs[uj], 8 * upart, m0);
        store_split(sm.cs[uj], 8 * upart + 4, m1);
        *(float4*)&cent[(int64_t)uj * dim + d0 + 8 * upart] = m0;
        *(float4*)&cent[(int64_t)uj * dim + d0 + 8 * upart + 4] = m1;
      }
      __syncthreads();
    }
    if (first && tid < n) {
#pragma unroll
      for (int c8 = 0; c8 < kTile / 8; ++c8) {
        float t[8];
        load_joined(sm.xs[tid], 8 * c8, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) nx = fmaf(t[e], t[e], nx);
      }
    }
    if (uj < k) {   // the eight channels of thread (cluster, part), as the products will see them
      float t[8];
      load_joined(sm.cs[uj], 8 * upart, t);
#pragma unroll
      for (int e = 0; e < 8; ++e) nc = fmaf(t[e], t[e], nc);
    }
    if (16 * cb < k) {
#pragma unroll
      for (int ks = 0; ks < kTile / 32; ++ks) {
        // lane (r, g) holds channels 32 ks + 8 g .. + 7 of its row, on both sides
        const f16x8 bh = *(const f16x8*)&sm.cs[16 * cb + r][32 * ks + 8 * g];
        const f16x8 bl = *(const f16x8*)&sm.cs[16 * cb + r][kTile + 32 * ks + 8 * g];
#pragma unroll
        for (int t = 0; t < kRBW; ++t)
          if (kRowSplit * t + half < rbs) {
            const _Float16* row = sm.xs[16 * (kRowSplit * t + half) + r];
            const f16x8 ah = *(const f16x8*)&row[32 * ks + 8 * g];
            const f16x8 al = *(const f16x8*)&row[kTile + 32 * ks + 8 * g];
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bl, acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, bh, acc[t], 0, 0, 0);
          }
      }
    }
  }
  __syncthreads();
  if (first && tid < n) sm.xx[tid] = nx;
  // the eight parts of a cluster's norm sit in eight neighbouring lanes
  nc += __shfl_xor(nc, 1, 64);
  nc += __shfl_xor(nc, 2, 64);
  nc += __shfl_xor(nc, 4, 64);
  if (upart == 0 && uj < kTbeMaxKeep) sm.cc[uj] = uj < k ? nc : 0.f;
  __syncthreads();
}

__global__ __launch_bounds__(kKmThreads) void tbe_kmeans_kernel(thinkv_view v, TbeArgs a) {
  const thinkv_config& c = v.cfg;
  const int seg = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = a.seg_offset[seg], hi = a.seg_offset[seg + 1];
  const int n = hi - lo, want = a.seg_keep[seg];
  if (n <= 0) return;
  if (n > kTbeMaxTokens || want > kTbeMaxKeep || want < 1 || lo < 0 || hi > a.n_tok) {
    // outside what this kernel covers: nothing is evicted, and the caller is told
    if (tid == 0) atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEGMENT);
    for (int i = tid; i < n && lo >= 0 && lo + i < a.n_tok; i += kKmThreads) {
      a.ev_handle[lo + i] = -1;
      a.assign[lo + i] = -1;
    }
    return;
  }
  if (want >= n) {
    for (int i = tid; i < n; i += kKmThreads) {
      a.ev_handle[lo + i] = -1;
      a.assign[lo + i] = -1;
    }
    return;
  }
  const int k = want, dim = a.dim, pt = (n + 63) / 64, rbs = (n + 15) >> 4;
  const float* x = a.x + (int64_t)lo * dim;
  float* cent = a.cent + (int64_t)seg * kTbeMaxKeep * dim;
  __shared__ __attribute__((aligned(16))) KmScratch sm;
  __shared__ float s_bd[4][kTbeMaxTokens];   // per cluster quarter: best distance of every point ...
  __shared__ int s_bj[4][kTbeMaxTokens];     // ... and the cluster it belongs to
  __shared__ int s_assign[kTbeMaxTokens];
  __shared__ int s_cnt[kTbeMaxKeep], s_start[kTbeMaxKeep];   // survivors: members and lowest index of every cluster
  __shared__ unsigned long long s_best[kTbeMaxKeep];
  // initial centroids: evenly spaced points
  for (int idx = tid; idx < k * dim; idx += kKmThreads) {
    const int j = idx / dim, d = idx % dim;
    cent[idx] = x[(int64_t)((j * n) / k) * dim + d];
  }
  __syncthreads();
  f32x4 acc[kRBW];
  int mine[kPT];
#pragma unroll
  for (int q = 0; q < kPT; ++q) mine[q] = -1;
  const int r = lane & 15, g = lane >> 4, cb = wave & 3, half = wave >> 2, my_cl = 16 * cb + r;
  // nearest cluster of every point: |c|^2 - 2 x.c decides (|x|^2 is common to a point's candidates);
  // best of the sixteen clusters of this wave by exchanges among the sixteen lanes that hold a point's
  // row, then best of the four cluster quarters (ties go to the lowest cluster)
  auto assign = [&](int* out) {
    const float ccj = my_cl < k ? sm.cc[my_cl] : 0.f;
#pragma unroll
    for (int t = 0; t < kRBW; ++t)
      if (kRowSplit * t + half < rbs) {
        const int rb = kRowSplit * t + half;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float bd = my_cl < k ? fmaf(-2.f, acc[t][i], ccj) : INFINITY;
          int bj = my_cl;
#pragma unroll
          for (int d = 1; d < 16; d <<= 1) {
            const float od = __shfl_xor(bd, d, 64);
            const int oj = __shfl_xor(bj, d, 64);
            if (od < bd || (od == bd && oj < bj)) {
              bd = od;
              bj = oj;
            }
          }
          if (r == 0) {
            s_bd[cb][16 * rb + 4 * g + i] = bd;
            s_bj[cb][16 * rb + 4 * g + i] = bj;
          }
        }
      }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      const int p = lane + 64 * q;
      float bd = s_bd[0][p];
      int bj = s_bj[0][p];
#pragma unroll
      for (int w = 1; w < 4; ++w)
        if (s_bd[w][p] < bd) {
          bd = s_bd[w][p];
          bj = s_bj[w][p];
        }
      out[q] = q < pt ? bj : -1;
    }
  };
  bool converged = false;
  for (int it = 0; it < a.max_iters; ++it) {
    // centroids: the initial ones, later the means under the previous assignment; then all products
    pass_over_channels(x, cent, n, k, dim, it == 0, it > 0, sm, acc);
    int now[kPT];
    assign(now);
    int changed = 0;
#pragma unroll
    for (int q = 0; q < kPT; ++q) {
      changed |= (lane + 64 * q < n) && now[q] != mine[q];
      mine[q] = now[q];
    }
    if (!__syncthreads_or(changed)) {
      converged = true;   // the products at hand are those with the final centroids
      break;
    }
    // ---- members of every cluster in index order, for the next pass
    if (tid < kTbeMaxKeep) sm.cnt[tid] = 0;
    if (wave == 0) {
#pragma unroll
      for (int q = 0; q < kPT; ++q)
        if (lane + 64 * q < n) s_assign[lane + 64 * q] = mine[q];
    }
    __syncthreads();
    int rank = 0;
    if (tid < n) {
      const int cl = s_assign[tid];
      for (int i = 0; i < tid; ++i) rank += s_assign[i] == cl;
      atomicAdd(&sm.cnt[cl], 1);
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int j = 0; j < k; ++j) {
        sm.start[j] = run;
        run += sm.cnt[j];
      }
    }
    __syncthreads();
    if (tid < n) sm.order[sm.start[s_assign[tid]] + rank] = tid;
    __syncthreads();
  }
  // ---- survivors: nearest member of every cluster under the final centroids
  if (!converged) pass_over_channels(x, cent, n, k, dim, false, true, sm, acc);
  if (tid < kTbeMaxKeep) {
    s_cnt[tid] = 0;
    s_start[tid] = kTbeMaxTokens;   // here: lowest index among the cluster's members
    s_best[tid] = ~0ull;
  }
  if (wave == 0) {
#pragma unroll
    for (int q = 0; q < kPT; ++q)
      if (lane + 64 * q < n) s_assign[lane + 64 * q] = mine[q];
  }
  __syncthreads();
  if (my_cl < k) {
    const float ccj = sm.cc[my_cl];
#pragma unroll
    for (int t = 0; t < kRBW; ++t)
      if (kRowSplit * t + half < rbs) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int p = 16 * (kRowSplit * t + half) + 4 * g + i;
          if (p < n && s_assign[p] == my_cl) {   // this lane holds the point's product with its own cluster
            const float own = fmaxf(fmaf(-2.f, acc[t][i], sm.xx[p]) + ccj, 0.f);
            atomicAdd(&s_cnt[my_cl], 1);
            atomicMin(&s_start[my_cl], p);
            // distances are not negative, so their bit patterns order like the numbers; the index breaks ties
            atomicMin(&s_best[my_cl], ((unsigned long long)__builtin_bit_cast(uint32_t, own) << 32) | (unsigned)p);
          }
        }
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
        a.assign[lo + p] = mine[q];
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
  a.assign = (int32_t*)(a.cent + (size_t)n_seg * kTbeMaxKeep * a.dim);
  a.layer = layer;
  a.n_seg = n_seg;
  a.n_tok = n_tok;
  a.max_iters = max_iters;
  hipLaunchKernelGGL(tbe_gather_kernel, dim3((n_tok + kGatherTokens - 1) / kGatherTokens), dim3(256), 0, st, v, a);
  hipLaunchKernelGGL(tbe_kmeans_kernel, dim3(n_seg), dim3(kKmThreads), 0, st, v, a);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

// ---------------------------------------------------------------------------------------------
// The plan: which segments of which sequences are cut, and to how many tokens (Sec. 4.3: Case 1,
// every preceding segment goes down one retention level when a transition segment has ended;
// Case 2, while the sequence holds more live tokens than the budget, the oldest segment of the
// least important type that can still shrink goes down one level).  A segment is cut at most
// once per call (one K-means per segment and call).  Its level follows from the number n of times
// it has been selected before (a column the caller keeps): it keeps min(live, R_n) tokens, and a
// selection that removes nothing only advances n (problem statement "Thought-Adaptive Eviction");
// or, as an option for callers without that column, from its live size: it is cut to the largest
// retention value below that size.  The open (last) segment is never touched.
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
  int32_t* seg_count;   // [max_seqs][max_segs] selections so far (rule THINKV_TBE_BY_COUNT)
  int rule;
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

// calls f(segment, position, handle) for every live token of the sequence; every thread takes pages.
// The walk is a chain of dependent loads (page count -> live mask and page id -> the page's sixteen
// positions) and little else, so the chains of the three page lists run side by side.
template <typename F>
__device__ inline void for_live_tokens(const thinkv_view& v, int seq, int layer, const int* s_start, int ns, F f) {
  const thinkv_config& c = v.cfg;
  int np[3], most = 0;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    np[k] = v.n_pages[npages_index(c, seq, layer, k)];
    most = np[k] > most ? np[k] : most;
  }
  for (int pi = threadIdx.x; pi < most; pi += blockDim.x) {
    uint32_t m[3];
    int pid[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const bool in = pi < np[k];
      const int64_t at = table_base(c, seq, layer, k) + (in ? pi : 0);
      m[k] = in ? v.slot_mask[at] & 0xFFFFu : 0u;
      pid[k] = in ? v.block_table[at] : 0;
    }
    int pos[3][kPage];
#pragma unroll
    for (int k = 0; k < 3; ++k)
      if (m[k]) {
        const int4* sp = (const int4*)(v.slot_pos[k] + (int64_t)pid[k] * kPage);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int4 w = sp[q];
          pos[k][4 * q] = w.x; pos[k][4 * q + 1] = w.y; pos[k][4 * q + 2] = w.z; pos[k][4 * q + 3] = w.w;
        }
      }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      if (!m[k]) continue;
      // neighbours in a page are mostly neighbours in the sequence: the segment of the slot before is
      // tried first (two LDS reads), the binary search (eleven dependent ones) only when that fails
      int sg = -1, lo_pos = 0, hi_pos = -1;   // [lo_pos, hi_pos): positions of segment sg
#pragma unroll
      for (int slot = 0; slot < kPage; ++slot) {
        if (!(m[k] >> slot & 1)) continue;
        const int p = pos[k][slot];
        if (p < lo_pos || p >= hi_pos) {
          sg = segment_of(s_start, ns, p);
          lo_pos = sg >= 0 ? s_start[sg] : 0;
          hi_pos = sg >= 0 ? (sg + 1 < ns ? s_start[sg + 1] : 0x7fffffff) : -1;
        }
        if (sg >= 0) f(sg, p, THINKV_HANDLE(k, pi, slot));
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
  __shared__ uint8_t s_lvl[kMaxSegs];   // selections so far, capped at the number of levels
  const bool by_count = a.rule == THINKV_TBE_BY_COUNT;
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
  int32_t* sel = by_count ? a.seg_count + (int64_t)seq * a.max_segs : nullptr;
  for (int i = tid; i < ns; i += kPlanThreads) {
    s_start[i] = starts[i];
    s_type[i] = types[i];
    s_cnt[i] = 0;
    const int n = by_count ? sel[i] : 0;
    s_lvl[i] = (uint8_t)(n < 0 ? 0 : (n > 5 ? 5 : n));
  }
  __syncthreads();
  for_live_tokens(v, seq, a.layer, s_start, ns, [&](int sg, int, int) { atomicAdd(&s_cnt[sg], 1); });
  __syncthreads();
  int32_t* o_seg = a.st_seg + (int64_t)b * a.max_cuts;
  int32_t* o_keep = a.st_keep + (int64_t)b * a.max_cuts;
  int32_t* o_cnt = a.st_cnt + (int64_t)b * a.max_cuts;
  const int last = ns - 1;
  // Case 1: every closed segment that can still shrink, in ascending order, is independent of the
  // others: all threads, with a prefix sum for the place of each cut in the list
  __shared__ int s_wave[3][kPlanThreads / 64];
  __shared__ int s_c1[4];   // cuts, tokens listed, tokens dropped, a segment too large for one workgroup was met
  if (tid < 4) s_c1[tid] = 0;
  __syncthreads();
  if (a.transition_ended && a.transition_ended[b]) {
    for (int i0 = 0; i0 < last; i0 += kPlanThreads) {
      const int i = i0 + tid, lane = tid & 63, wave = tid >> 6;
      const int cnt = i < last ? s_cnt[i] : 0;
      // what the segment keeps if it is selected now (0: it cannot be selected, or nothing would go)
      int r = 0;
      if (i < last) {
        if (by_count) {
          const int n = s_lvl[i];
          if (n < 5) {
            r = cnt < kRetention[n] ? cnt : kRetention[n];
            if (r >= cnt) {           // removes nothing: not a cut, the count moves on
              s_lvl[i] = (uint8_t)(n + 1);
              sel[i] = n + 1;
              r = 0;
            }
          }
        } else {
          r = next_level(cnt);
        }
      }
      const bool big = r && cnt > kTbeMaxTokens;
      const int flag = r && !big;
      int inc = flag;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d, 64);
        if (lane >= d) inc += o;
      }
      if (lane == 63) s_wave[0][wave] = inc;
      __syncthreads();
      int before = s_c1[0];
      for (int w = 0; w < wave; ++w) before += s_wave[0][w];
      const int at = before + inc - flag;
      const bool take = flag && at < a.max_cuts;
      if (take) {
        o_seg[at] = i;
        o_keep[at] = r;
        o_cnt[at] = cnt;
        s_cnt[i] = -r;          // negative: cut in this call, now holding r tokens
      }
      int n_take = take, listed = take ? cnt : 0, dropped = take ? cnt - r : 0;
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) {
        n_take += __shfl_xor(n_take, d, 64);
        listed += __shfl_xor(listed, d, 64);
        dropped += __shfl_xor(dropped, d, 64);
      }
      __syncthreads();   // s_wave[0] and s_c1[0] have been read
      if (lane == 0) {
        s_wave[0][wave] = n_take;
        s_wave[1][wave] = listed;
        s_wave[2][wave] = dropped;
      }
      if (big) s_c1[3] = 1;
      __syncthreads();
      if (tid == 0)
        for (int w = 0; w < kPlanThreads / 64; ++w) {
          s_c1[0] += s_wave[0][w];
          s_c1[1] += s_wave[1][w];
          s_c1[2] += s_wave[2][w];
        }
      __syncthreads();
    }
  }
  if (tid != 0) return;
  int total = v.n_live[sl_index(c, seq, a.layer)] - s_c1[2];
  int n_cuts = s_c1[0], listed = s_c1[1];
  bool oversize = s_c1[3] != 0;
  auto cut = [&](int i, int r) {
    o_seg[n_cuts] = i;
    o_keep[n_cuts] = r;
    o_cnt[n_cuts] = s_cnt[i];
    ++n_cuts;
    listed += s_cnt[i];
    total -= s_cnt[i] - r;
    s_cnt[i] = -r;          // negative: cut in this call, now holding r tokens
  };
  // Case 2.  A segment that cannot be cut now cannot be cut later in this call either (one cut per
  // segment and call), so "the oldest segment of the least important type that can still shrink",
  // asked again after every cut, is one walk over the types in order of importance and over the
  // segments of each from the oldest on.
  for (int t = 0; t < 3; ++t)
    for (int i = 0; i < last && total > a.budget && n_cuts < a.max_cuts; ++i) {
      if (s_type[i] != t || s_cnt[i] < 0) continue;
      int r = 0;
      if (by_count) {
        // selections that remove nothing follow one another at once (each advances the count)
        int n = s_lvl[i];
        while (n < 5 && r == 0) {
          const int keep = s_cnt[i] < kRetention[n] ? s_cnt[i] : kRetention[n];
          if (keep < s_cnt[i]) r = keep; else ++n;
        }
        if (n != s_lvl[i]) {
          s_lvl[i] = (uint8_t)n;
          sel[i] = n;
        }
      } else {
        r = next_level(s_cnt[i]);
      }
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
  for (int i = tid; i < n_cuts; i += kPlanThreads) {
    const int sg = a.st_seg[(int64_t)b * a.max_cuts + i];
    s_cut[sg] = i;
    // the cut is made (it fitted the lists): this was a selection of the segment
    if (a.rule == THINKV_TBE_BY_COUNT) a.seg_count[(int64_t)seq * a.max_segs + sg] += 1;
  }
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
                    const int32_t* n_segs, const uint8_t* transition_ended, int32_t* seg_count, int rule, int B, int max_segs, int budget, int max_cuts,
                    int cap_seg, int cap_tok, int32_t* tok_seq, int32_t* tok_handle, int32_t* seg_offset, int32_t* seg_keep,
                    int32_t* counts, void* workspace, hipStream_t st) {
  PlanArgs a;
  a.seq_ids = seq_ids;
  a.seg_start = seg_start;
  a.seg_type = seg_type;
  a.n_segs = n_segs;
  a.transition_ended = transition_ended;
  a.seg_count = seg_count;
  a.rule = rule;
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
