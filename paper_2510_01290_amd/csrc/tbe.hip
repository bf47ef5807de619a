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
// kmeans: one workgroup of 256 threads per segment, thread i owns point i (segments hold at
// most 256 live tokens, the schedule keeps at most 64): the N x K distances are accumulated
// tile by tile (32 channels of all points and all centroids staged in LDS, 64 accumulators per
// thread), the update sums the members of a cluster in index order (fixed summation order, so
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
// squared distances of point `me` (this thread's) to all centroids, accumulated over the channels
__device__ inline void distances(const float* __restrict__ x, const float* __restrict__ cent, int n, int k, int dim, float (*xs)[kPad],
                                 float (*cs)[kPad], float* acc /*[kTbeMaxKeep]*/) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < kTbeMaxKeep; ++j) acc[j] = 0.f;
  for (int d0 = 0; d0 < dim; d0 += kTile) {
    __syncthreads();
    for (int idx = tid; idx < kTbeMaxTokens * kTile; idx += 256) {
      const int r = idx / kTile, cc = idx % kTile;
      xs[r][cc] = r < n ? x[(int64_t)r * dim + d0 + cc] : 0.f;
    }
    for (int idx = tid; idx < kTbeMaxKeep * kTile; idx += 256) {
      const int r = idx / kTile, cc = idx % kTile;
      cs[r][cc] = r < k ? cent[(int64_t)r * dim + d0 + cc] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int c4 = 0; c4 < kTile / 4; ++c4) {
      const float4 xv = *(const float4*)&xs[tid][4 * c4];
#pragma unroll
      for (int j = 0; j < kTbeMaxKeep; ++j) {
        const float4 cv = *(const float4*)&cs[j][4 * c4];
        const float e0 = xv.x - cv.x, e1 = xv.y - cv.y, e2 = xv.z - cv.z, e3 = xv.w - cv.w;
        acc[j] = fmaf(e3, e3, fmaf(e2, e2, fmaf(e1, e1, fmaf(e0, e0, acc[j]))));
      }
    }
  }
}

__global__ __launch_bounds__(256) void tbe_kmeans_kernel(thinkv_view v, TbeArgs a) {
  const thinkv_config& c = v.cfg;
  const int seg = blockIdx.x, tid = threadIdx.x;
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
  const int k = want, dim = a.dim;
  const float* x = a.x + (int64_t)lo * dim;
  float* cent = a.cent + (int64_t)seg * kTbeMaxKeep * dim;
  __shared__ __attribute__((aligned(16))) float xs[kTbeMaxTokens][kPad];
  __shared__ __attribute__((aligned(16))) float cs[kTbeMaxKeep][kPad];
  __shared__ int s_assign[kTbeMaxTokens], s_order[kTbeMaxTokens];
  __shared__ int s_cnt[kTbeMaxKeep], s_start[kTbeMaxKeep];
  __shared__ unsigned long long s_best[kTbeMaxKeep];
  // initial centroids: evenly spaced points
  for (int idx = tid; idx < k * dim; idx += 256) {
    const int j = idx / dim, d = idx % dim;
    cent[idx] = x[(int64_t)((j * n) / k) * dim + d];
  }
  float acc[kTbeMaxKeep];
  int mine = -1;
  for (int it = 0; it < a.max_iters; ++it) {
    __threadfence_block();
    distances(x, cent, n, k, dim, xs, cs, acc);
    int best = 0;
    float bd = acc[0];
#pragma unroll
    for (int j = 1; j < kTbeMaxKeep; ++j)
      if (j < k && acc[j] < bd) {
        bd = acc[j];
        best = j;
      }
    const int changed = tid < n && best != mine;
    mine = best;
    if (!__syncthreads_or(changed)) break;
    // ---- update: members of every cluster in index order
    if (tid < kTbeMaxKeep) s_cnt[tid] = 0;
    if (tid < n) s_assign[tid] = mine;
    __syncthreads();
    int rank = 0;
    if (tid < n) {
      for (int i = 0; i < tid; ++i) rank += s_assign[i] == mine;
      atomicAdd(&s_cnt[mine], 1);
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
    if (tid < n) s_order[s_start[mine] + rank] = tid;
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
  __threadfence_block();
  distances(x, cent, n, k, dim, xs, cs, acc);
  if (tid < kTbeMaxKeep) {
    s_cnt[tid] = 0;
    s_start[tid] = kTbeMaxTokens;   // here: lowest index among the cluster's members
    s_best[tid] = ~0ull;
  }
  __syncthreads();
  float own = 0.f;
#pragma unroll
  for (int j = 0; j < kTbeMaxKeep; ++j)
    if (j == mine) own = acc[j];
  if (tid < n) {
    atomicAdd(&s_cnt[mine], 1);
    atomicMin(&s_start[mine], tid);
    // distances are not negative, so their bit patterns order like the numbers; the index breaks ties
    atomicMin(&s_best[mine], ((unsigned long long)__builtin_bit_cast(uint32_t, own) << 32) | (unsigned)tid);
  }
  __syncthreads();
  if (tid < n) {
    // two members are equally near their mean whatever the rounding says: the earlier one stays
    const bool keep = s_cnt[mine] <= 2 ? tid == s_start[mine] : (int)(s_best[mine] & 0xFFFFFFFFull) == tid;
    a.ev_handle[lo + tid] = keep ? -1 : a.tok_handle[lo + tid];
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

}  // namespace thinkv
