// Attention-sparsity statistic of a decode step (Sec. 4.1 of the paper: the thought type of a
// step is read off how sparse its normalised attention scores are; appendix "Grouped-Query
// Attention": the scaled scores of the G query heads of a group are max-pooled, the pooled row
// is renormalised by a softmax over the keys, an entry is negligible when it lies below 1 % of
// the row's maximum, and the fractions of negligible entries are averaged over the groups).
//
// The scores are those the attention kernel computes anyway, so the statistic rides on a decode
// call: the STAT instantiation of the attention kernel stores the pooled score of every slot it
// visits (16 floats per page, log2 domain), after a fill kernel has set the buffer to -inf (dead
// and invisible slots, pages skipped because nothing in them is live), and two small kernels take
// the maximum of each (query, kv-head) row, count, and average over the kv-heads.  w_j < 0.01 max w  <=>  pooled_j <
// max pooled - log2(100) in the log2 domain, so no softmax is ever formed.
#include "decode_mfma_kernel.h"

namespace thinkv {

__global__ __launch_bounds__(256) void stat_fill_kernel(float4* p, int64_t n4) {
  const float ninf = -INFINITY;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = make_float4(ninf, ninf, ninf, ninf);
}

// One workgroup per (query, kv-head): the row maximum, then the counts of visible and of
// negligible entries; the row's fraction negligible / visible (0 where nothing is visible) goes
// to frac[b][kv-head].  Rows are read 16 bytes a lane; the second pass finds them in L2.
__global__ __launch_bounds__(1024) void stat_count_kernel(thinkv_view v, DecodeArgs a, float* frac) {
  const thinkv_config& c = v.cfg;
  const int hkv = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ float s_max[16];
  __shared__ int s_cnt[2][16];
  const int seq = a.seq_ids[b];
  int64_t n = 0;
  if (seq >= 0 && seq < c.max_seqs)
    for (int k = 0; k < 3; ++k) n += v.n_pages[npages_index(c, seq, a.layer, k)];
  n *= kPage;
  if (n > a.stat_stride) n = a.stat_stride;   // the host's bound on the context was too small: count what was kept
  const float4* row = (const float4*)(a.stat + ((int64_t)b * c.n_kv_heads + hkv) * a.stat_stride);
  const int n4 = (int)(n / 4);                // whole pages: a multiple of four
  float m = -INFINITY;
  for (int i = tid; i < n4; i += 1024) {
    const float4 x = row[i];
    m = fmaxf(fmaxf(m, fmaxf(x.x, x.y)), fmaxf(x.z, x.w));
  }
  for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
  if (lane == 0) s_max[wave] = m;
  __syncthreads();
  m = s_max[0];
  for (int w = 1; w < 16; ++w) m = fmaxf(m, s_max[w]);
  const float cut = m - 6.643856189774724f;   // log2(100)
  int vis = 0, neg = 0;
  for (int i = tid; i < n4; i += 1024) {
    const float4 x = row[i];
    vis += (x.x > -INFINITY) + (x.y > -INFINITY) + (x.z > -INFINITY) + (x.w > -INFINITY);
    neg += (x.x > -INFINITY && x.x < cut) + (x.y > -INFINITY && x.y < cut) + (x.z > -INFINITY && x.z < cut) +
           (x.w > -INFINITY && x.w < cut);
  }
  for (int d = 32; d >= 1; d >>= 1) {
    vis += __shfl_xor(vis, d, 64);
    neg += __shfl_xor(neg, d, 64);
  }
  if (lane == 0) {
    s_cnt[0][wave] = vis;
    s_cnt[1][wave] = neg;
  }
  __syncthreads();
  if (tid == 0) {
    int tv = 0, tn = 0;
    for (int w = 0; w < 16; ++w) {
      tv += s_cnt[0][w];
      tn += s_cnt[1][w];
    }
    frac[(int64_t)b * c.n_kv_heads + hkv] = tv > 0 ? (float)tn / (float)tv : 0.f;
  }
}

// sparsity[b] = mean over kv-heads, summed in head order (the same bits on every run)
__global__ __launch_bounds__(256) void stat_mean_kernel(const float* frac, float* sparsity, int B, int Hkv) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  float total = 0.f;
  for (int h = 0; h < Hkv; ++h) total += frac[(int64_t)b * Hkv + h];
  sparsity[b] = total / (float)Hkv;
}

int launch_stat_fill(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  const int64_t n4 = (int64_t)a.B * v.cfg.n_kv_heads * a.stat_stride / 4;
  int64_t blocks = (n4 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(stat_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (float4*)a.stat, n4);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

int launch_decode_mfma_stat(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) { return launch_decode_mfma_t<true>(v, a, st); }

int launch_stat_count(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) {
  // the per-row fractions live behind the pooled scores
  float* frac = a.stat + (int64_t)a.B * v.cfg.n_kv_heads * a.stat_stride;
  hipLaunchKernelGGL(stat_count_kernel, dim3(v.cfg.n_kv_heads, a.B), dim3(1024), 0, st, v, a, frac);
  hipLaunchKernelGGL(stat_mean_kernel, dim3((a.B + 255) / 256), dim3(256), 0, st, frac, a.sparsity, a.B, v.cfg.n_kv_heads);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
