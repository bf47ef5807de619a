// Soft eviction and view initialisation.
#include "common.h"

namespace thinkv {

// One thread per handle.
__global__ __launch_bounds__(256) void evict_kernel(thinkv_view v, int layer, const int32_t* __restrict__ ev_seq,
                                                    const int32_t* __restrict__ ev_handle, int n_ev) {
  const thinkv_config& c = v.cfg;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_ev) return;
  const int s = ev_seq[i];
  if (s < 0 || s >= c.max_seqs) {
    atomicOr(&v.dev_status[c.max_seqs * c.n_layers], THINKV_ST_BAD_SEQ);
    return;
  }
  evict_one(v, layer, s, ev_handle[i]);
}

__global__ __launch_bounds__(256) void init_kernel(thinkv_view v) {
  const thinkv_config& c = v.cfg;
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int k = 0; k < 3; ++k) {
    const int64_t n = v.arena_pages[k];
    for (int64_t i = tid; i < n; i += stride) {
      v.free_stack[k][i] = (int32_t)(n - 1 - i);
      v.page_filled[k][i] = 0;
      v.page_pos_max[k][i] = -1;
    }
    for (int64_t i = tid; i < n * kPage; i += stride) v.slot_pos[k][i] = -1;
    if (tid == 0) v.free_top[k] = (int32_t)n;
  }
  const int64_t nt = (int64_t)c.max_seqs * c.n_layers * 3 * c.max_pages;
  for (int64_t i = tid; i < nt; i += stride) {
    v.block_table[i] = -1;
    v.slot_mask[i] = 0;
  }
  const int64_t nsl = (int64_t)c.max_seqs * c.n_layers;
  for (int64_t i = tid; i < nsl * 3; i += stride) v.n_pages[i] = 0;
  for (int64_t i = tid; i < nsl; i += stride) v.n_live[i] = 0;
  for (int64_t i = tid; i < nsl + 1; i += stride) v.dev_status[i] = 0;
  for (int64_t i = tid; i < c.max_seqs; i += stride) v.append_counters[i] = 0;
  for (int64_t i = tid; i < nsl * c.n_kv_heads * 4; i += stride) v.work_counters[i] = 0;
}

int launch_evict(const thinkv_view& v, int layer, const int32_t* ev_seq, const int32_t* ev_handle, int n_ev, hipStream_t st) {
  if (n_ev == 0) return THINKV_OK;
  hipLaunchKernelGGL(evict_kernel, dim3((n_ev + 255) / 256), dim3(256), 0, st, v, layer, ev_seq, ev_handle, n_ev);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

// Zero-fill of an arena in 16-byte stores (page sizes are multiples of 16 bytes).  A page can
// hold slots that were never written; attention reads them and discards them by their live
// bit, which is only safe if their scales and zero-points are finite numbers.
__global__ __launch_bounds__(256) void arena_clear_kernel(uint4* p, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = uint4{0u, 0u, 0u, 0u};
}

int launch_init(const thinkv_view& v, hipStream_t st) {
  hipLaunchKernelGGL(init_kernel, dim3(1024), dim3(256), 0, st, v);
  for (int k = 0; k < 3; ++k) {
    const int64_t n16 = v.arena_pages[k] * (int64_t)v.cfg.n_kv_heads * block_geom(v.cfg.bits_of_class[k], v.cfg.head_dim, v.cfg.format).block_bytes / 16;
    if (n16 > 0) hipLaunchKernelGGL(arena_clear_kernel, dim3(2048), dim3(256), 0, st, (uint4*)v.arena[k], n16);
  }
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
