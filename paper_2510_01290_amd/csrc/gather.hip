// What in-place slot reuse avoids (Sec. 5.1 of the paper, "The Cost of Gather-Based Compaction"): a cache kept
// contiguous has to be compacted after every eviction, the surviving rows gathered into a dense buffer.  This is
// that gather, for the comparison bench.py --contrast makes: dst[i] = src[rows[i]] over rows of row_bytes bytes
// (a multiple of 16: one token's K or V of all kv-heads in a 16-bit cache is 2 * n_kv_heads * head_dim bytes).
// A thread moves 16 bytes at a time, four of them in flight, with streaming loads and stores; consecutive threads
// take consecutive 16-byte pieces of a row, so both sides are coalesced row by row.
#include "common.h"

namespace thinkv {

typedef uint32_t u32x4g __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void gather_rows_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, const int32_t* __restrict__ rows,
                                                          int64_t n_rows, int pieces) {   // pieces = row_bytes / 16
  const int64_t total = n_rows * pieces;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i0 = (int64_t)blockIdx.x * 256 + threadIdx.x; i0 < total; i0 += 4 * stride) {
    u32x4g w[4];
    int64_t at[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      at[u] = i0 + u * stride;
      if (at[u] < total) {
        const int64_t r = at[u] / pieces;
        const int p = (int)(at[u] - r * pieces);
        w[u] = __builtin_nontemporal_load((const u32x4g*)(src + ((int64_t)rows[r] * pieces + p) * 16));
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (at[u] < total) __builtin_nontemporal_store(w[u], (u32x4g*)(dst + at[u] * 16));
  }
}

int launch_gather_rows(const void* src, void* dst, const int32_t* rows, int64_t n_rows, int row_bytes, int n_wg, hipStream_t st) {
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)n_wg), dim3(256), 0, st, (const uint8_t*)src, (uint8_t*)dst, rows, n_rows, row_bytes / 16);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
