// Measurement aid: read exactly the (page, kv-head) blocks a full-attention decode call reads, and
// nothing else -- what the memory system gives for this layout when no arithmetic is in the way.
// Same split as the attention launch has: `per_head` workgroups per (query, kv-head), workgroup j
// of a head taking every per_head-th page of each type's list, a wave every fourth of those; a
// block is read with 16-byte non-temporal loads, lane after lane, and folded into a checksum.
#include "common.h"

namespace thinkv {

typedef uint32_t u32x4p __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_stream_kernel(thinkv_view v, int layer, const int32_t* seq_ids, int B, int per_head,
                                                            uint32_t* checksum) {
  const thinkv_config& c = v.cfg;
  const int H = c.n_kv_heads, heads = H * B;
  const int j = blockIdx.x / heads, rest = blockIdx.x % heads;
  const int hkv = rest % H, b = rest / H;
  const int seq = seq_ids[b];
  if (seq < 0 || seq >= c.max_seqs) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t acc = 0;
  for (int k = 0; k < 3; ++k) {
    const int np = v.n_pages[npages_index(c, seq, layer, k)];
    const int bb = block_geom(c.bits_of_class[k], c.head_dim, c.format).block_bytes;
    const int32_t* tab = v.block_table + table_base(c, seq, layer, k);
    const int stride = 4 * per_head;
    // the wave's pages are first + i * stride; their ids are fetched 64 at a time (lane i: page i of the run), then
    // four blocks are kept in flight
    for (int first = j + per_head * wave; first < np; first += 64 * stride) {
      const int mine = first + lane * stride;
      const int pid_l = mine < np ? tab[mine] : 0;
      int cnt = (np - first + stride - 1) / stride;
      cnt = cnt > 64 ? 64 : cnt;
      for (int i = 0; i < cnt; i += 4) {
        const uint8_t* blk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int pid = __builtin_amdgcn_readlane(pid_l, i + u < cnt ? i + u : i);
          blk[u] = v.arena[k] + ((int64_t)pid * H + hkv) * bb;
        }
        // every load of the four blocks is requested before the first word is looked at (a block is at most 4.5 KB: five rounds)
        u32x4p w[4][5];
#pragma unroll
        for (int t = 0; t < 5; ++t)
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int off = 16 * lane + 1024 * t;
            w[u][t] = off < bb ? __builtin_nontemporal_load((const u32x4p*)(blk[u] + off)) : u32x4p{0u, 0u, 0u, 0u};
          }
#pragma unroll
        for (int t = 0; t < 5; ++t)
#pragma unroll
          for (int u = 0; u < 4; ++u) acc ^= i + u < cnt ? (w[u][t].x ^ w[u][t].y ^ w[u][t].z ^ w[u][t].w) : 0u;
      }
    }
  }
  if (acc == 0x9E3779B9u) atomicXor(checksum, acc);   // practically never: keeps the loads alive
}

int launch_probe_stream(const thinkv_view& v, int layer, const int32_t* seq_ids, int B, int per_head, uint32_t* checksum, hipStream_t st) {
  hipLaunchKernelGGL(probe_stream_kernel, dim3((unsigned)(per_head * v.cfg.n_kv_heads * B)), dim3(256), 0, st, v, layer, seq_ids, B, per_head,
                     checksum);
  return hipGetLastError() == hipSuccess ? THINKV_OK : THINKV_E_HIP;
}

}  // namespace thinkv
